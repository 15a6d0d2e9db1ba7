// Flash-style attention for the local heads of one TMP rank (gfx950, bf16 MFMA, fp32 softmax).
//
// Work decomposition.  A workgroup owns 32 rows of one (sequence, head): 32 queries (forward, dQ) or 32 keys
// (dK/dV).  Its four waves split the reduction range -- the 32-row key tiles a query block sees, or the 32-row
// query tiles that see a key block -- round-robin, each wave staging its own tiles in a private slice of LDS, so
// the main loops need no workgroup barrier; the four partial results meet once, through LDS, at the end.  This
// keeps every SIMD busy on a workload that has few (query, head) rows per sub-batch and shortens the longest
// causal row of work fourfold.
//
// Forward and dQ compute the TRANSPOSED score tile S^T = K*Q^T with v_mfma_f32_32x32x16_bf16, so that a lane owns
// one query (accumulator column l%32) and 16 keys of the tile: the online softmax is lane-local except for one
// exchange between the two lane halves, and the exponentials are already in B-operand position for
// O^T = V^T * P^T (the k index of that product is permuted the same way for both operands: rows 4*(l/32)+{0..3}
// and +8 of each 16-key step; the V^T operand comes from the LDS transpose read ds_read_b64_tr_b16).
// dK/dV keeps S = Q*K^T un-transposed so a lane owns one key and P^T / dS^T are in A-operand position.
// No atomics: dQ and dK/dV are separate passes, results are deterministic.
#include <type_traits>

#include "common.h"

namespace oases {

namespace {

constexpr int NT = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const uint16_t* qkv;   // [batch*seq, ld]
  const uint16_t* out;   // [batch*seq, hp]
  const uint16_t* dout;  // [batch*seq, hp]
  uint16_t* out_w;       // forward output
  uint16_t* dqkv;        // [batch*seq, ld]
  float* lse;            // [batch, heads, seq]
  float* delta;          // [batch, heads, seq]
  int seq, heads, ld, hp;
  int seq0;    // first sequence of the row range
  int pos0;    // first position (within each sequence) of the row range
  int npos;    // positions per sequence in the row range
  int blocks;  // 32-row blocks per sequence
  int nseq;    // sequences in the row range
  float scale, scale_log2;
  // dropout on the probabilities (DROP kernels): Philox key, counter word 3 (layer | 2^31), byte threshold, 1/(1 - T/256),
  // global index of local head 0 and heads of the unsharded layer
  uint32_t dk0, dk1, dc3, dthresh;
  float dscale;
  int head0, heads_total;
};

// Dropout mask of the probabilities: the 4 x 4 block (q div 4, k div 4) of (sequence b, global head) draws one
// Philox4x32-10 output with counter (k div 4, q div 4, b * heads_total + head, layer | 2^31); element (q, k) keeps its
// value iff byte (k mod 4) of word (q mod 4) is >= the threshold.
__device__ __forceinline__ Philox4 attn_drop_block(const AttnArgs& a, uint32_t k4, uint32_t q4, uint32_t bh) {
  return philox4x32_10(k4, q4, bh, a.dc3, a.dk0, a.dk1);
}
__device__ __forceinline__ uint32_t pick_word(const Philox4& w, int j) {
  return j == 0 ? w.v[0] : j == 1 ? w.v[1] : j == 2 ? w.v[2] : w.v[3];
}

// A 32-row tile of a [*, D] bf16 slice in LDS, rows padded so that BOTH access patterns are conflict-free on 64
// banks: ds_read_b128 of 16 consecutive rows at one column (row stride = 4 resp. 12 banks mod 64) and the
// transpose read of 4 consecutive rows x 32 bytes.
template <int D>
struct AT {
  static constexpr int pad = D == 128 ? 48 : 16;
  static constexpr int row = D * 2 + pad;
  static constexpr int bytes = 32 * row;
  static constexpr int cpr = D / 8;            // 16-byte chunks per row
  static constexpr int per_lane = 32 * cpr / 64;  // chunks per lane when one wave moves the tile
};

// Workgroup id -> ((sequence, head) pair, 32-row block).  Workgroup ids go round-robin over the 8 XCDs, so pair p
// of every group of 8 pairs is given the ids congruent to p mod 8: all blocks of one (sequence, head) then run on
// one XCD and its K/V (about 1 MB) stays in that XCD's L2 instead of every L2 streaming every head.
__device__ __forceinline__ void decode_block(int wg, int pairs, int blocks, int& pair, int& blk) {
  const int per_group = 8 * blocks;
  const int gi = wg / per_group, w = wg - gi * per_group;
  const int pg = min(8, pairs - 8 * gi);
  pair = 8 * gi + w % pg;
  blk = w / pg;
}

// one wave: rows [r0, r0+32) of a [*, D] slice (row stride ld elements) -> registers; rows outside [rmin, rmax) read
// as ZERO: such rows may hold anything (rows of a sub-batch that has not been computed yet), and a masked
// probability of 0 would still turn an inf/NaN there into NaN inside the MFMA.  Tiles inside the range take the
// path without clamps and selects (uniform branch).
template <int D>
__device__ __forceinline__ void wave_load(u32x4* regs, const uint16_t* __restrict__ base, int ld, int r0, int rmin, int rmax, int lane) {
  constexpr int cpr = AT<D>::cpr, rows_per_pass = 64 / cpr;
  if (r0 >= rmin && r0 + 32 <= rmax) {
    const char* sb = reinterpret_cast<const char*>(base) + (size_t)r0 * ld * 2;
    const uint32_t voff = (uint32_t)(((lane / cpr) * ld + (lane % cpr) * 8) * 2);
#pragma unroll
    for (int i = 0; i < AT<D>::per_lane; i++)
      regs[i] = *reinterpret_cast<const u32x4*>(sb + (size_t)i * rows_per_pass * ld * 2 + voff);
  } else {
#pragma unroll
    for (int i = 0; i < AT<D>::per_lane; i++) {
      int c = lane + 64 * i;
      int row = c / cpr, cc = c % cpr;
      int r = max(min(r0 + row, rmax - 1), rmin);
      u32x4 v = *reinterpret_cast<const u32x4*>(base + (size_t)r * ld + cc * 8);
      regs[i] = (r0 + row >= rmin && r0 + row < rmax) ? v : u32x4{0u, 0u, 0u, 0u};
    }
  }
}
template <int D>
__device__ __forceinline__ void wave_store(const u32x4* regs, char* lds, int lane) {
#pragma unroll
  for (int i = 0; i < AT<D>::per_lane; i++) {
    int c = lane + 64 * i;
    int row = c / AT<D>::cpr, cc = c % AT<D>::cpr;
    *reinterpret_cast<u32x4*>(lds + row * AT<D>::row + (cc << 4)) = regs[i];
  }
}
// operand fragment (32 tile rows x 16 contraction), contraction along D (16-wide step ks)
template <int D>
__device__ __forceinline__ bf16x8 kc_frag(const char* lds, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(lds + (lane & 31) * AT<D>::row + ((ks * 2 + (lane >> 5)) << 4));
}
// operand fragment whose contraction index is the tile ROW (16-row step j) and whose free index is the column
// c0 + l%32; element e of lane half g is row 16j + 8*(e/4) + 4g + e%4 (matches an accumulator column)
template <int D>
__device__ __forceinline__ bf16x8 mc_frag(const char* lds, int j, int c0, int lane) {
  constexpr int rowb = AT<D>::row;
  int krow = j * 16 + 4 * (lane >> 5) + ((lane & 15) >> 2);
  int col = c0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const char* p = lds + krow * rowb + col * 2;
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((OASES_LDS short4v*)(p));
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((OASES_LDS short4v*)(p + 8 * rowb));
  typedef short short8v __attribute__((ext_vector_type(8)));
  short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int o) {
  u32x4 r = {pack_bf16x2(v[o], v[o + 1]), pack_bf16x2(v[o + 2], v[o + 3]), pack_bf16x2(v[o + 4], v[o + 5]),
             pack_bf16x2(v[o + 6], v[o + 7])};
  return __builtin_bit_cast(bf16x8, r);
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; i++) z[i] = 0.f;
  return z;
}
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

// 32 x D bf16 rows of one operand straight from global memory into B/A-operand registers: lane l holds row l%32,
// columns 16 ks + 8 (l/32) .. +7
template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8* f, const uint16_t* __restrict__ rowp, bool ok, int g) {
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) v = *reinterpret_cast<const u32x4*>(rowp + ks * 16 + 8 * g);
    f[ks] = __builtin_bit_cast(bf16x8, v);
  }
}

// sum of the four waves' partial accumulators through LDS: wave w ends up with elements [w*E/4, (w+1)*E/4) of the
// flattened (tile, element) index, summed over the four partials with the weights sc[0..3]
template <int E>
__device__ __forceinline__ void combine4(const f32x16* acc, float* lds_part, int wave, int lane, const float* sc, float* out) {
  __syncthreads();  // every wave is done with its tiles: the staging area is free
#pragma unroll
  for (int e = 0; e < E; e++) lds_part[(wave * E + e) * 64 + lane] = acc[e / 16][e % 16];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < E / 4; k++) {
    const int e = wave * (E / 4) + k;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) v += lds_part[(w * E + e) * 64 + lane] * sc[w];
    out[k] = v;
  }
}

// =================================================================================================
// forward
// =================================================================================================
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT, 2) void attn_fwd_kernel(AttnArgs a) {
  constexpr int KS = D / 16, DT = D / 32, E = DT * 16;
  constexpr int kStageBytes = 4 * 2 * AT<D>::bytes;
  constexpr int kPartBytes = 4 * E * 64 * 4;
  __shared__ __attribute__((aligned(16))) char lds[(kStageBytes > kPartBytes ? kStageBytes : kPartBytes) + 1024];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  int pair, blk;
  decode_block(blockIdx.x, a.nseq * a.heads, a.blocks, pair, blk);
  const int sq = pair / a.heads, head = pair % a.heads, qb = a.blocks - 1 - blk;  // long rows first
  const int seq_idx = a.seq0 + sq;
  const int q_begin = a.pos0 + qb * 32;
  const int q_end = min(a.pos0 + a.npos, q_begin + 32);
  const size_t rowbase = (size_t)seq_idx * a.seq;
  const uint16_t* Qp = a.qkv + rowbase * a.ld + head * D;
  const uint16_t* Kp = Qp + a.hp;
  const uint16_t* Vp = Qp + 2 * a.hp;
  const int qpos = q_begin + (lane & 31);
  const bool qok = qpos < q_end;

  bf16x8 qf[KS];
  load_row_frags<D>(qf, Qp + (size_t)qpos * a.ld, qok, g);
  f32x16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; i++) o[i] = zero16();
  float m = -INFINITY, l = 0.f;

  const int kv_end = CAUSAL ? q_end : a.seq;
  const int nt = (kv_end + 31) / 32;
  char* lk = lds + wave * 2 * AT<D>::bytes;
  char* lv = lk + AT<D>::bytes;
  u32x4 rk[AT<D>::per_lane], rv[AT<D>::per_lane];
  if (wave < nt) {
    wave_load<D>(rk, Kp, a.ld, wave * 32, 0, kv_end, lane);
    wave_load<D>(rv, Vp, a.ld, wave * 32, 0, kv_end, lane);
  }
  for (int t = wave; t < nt; t += 4) {
    const int kv0 = t * 32;
    wave_store<D>(rk, lk, lane);  // LDS operations of one wave execute in order: no barrier for a private tile
    wave_store<D>(rv, lv, lane);
    if (t + 4 < nt) {
      wave_load<D>(rk, Kp, a.ld, kv0 + 128, 0, kv_end, lane);
      wave_load<D>(rv, Vp, a.ld, kv0 + 128, 0, kv_end, lane);
    }
    f32x16 s = zero16(), s1 = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ks += 2) {  // two independent accumulation chains
      s = MFMA(kc_frag<D>(lk, ks, lane), qf[ks], s);
      s1 = MFMA(kc_frag<D>(lk, ks + 1, lane), qf[ks + 1], s1);
    }
    const bool need_mask = (kv0 + 32 > a.seq) || (CAUSAL && kv0 + 31 > q_begin);
    float mloc = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; i++) {
      float v = (s[i] + s1[i]) * a.scale_log2;
      if (need_mask) {
        int kvpos = kv0 + 8 * (i >> 2) + 4 * g + (i & 3);
        if (kvpos >= a.seq || (CAUSAL && kvpos > qpos)) v = -INFINITY;
      }
      s[i] = v;
      mloc = fmaxf(mloc, v);
    }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    // wave 0 starts with tile 0, which holds key 0, visible to every query; a later wave may start on a tile that is
    // masked for some of its queries: keep the running maximum finite there so that exp2 never sees inf - inf
    const float mnew = fmaxf(fmaxf(m, mloc), -1e30f);
    const float alpha = __builtin_amdgcn_exp2f(m - mnew);
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i++) {
      float p = __builtin_amdgcn_exp2f(s[i] - mnew);
      s[i] = p;
      psum += p;
    }
    l = l * alpha + psum;
    m = mnew;
    if (DROP) {  // the row sum keeps every probability; what goes on to V is dropped and rescaled
      const uint32_t bh = (uint32_t)(seq_idx * a.heads_total + a.head0 + head);
#pragma unroll
      for (int grp = 0; grp < 4; grp++) {
        const uint32_t ww = pick_word(attn_drop_block(a, (uint32_t)(kv0 + 8 * grp + 4 * g) >> 2, (uint32_t)qpos >> 2, bh), qpos & 3);
#pragma unroll
        for (int e = 0; e < 4; e++) s[4 * grp + e] = ((ww >> (8 * e)) & 0xffu) >= a.dthresh ? s[4 * grp + e] * a.dscale : 0.f;
      }
    }
    if (__any(alpha != 1.0f)) {  // the running maximum rarely moves after the first tiles
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int i = 0; i < 16; i++) o[dt][i] *= alpha;
    }
#pragma unroll
    for (int j = 0; j < 2; j++) {
      bf16x8 pb = pack8(s, 8 * j);
#pragma unroll
      for (int dt = 0; dt < DT; dt++) o[dt] = MFMA(mc_frag<D>(lv, j, 32 * dt, lane), pb, o[dt]);
    }
  }
  l += __shfl_xor(l, 32, 64);

  // merge the four partial (m, l, O): weights 2^(m_w - m)
  float* part = reinterpret_cast<float*>(lds);
  float* stat = reinterpret_cast<float*>(lds + (kStageBytes > kPartBytes ? kStageBytes : kPartBytes));  // m[4][32], l[4][32]
  __syncthreads();
  if (g == 0) { stat[wave * 32 + lane] = m; stat[128 + wave * 32 + lane] = l; }
  __syncthreads();
  float sc[4], mt = -INFINITY, lt = 0.f;
#pragma unroll
  for (int w = 0; w < 4; w++) mt = fmaxf(mt, stat[w * 32 + (lane & 31)]);
#pragma unroll
  for (int w = 0; w < 4; w++) {
    sc[w] = __builtin_amdgcn_exp2f(stat[w * 32 + (lane & 31)] - mt);
    lt += stat[128 + w * 32 + (lane & 31)] * sc[w];
  }
  float res[E / 4];
  combine4<E>(o, part, wave, lane, sc, res);
  if (qok) {
    const float inv = 1.0f / lt;
    uint16_t* op = a.out_w + (rowbase + qpos) * a.hp + head * D;
#pragma unroll
    for (int k = 0; k < E / 4; k += 4) {
      const int e = wave * (E / 4) + k, dt = e / 16, i = e % 16;
      const int d = dt * 32 + 8 * (i >> 2) + 4 * g;
      u32x2 v = {pack_bf16x2(res[k] * inv, res[k + 1] * inv), pack_bf16x2(res[k + 2] * inv, res[k + 3] * inv)};
      *reinterpret_cast<u32x2*>(op + d) = v;
    }
    if (wave == 0 && g == 0) a.lse[((size_t)seq_idx * a.heads + head) * a.seq + qpos] = (mt + __builtin_amdgcn_logf(lt)) * kLn2;
  }
}

// =================================================================================================
// backward: delta = rowsum(dO * O)
// =================================================================================================
template <int D>
__global__ __launch_bounds__(NT) void attn_delta_kernel(AttnArgs a, int first_row, int n_rows) {
  constexpr int LPR = D / 8;  // lanes per (row, head)
  const int gid = blockIdx.x * NT + threadIdx.x;
  const int pair = gid / LPR, c = gid % LPR;
  const int r = pair / a.heads, head = pair % a.heads;
  float s = 0.f;
  const bool ok = r < n_rows;
  const size_t row = (size_t)first_row + r;
  if (ok) {
    u32x4 x = *reinterpret_cast<const u32x4*>(a.out + row * a.hp + head * D + c * 8);
    u32x4 y = *reinterpret_cast<const u32x4*>(a.dout + row * a.hp + head * D + c * 8);
#pragma unroll
    for (int j = 0; j < 4; j++) {
      s += bf16_bits_to_f32(x[j] & 0xffffu) * bf16_bits_to_f32(y[j] & 0xffffu);
      s += bf16_bits_to_f32(x[j] >> 16) * bf16_bits_to_f32(y[j] >> 16);
    }
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (ok && c == 0) {
    int b = (int)(row / a.seq), pos = (int)(row % a.seq);
    a.delta[((size_t)b * a.heads + head) * a.seq + pos] = s;
  }
}

// =================================================================================================
// backward: dQ for a 32-query block; the four waves split the key tiles
// =================================================================================================
template <int D>
struct BwdLds {  // LDS of a backward workgroup: the larger of the two passes' staging areas and of the partial-sum exchange
  static constexpr int E = (D / 32) * 16;
  static constexpr int kStageDq = 4 * 2 * AT<D>::bytes, kStageDkv = 4 * (2 * AT<D>::bytes + 256), kPart = 4 * E * 64 * 4;
  static constexpr int bytes = kStageDkv > kPart ? kStageDkv : kPart;
  static_assert(kStageDkv >= kStageDq, "the dK/dV staging area is the larger one");
};

template <int D, bool CAUSAL, bool DROP>
__device__ __forceinline__ void attn_dq_block(const AttnArgs& a, int wg, char* lds) {
  constexpr int KS = D / 16, DT = D / 32, E = DT * 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  int pair, blk;
  decode_block(wg, a.nseq * a.heads, a.blocks, pair, blk);
  const int sq = pair / a.heads, head = pair % a.heads, qb = a.blocks - 1 - blk;
  const int seq_idx = a.seq0 + sq;
  const int q_begin = a.pos0 + qb * 32;
  const int q_end = min(a.pos0 + a.npos, q_begin + 32);
  const size_t rowbase = (size_t)seq_idx * a.seq;
  const uint16_t* Qp = a.qkv + rowbase * a.ld + head * D;
  const uint16_t* Kp = Qp + a.hp;
  const uint16_t* Vp = Qp + 2 * a.hp;
  const uint16_t* dOp = a.dout + rowbase * a.hp + head * D;
  const int qpos = q_begin + (lane & 31);
  const bool qok = qpos < q_end;

  bf16x8 qf[KS], dof[KS];
  load_row_frags<D>(qf, Qp + (size_t)qpos * a.ld, qok, g);
  load_row_frags<D>(dof, dOp + (size_t)qpos * a.hp, qok, g);
  float lse2 = 0.f, dl = 0.f;
  if (qok) {
    size_t si = ((size_t)seq_idx * a.heads + head) * a.seq + qpos;
    lse2 = a.lse[si] * kLog2e;
    dl = a.delta[si];
  }
  f32x16 acc[DT];
#pragma unroll
  for (int i = 0; i < DT; i++) acc[i] = zero16();

  const int kv_end = CAUSAL ? q_end : a.seq;
  const int nt = (kv_end + 31) / 32;
  char* lk = lds + wave * 2 * AT<D>::bytes;
  char* lv = lk + AT<D>::bytes;
  u32x4 rk[AT<D>::per_lane], rv[AT<D>::per_lane];
  if (wave < nt) {
    wave_load<D>(rk, Kp, a.ld, wave * 32, 0, kv_end, lane);
    wave_load<D>(rv, Vp, a.ld, wave * 32, 0, kv_end, lane);
  }
  for (int t = wave; t < nt; t += 4) {
    const int kv0 = t * 32;
    wave_store<D>(rk, lk, lane);
    wave_store<D>(rv, lv, lane);
    if (t + 4 < nt) {
      wave_load<D>(rk, Kp, a.ld, kv0 + 128, 0, kv_end, lane);
      wave_load<D>(rv, Vp, a.ld, kv0 + 128, 0, kv_end, lane);
    }
    f32x16 s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      s = MFMA(kc_frag<D>(lk, ks, lane), qf[ks], s);
      dp = MFMA(kc_frag<D>(lv, ks, lane), dof[ks], dp);
    }
    const bool need_mask = (kv0 + 32 > a.seq) || (CAUSAL && kv0 + 31 > q_begin);
    if (DROP) {  // dP = dropout factor * (dO V^T)
      const uint32_t bh = (uint32_t)(seq_idx * a.heads_total + a.head0 + head);
#pragma unroll
      for (int grp = 0; grp < 4; grp++) {
        const uint32_t ww = pick_word(attn_drop_block(a, (uint32_t)(kv0 + 8 * grp + 4 * g) >> 2, (uint32_t)qpos >> 2, bh), qpos & 3);
#pragma unroll
        for (int e = 0; e < 4; e++) dp[4 * grp + e] = ((ww >> (8 * e)) & 0xffu) >= a.dthresh ? dp[4 * grp + e] * a.dscale : 0.f;
      }
    }
    // only tiles on the diagonal or at the end of the sequence pay for the mask (a wave-uniform branch)
    auto scores = [&](auto mask_c) {
#pragma unroll
      for (int i = 0; i < 16; i++) {
        float ds = __builtin_amdgcn_exp2f(s[i] * a.scale_log2 - lse2) * (dp[i] - dl);
        if (decltype(mask_c)::value) {
          int kvpos = kv0 + 8 * (i >> 2) + 4 * g + (i & 3);
          if (kvpos >= a.seq || (CAUSAL && kvpos > qpos)) ds = 0.f;
        }
        s[i] = ds;
      }
    };
    if (need_mask) scores(std::true_type{}); else scores(std::false_type{});
#pragma unroll
    for (int j = 0; j < 2; j++) {
      bf16x8 db = pack8(s, 8 * j);
#pragma unroll
      for (int dt = 0; dt < DT; dt++) acc[dt] = MFMA(mc_frag<D>(lk, j, 32 * dt, lane), db, acc[dt]);
    }
  }
  const float one[4] = {1.f, 1.f, 1.f, 1.f};
  float res[E / 4];
  combine4<E>(acc, reinterpret_cast<float*>(lds), wave, lane, one, res);
  if (qok) {
    uint16_t* op = a.dqkv + (rowbase + qpos) * a.ld + head * D;
#pragma unroll
    for (int k = 0; k < E / 4; k += 4) {
      const int e = wave * (E / 4) + k, dt = e / 16, i = e % 16;
      const int d = dt * 32 + 8 * (i >> 2) + 4 * g;
      u32x2 v = {pack_bf16x2(res[k] * a.scale, res[k + 1] * a.scale), pack_bf16x2(res[k + 2] * a.scale, res[k + 3] * a.scale)};
      *reinterpret_cast<u32x2*>(op + d) = v;
    }
  }
}

// =================================================================================================
// backward: dK, dV for a 32-key block; the four waves split the 32-query tiles that see it
// =================================================================================================
template <int D, bool CAUSAL, bool DROP>
__device__ __forceinline__ void attn_dkv_block(const AttnArgs& a, int wg, char* lds) {
  constexpr int KS = D / 16, DT = D / 32, E = DT * 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  int pair, kb;
  decode_block(wg, a.nseq * a.heads, a.blocks, pair, kb);  // early key blocks are the long ones
  const int sq = pair / a.heads, head = pair % a.heads;
  const int seq_idx = a.seq0 + sq;
  const int k_begin = a.pos0 + kb * 32;
  const int k_end = min(a.pos0 + a.npos, k_begin + 32);
  const size_t rowbase = (size_t)seq_idx * a.seq;
  const uint16_t* Qp = a.qkv + rowbase * a.ld + head * D;
  const uint16_t* Kp = Qp + a.hp;
  const uint16_t* Vp = Qp + 2 * a.hp;
  const uint16_t* dOp = a.dout + rowbase * a.hp + head * D;
  const float* lsep = a.lse + ((size_t)seq_idx * a.heads + head) * a.seq;
  const float* dlp = a.delta + ((size_t)seq_idx * a.heads + head) * a.seq;
  const int kpos = k_begin + (lane & 31);
  const bool kok = kpos < k_end;

  bf16x8 kf[KS], vf[KS];
  load_row_frags<D>(kf, Kp + (size_t)kpos * a.ld, kok, g);
  load_row_frags<D>(vf, Vp + (size_t)kpos * a.ld, kok, g);
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int i = 0; i < DT; i++) { dk[i] = zero16(); dv[i] = zero16(); }

  const int qt0 = CAUSAL ? k_begin / 32 : 0;   // first query tile that sees this key block
  const int qmin = CAUSAL ? a.pos0 : 0;        // earlier queries never see a key of this row range
  const int nqt = (a.seq + 31) / 32;
  char* lq = lds + wave * (2 * AT<D>::bytes + 256);
  char* ldo = lq + AT<D>::bytes;
  float* lstat = reinterpret_cast<float*>(ldo + AT<D>::bytes);  // [32] lse * log2(e), [32] delta
  u32x4 rq[AT<D>::per_lane], rdo[AT<D>::per_lane];
  float rstat = 0.f;
  auto fetch = [&](int t) {
    wave_load<D>(rq, Qp, a.ld, t * 32, qmin, a.seq, lane);
    wave_load<D>(rdo, dOp, a.hp, t * 32, qmin, a.seq, lane);
    const int qp = min(t * 32 + (lane & 31), a.seq - 1);
    rstat = g == 0 ? lsep[qp] * kLog2e : dlp[qp];
  };
  if (qt0 + wave < nqt) fetch(qt0 + wave);
  for (int t = qt0 + wave; t < nqt; t += 4) {
    const int q0 = t * 32;
    wave_store<D>(rq, lq, lane);
    wave_store<D>(rdo, ldo, lane);
    lstat[lane] = rstat;
    if (t + 4 < nqt) fetch(t + 4);
    f32x16 s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      s = MFMA(kc_frag<D>(lq, ks, lane), kf[ks], s);
      dp = MFMA(kc_frag<D>(ldo, ks, lane), vf[ks], dp);
    }
    const bool need_mask = (q0 + 32 > a.seq) || (CAUSAL && q0 < k_begin + 31);
    // only tiles on the diagonal or at the end of the sequence pay for the mask (a wave-uniform branch)
    auto scores = [&](auto mask_c) {
#pragma unroll
      for (int i4 = 0; i4 < 4; i4++) {
        const int ql = 8 * i4 + 4 * g;  // 4 consecutive queries
        f32x4 l4 = *reinterpret_cast<const f32x4*>(lstat + ql);
        f32x4 d4 = *reinterpret_cast<const f32x4*>(lstat + 32 + ql);
        Philox4 dw;
        if (DROP) dw = attn_drop_block(a, (uint32_t)kpos >> 2, (uint32_t)(q0 + ql) >> 2, (uint32_t)(seq_idx * a.heads_total + a.head0 + head));
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const int i = 4 * i4 + e;
          const float p = __builtin_amdgcn_exp2f(s[i] * a.scale_log2 - l4[e]);
          float dpe = dp[i], pv = p;  // pv: what multiplied V in forward
          if (DROP) {  // this lane's key is byte (kpos mod 4) of the word of query e of the group
            const bool keep = ((dw.v[e] >> (8 * (kpos & 3))) & 0xffu) >= a.dthresh;
            dpe = keep ? dpe * a.dscale : 0.f;
            pv = keep ? p * a.dscale : 0.f;
          }
          float ds = p * (dpe - d4[e]);
          if (decltype(mask_c)::value) {
            int qp = q0 + ql + e;
            if (qp >= a.seq || (CAUSAL && kpos > qp)) { pv = 0.f; ds = 0.f; }   // select, never multiply: the rest may be NaN
          }
          s[i] = pv;
          dp[i] = ds;
        }
      }
    };
    if (need_mask) scores(std::true_type{}); else scores(std::false_type{});
#pragma unroll
    for (int j = 0; j < 2; j++) {
      bf16x8 pa = pack8(s, 8 * j);
      bf16x8 da = pack8(dp, 8 * j);
#pragma unroll
      for (int dt = 0; dt < DT; dt++) {
        dv[dt] = MFMA(pa, mc_frag<D>(ldo, j, 32 * dt, lane), dv[dt]);
        dk[dt] = MFMA(da, mc_frag<D>(lq, j, 32 * dt, lane), dk[dt]);
      }
    }
  }
  // accumulator row = key 8*(i/4) + 4g + i%4 of the block, column = d = 32*dt + l%32
  const float one[4] = {1.f, 1.f, 1.f, 1.f};
  float rk_[E / 4], rv_[E / 4];
  combine4<E>(dk, reinterpret_cast<float*>(lds), wave, lane, one, rk_);
  combine4<E>(dv, reinterpret_cast<float*>(lds), wave, lane, one, rv_);
  uint16_t* dKp = a.dqkv + rowbase * a.ld + a.hp + head * D;
  uint16_t* dVp = dKp + a.hp;
#pragma unroll
  for (int k = 0; k < E / 4; k++) {
    const int e = wave * (E / 4) + k, dt = e / 16, i = e % 16;
    const int kp = k_begin + 8 * (i >> 2) + 4 * g + (i & 3);
    if (kp < k_end) {
      size_t o = (size_t)kp * a.ld + dt * 32 + (lane & 31);
      dKp[o] = (uint16_t)f32_to_bf16_bits(rk_[k] * a.scale);
      dVp[o] = (uint16_t)f32_to_bf16_bits(rv_[k]);
    }
  }
}

// The two backward passes as launches of their own (many blocks: each pass fills the chip by itself, and keeps the L2 of an
// XCD to one pass's operands) ...
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT, 1) void attn_dq_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) char lds[BwdLds<D>::bytes];
  attn_dq_block<D, CAUSAL, DROP>(a, blockIdx.x, lds);
}
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT, 1) void attn_dkv_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) char lds[BwdLds<D>::bytes];
  attn_dkv_block<D, CAUSAL, DROP>(a, blockIdx.x, lds);
}

// ... and in ONE launch, for calls with few blocks (at most one workgroup per CU and pass: a sub-batch that is a chunk of a
// sequence, short sequences): the passes are independent (dK/dV per key block, dQ per query block) and each alone leaves
// the chip waiting for its longest workgroups, so their workgroups are dealt out together -- groups of eight ids (one per
// XCD) alternate between a dK/dV block and a dQ block, long blocks of both kinds first.  Measured (C5's chunks, 256 blocks):
// 40 -> 32 us; with 512 blocks and more the single launch is about 10 % slower than two.
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT, 1) void attn_bwd_kernel(AttnArgs a, int n_blocks) {
  __shared__ __attribute__((aligned(16))) char lds[BwdLds<D>::bytes];
  const int w = blockIdx.x, idx = (w >> 4) * 8 + (w & 7);
  if (idx >= n_blocks) return;  // the last group of eight may be ragged (whole workgroup leaves: no barrier is skipped by part of it)
  if ((w >> 3) & 1) attn_dq_block<D, CAUSAL, DROP>(a, idx, lds);
  else attn_dkv_block<D, CAUSAL, DROP>(a, idx, lds);
}

int fill_args(AttnArgs& a, int batch, int seq, int heads, int head_dim, int causal, int row0, int rows, const char* who) {
  if (batch <= 0 || seq <= 0 || heads <= 0 || (head_dim != 64 && head_dim != 128) || row0 < 0 || rows <= 0 ||
      (long)row0 + rows > (long)batch * seq) {
    set_error("%s: bad shape (batch=%d seq=%d heads=%d head_dim=%d row0=%d rows=%d)", who, batch, seq, heads, head_dim, row0, rows);
    return OASES_EINVAL;
  }
  a.seq = seq;
  a.heads = heads;
  a.hp = heads * head_dim;
  a.ld = 3 * a.hp;
  a.seq0 = row0 / seq;
  if (row0 % seq == 0 && rows % seq == 0) {
    a.pos0 = 0;
    a.npos = seq;
    a.blocks = (seq + 31) / 32;
    return rows / seq;  // number of sequences
  }
  if (row0 / seq != (row0 + rows - 1) / seq) {
    set_error("%s: rows [%d,%d) are neither whole sequences nor part of one sequence", who, row0, row0 + rows);
    return OASES_EINVAL;
  }
  if (!causal) {
    set_error("%s: a row range inside one sequence needs causal attention", who);
    return OASES_EINVAL;
  }
  a.pos0 = row0 % seq;
  a.npos = rows;
  a.blocks = (rows + 31) / 32;
  return 1;
}

}  // namespace

// fills the dropout fields; false (after set_error) on a bad rate or head range
static bool fill_dropout(AttnArgs& a, uint64_t seed, int layer, float p_attn, int head0, int heads_total, int heads, const char* who) {
  if (!(p_attn >= 0.f && p_attn < 1.f)) { set_error("%s: attention dropout rate %g outside [0,1)", who, (double)p_attn); return false; }
  int T = (int)__builtin_rint((double)p_attn * 256.0);
  if (T > 255) T = 255;
  a.dthresh = (uint32_t)T;
  if (T == 0) return true;
  if (heads_total <= 0 || head0 < 0 || head0 + heads > heads_total) { set_error("%s: heads [%d,%d) outside the %d heads of the layer", who, head0, head0 + heads, heads_total); return false; }
  a.dk0 = (uint32_t)seed;
  a.dk1 = (uint32_t)(seed >> 32);
  a.dc3 = ((uint32_t)layer & 0x7fffffffu) | 0x80000000u;
  a.dscale = (float)(256.0 / (256.0 - T));
  a.head0 = head0;
  a.heads_total = heads_total;
  return true;
}

int launch_attention_fwd(const void* qkv, void* out, float* lse, int batch, int seq, int heads, int head_dim, int causal,
                         int row0, int rows, hipStream_t s, uint64_t seed, int layer, float p_attn, int head0, int heads_total) {
  if (!qkv || !out || !lse) { set_error("attention_fwd: NULL argument"); return OASES_ENULL; }
  if (!aligned16(qkv) || !aligned16(out)) { set_error("attention_fwd: pointer not 16-byte aligned"); return OASES_EALIGN; }
  AttnArgs a{};
  int nseq = fill_args(a, batch, seq, heads, head_dim, causal, row0, rows, "attention_fwd");
  if (nseq < 0) return nseq;
  a.qkv = (const uint16_t*)qkv;
  a.out_w = (uint16_t*)out;
  a.lse = lse;
  a.scale = 1.0f / sqrtf((float)head_dim);
  a.scale_log2 = a.scale * kLog2e;
  a.nseq = nseq;
  if (!fill_dropout(a, seed, layer, p_attn, head0, heads_total, heads, "attention_fwd")) return OASES_EINVAL;
  dim3 grid(nseq * a.blocks * heads), block(NT);
#define OASES_ATTN_FWD(DD, CC)                                                                              \
  do {                                                                                                      \
    if (a.dthresh) hipLaunchKernelGGL((attn_fwd_kernel<DD, CC, true>), grid, block, 0, s, a);               \
    else hipLaunchKernelGGL((attn_fwd_kernel<DD, CC, false>), grid, block, 0, s, a);                        \
  } while (0)
  if (head_dim == 64) { if (causal) OASES_ATTN_FWD(64, true); else OASES_ATTN_FWD(64, false); }
  else { if (causal) OASES_ATTN_FWD(128, true); else OASES_ATTN_FWD(128, false); }
#undef OASES_ATTN_FWD
  OASES_LAUNCH_CHECK("attn_fwd_kernel");
  return 0;
}

int launch_attention_bwd(const void* qkv, const void* out, const void* dout, const float* lse, float* delta, void* dqkv,
                         int batch, int seq, int heads, int head_dim, int causal, int row0, int rows, hipStream_t s, uint64_t seed,
                         int layer, float p_attn, int head0, int heads_total) {
  if (!qkv || !out || !dout || !lse || !delta || !dqkv) { set_error("attention_bwd: NULL argument"); return OASES_ENULL; }
  if (!aligned16(qkv) || !aligned16(out) || !aligned16(dout) || !aligned16(dqkv)) {
    set_error("attention_bwd: pointer not 16-byte aligned");
    return OASES_EALIGN;
  }
  AttnArgs a{};
  int nseq = fill_args(a, batch, seq, heads, head_dim, causal, row0, rows, "attention_bwd");
  if (nseq < 0) return nseq;
  a.qkv = (const uint16_t*)qkv;
  a.out = (const uint16_t*)out;
  a.dout = (const uint16_t*)dout;
  a.lse = const_cast<float*>(lse);
  a.delta = delta;
  a.dqkv = (uint16_t*)dqkv;
  a.scale = 1.0f / sqrtf((float)head_dim);
  a.scale_log2 = a.scale * kLog2e;
  // delta for every query that sees a key of the range: from the first row to the end of the last sequence
  const int first_row = row0;
  const int n_rows = (a.seq0 + nseq) * seq - row0;
  const long pairs = (long)n_rows * heads * (head_dim / 8);
  a.nseq = nseq;
  if (!fill_dropout(a, seed, layer, p_attn, head0, heads_total, heads, "attention_bwd")) return OASES_EINVAL;
  dim3 dgrid((unsigned)((pairs + NT - 1) / NT)), block(NT);
  if (head_dim == 64) hipLaunchKernelGGL((attn_delta_kernel<64>), dgrid, block, 0, s, a, first_row, n_rows);
  else hipLaunchKernelGGL((attn_delta_kernel<128>), dgrid, block, 0, s, a, first_row, n_rows);
  OASES_LAUNCH_CHECK("attn_delta_kernel");
  const int n_blocks = nseq * a.blocks * heads;
  const bool one_launch = n_blocks <= 256;
  const dim3 bgrid(2 * ((n_blocks + 7) / 8) * 8), grid(n_blocks);
#define OASES_ATTN_BWD(DD, CC, DR)                                                                        \
  do {                                                                                                    \
    if (one_launch) {                                                                                     \
      hipLaunchKernelGGL((attn_bwd_kernel<DD, CC, DR>), bgrid, block, 0, s, a, n_blocks);                 \
    } else {                                                                                              \
      hipLaunchKernelGGL((attn_dkv_kernel<DD, CC, DR>), grid, block, 0, s, a);                            \
      hipLaunchKernelGGL((attn_dq_kernel<DD, CC, DR>), grid, block, 0, s, a);                             \
    }                                                                                                     \
  } while (0)
#define OASES_ATTN_BWD_D(DD, CC) do { if (a.dthresh) OASES_ATTN_BWD(DD, CC, true); else OASES_ATTN_BWD(DD, CC, false); } while (0)
  if (head_dim == 64) { if (causal) OASES_ATTN_BWD_D(64, true); else OASES_ATTN_BWD_D(64, false); }
  else { if (causal) OASES_ATTN_BWD_D(128, true); else OASES_ATTN_BWD_D(128, false); }
#undef OASES_ATTN_BWD_D
#undef OASES_ATTN_BWD
  OASES_LAUNCH_CHECK("attn_bwd kernels");
  return 0;
}

}  // namespace oases
