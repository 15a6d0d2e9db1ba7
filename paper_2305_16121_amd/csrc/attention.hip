// Flash-style attention for the local heads of one TMP rank (gfx950, bf16 MFMA, fp32 softmax).
//
// Forward and the dQ kernel compute the TRANSPOSED score tile S^T = K*Q^T with
// v_mfma_f32_32x32x16_bf16, so that a lane owns one query (accumulator column l%32) and 16 keys of
// every 32-key tile: the online softmax is then lane-local except for one exchange between the two
// lane halves, and the exponentials are already in B-operand position for O^T = V^T * P^T (the
// k index of that product is permuted the same way for both operands: rows 4*(l/32)+{0..3} and
// +8 of each 16-key step; the V^T operand comes from the LDS transpose read).
// The dK/dV kernel keeps S = Q*K^T un-transposed so a lane owns one key and P^T / dS^T are in
// A-operand position.  No atomics: dQ and dK/dV are separate passes, results are deterministic.
#include "common.h"

namespace oases {

namespace {

constexpr int NT = 256;
constexpr int kPad = 64;  // bytes of row padding of tiles read through ds_read_b64_tr_b16
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
  int blocks;  // 128-row blocks per sequence
  float scale, scale_log2;
};

template <int ROWS, int D>
struct Tile {
  static constexpr int cpr = D / 8;
  static constexpr int chunks = ROWS * cpr;
  static constexpr int per_thread = chunks / NT;
  static constexpr int kc_row = D * 2;
  static constexpr int mc_row = D * 2 + kPad;
  static constexpr int kc_bytes = ROWS * kc_row;
  static constexpr int mc_bytes = ROWS * mc_row;
};

// XOR swizzle of the 16-byte chunk index of a row-major [rows][D] tile: 16 consecutive rows read at the same
// logical chunk must land on 16 different bank groups (64 banks x 4 bytes, 16 lanes per LDS cycle)
template <int D>
__device__ __forceinline__ int kc_swizzle(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}

// rows [r0, r0+ROWS) of a [*, D] slice with row stride ld; rows >= rmax read as zero
template <int ROWS, int D>
__device__ __forceinline__ void load_rows(u32x4* regs, const uint16_t* __restrict__ base, int ld,
                                          int r0, int rmax, int tid) {
  using T = Tile<ROWS, D>;
#pragma unroll
  for (int i = 0; i < T::per_thread; i++) {
    int c = tid + i * NT;
    int row = c / T::cpr, cc = c % T::cpr;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r0 + row < rmax) v = *reinterpret_cast<const u32x4*>(base + (size_t)(r0 + row) * ld + cc * 8);
    regs[i] = v;
  }
}
template <int ROWS, int D>
__device__ __forceinline__ void store_kc(const u32x4* regs, char* lds, int tid) {
  using T = Tile<ROWS, D>;
#pragma unroll
  for (int i = 0; i < T::per_thread; i++) {
    int c = tid + i * NT;
    int row = c / T::cpr, cc = c % T::cpr;
    *reinterpret_cast<u32x4*>(lds + row * T::kc_row + ((cc ^ kc_swizzle<D>(row)) << 4)) = regs[i];
  }
}
template <int ROWS, int D>
__device__ __forceinline__ void store_mc(const u32x4* regs, char* lds, int tid) {
  using T = Tile<ROWS, D>;
#pragma unroll
  for (int i = 0; i < T::per_thread; i++) {
    int c = tid + i * NT;
    int row = c / T::cpr, cc = c % T::cpr;
    *reinterpret_cast<u32x4*>(lds + row * T::mc_row + (cc << 4)) = regs[i];
  }
}
// operand fragment (32 rows x 16 contraction) of a row-major [rows][D] tile, contraction along D
template <int D>
__device__ __forceinline__ bf16x8 kc_frag(const char* lds, int r0, int ks, int lane) {
  int row = r0 + (lane & 31);
  int chunk = ks * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(lds + row * (D * 2) + ((chunk ^ kc_swizzle<D>(lane & 31)) << 4));
}
// operand fragment whose contraction index is the tile ROW (16-row step j) and whose free index is the
// column c0 + l%32; element e of lane half g is row 16j + 8*(e/4) + 4g + e%4 (matches an accumulator column)
template <int D>
__device__ __forceinline__ bf16x8 mc_frag(const char* lds, int j, int c0, int lane) {
  constexpr int rowb = D * 2 + kPad;
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

// =================================================================================================
// forward
// =================================================================================================
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_fwd_kernel(AttnArgs a) {
  using TK = Tile<64, D>;
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) char lds[2 * (TK::kc_bytes + TK::mc_bytes)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  const int sq = blockIdx.x / a.blocks, qb = blockIdx.x % a.blocks, head = blockIdx.y;
  const int seq_idx = a.seq0 + sq;
  const int q_begin = a.pos0 + qb * 128;
  const int q_end = min(a.pos0 + a.npos, q_begin + 128);
  const size_t rowbase = (size_t)seq_idx * a.seq;
  const uint16_t* Qp = a.qkv + rowbase * a.ld + head * D;
  const uint16_t* Kp = Qp + a.hp;
  const uint16_t* Vp = Qp + 2 * a.hp;
  const int qw = q_begin + 32 * wave;
  const int qpos = qw + (lane & 31);
  const bool qok = qpos < q_end;

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (qok) v = *reinterpret_cast<const u32x4*>(Qp + (size_t)qpos * a.ld + ks * 16 + 8 * g);
    qf[ks] = __builtin_bit_cast(bf16x8, v);
  }
  f32x16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; i++) o[i] = zero16();
  float m = -INFINITY, l = 0.f;

  const int kv_end = CAUSAL ? q_end : a.seq;
  const int nt = (kv_end + 63) / 64;
  constexpr int kStage = TK::kc_bytes + TK::mc_bytes;  // stage s: K at lds + s*kStage, V behind it
  u32x4 rk[TK::per_thread], rv[TK::per_thread];
  load_rows<64, D>(rk, Kp, a.ld, 0, a.seq, tid);
  load_rows<64, D>(rv, Vp, a.ld, 0, a.seq, tid);
  store_kc<64, D>(rk, lds, tid);
  store_mc<64, D>(rv, lds + TK::kc_bytes, tid);
  if (nt > 1) {
    load_rows<64, D>(rk, Kp, a.ld, 64, a.seq, tid);
    load_rows<64, D>(rv, Vp, a.ld, 64, a.seq, tid);
  }
  __syncthreads();

  for (int t = 0; t < nt; t++) {
    const int cur = t & 1, kv0 = t * 64;
    if (t + 1 < nt) {
      store_kc<64, D>(rk, lds + (cur ^ 1) * kStage, tid);
      store_mc<64, D>(rv, lds + (cur ^ 1) * kStage + TK::kc_bytes, tid);
      if (t + 2 < nt) {
        load_rows<64, D>(rk, Kp, a.ld, (t + 2) * 64, a.seq, tid);
        load_rows<64, D>(rv, Vp, a.ld, (t + 2) * 64, a.seq, tid);
      }
    }
    if (!(CAUSAL && kv0 > qw + 31)) {
      const char* lk = lds + cur * kStage;
      const char* lv = lk + TK::kc_bytes;
      f32x16 s[2];
#pragma unroll
      for (int u = 0; u < 2; u++) {
        s[u] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ks++) s[u] = MFMA(kc_frag<D>(lk, 32 * u, ks, lane), qf[ks], s[u]);
      }
      const bool need_mask = (kv0 + 64 > a.seq) || (CAUSAL && kv0 + 63 > qw);
      float mloc = -INFINITY;
#pragma unroll
      for (int u = 0; u < 2; u++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          float v = s[u][i] * a.scale_log2;
          if (need_mask) {
            int kvpos = kv0 + 32 * u + 8 * (i >> 2) + 4 * g + (i & 3);
            if (kvpos >= a.seq || (CAUSAL && kvpos > qpos)) v = -INFINITY;
          }
          s[u][i] = v;
          mloc = fmaxf(mloc, v);
        }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
      const float mnew = fmaxf(m, mloc);  // finite: the first tile always holds key 0, visible to every query
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);
      float psum = 0.f;
#pragma unroll
      for (int u = 0; u < 2; u++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          float p = __builtin_amdgcn_exp2f(s[u][i] - mnew);
          s[u][i] = p;
          psum += p;
        }
      l = l * alpha + psum;
      m = mnew;
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int i = 0; i < 16; i++) o[dt][i] *= alpha;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        bf16x8 pb = pack8(s[j >> 1], 8 * (j & 1));
#pragma unroll
        for (int dt = 0; dt < DT; dt++) o[dt] = MFMA(mc_frag<D>(lv, j, 32 * dt, lane), pb, o[dt]);
      }
    }
    __syncthreads();
  }
  l += __shfl_xor(l, 32, 64);
  if (qok) {
    const float inv = 1.0f / l;
    uint16_t* op = a.out_w + (rowbase + qpos) * a.hp + head * D;
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        int d = dt * 32 + 8 * q4 + 4 * g;
        u32x2 v = {pack_bf16x2(o[dt][4 * q4] * inv, o[dt][4 * q4 + 1] * inv),
                   pack_bf16x2(o[dt][4 * q4 + 2] * inv, o[dt][4 * q4 + 3] * inv)};
        *reinterpret_cast<u32x2*>(op + d) = v;
      }
    if (g == 0) a.lse[((size_t)seq_idx * a.heads + head) * a.seq + qpos] = (m + __builtin_amdgcn_logf(l)) * kLn2;
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
// backward: dQ for a 128-query block (same tiling as forward)
// =================================================================================================
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_dq_kernel(AttnArgs a) {
  using TK = Tile<64, D>;
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) char lds[2 * TK::kc_bytes + TK::mc_bytes];
  char* lk = lds;                    // K, contraction along d
  char* lv = lds + TK::kc_bytes;     // V, contraction along d
  char* lkt = lds + 2 * TK::kc_bytes;  // K again, read transposed
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  const int sq = blockIdx.x / a.blocks, qb = blockIdx.x % a.blocks, head = blockIdx.y;
  const int seq_idx = a.seq0 + sq;
  const int q_begin = a.pos0 + qb * 128;
  const int q_end = min(a.pos0 + a.npos, q_begin + 128);
  const size_t rowbase = (size_t)seq_idx * a.seq;
  const uint16_t* Qp = a.qkv + rowbase * a.ld + head * D;
  const uint16_t* Kp = Qp + a.hp;
  const uint16_t* Vp = Qp + 2 * a.hp;
  const uint16_t* dOp = a.dout + rowbase * a.hp + head * D;
  const int qw = q_begin + 32 * wave;
  const int qpos = qw + (lane & 31);
  const bool qok = qpos < q_end;

  bf16x8 qf[KS], dof[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    u32x4 v = {0u, 0u, 0u, 0u}, w = {0u, 0u, 0u, 0u};
    if (qok) {
      v = *reinterpret_cast<const u32x4*>(Qp + (size_t)qpos * a.ld + ks * 16 + 8 * g);
      w = *reinterpret_cast<const u32x4*>(dOp + (size_t)qpos * a.hp + ks * 16 + 8 * g);
    }
    qf[ks] = __builtin_bit_cast(bf16x8, v);
    dof[ks] = __builtin_bit_cast(bf16x8, w);
  }
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
  const int nt = (kv_end + 63) / 64;
  u32x4 rk[TK::per_thread], rv[TK::per_thread];
  load_rows<64, D>(rk, Kp, a.ld, 0, a.seq, tid);
  load_rows<64, D>(rv, Vp, a.ld, 0, a.seq, tid);
  for (int t = 0; t < nt; t++) {
    const int kv0 = t * 64;
    __syncthreads();
    store_kc<64, D>(rk, lk, tid);
    store_mc<64, D>(rk, lkt, tid);
    store_kc<64, D>(rv, lv, tid);
    __syncthreads();
    if (t + 1 < nt) {
      load_rows<64, D>(rk, Kp, a.ld, kv0 + 64, a.seq, tid);
      load_rows<64, D>(rv, Vp, a.ld, kv0 + 64, a.seq, tid);
    }
    if (CAUSAL && kv0 > qw + 31) continue;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
      s[u] = zero16();
      dp[u] = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        s[u] = MFMA(kc_frag<D>(lk, 32 * u, ks, lane), qf[ks], s[u]);
        dp[u] = MFMA(kc_frag<D>(lv, 32 * u, ks, lane), dof[ks], dp[u]);
      }
    }
    const bool need_mask = (kv0 + 64 > a.seq) || (CAUSAL && kv0 + 63 > qw);
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
      for (int i = 0; i < 16; i++) {
        float p = __builtin_amdgcn_exp2f(s[u][i] * a.scale_log2 - lse2);
        if (need_mask) {
          int kvpos = kv0 + 32 * u + 8 * (i >> 2) + 4 * g + (i & 3);
          if (kvpos >= a.seq || (CAUSAL && kvpos > qpos)) p = 0.f;
        }
        s[u][i] = p * (dp[u][i] - dl);
      }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      bf16x8 db = pack8(s[j >> 1], 8 * (j & 1));
#pragma unroll
      for (int dt = 0; dt < DT; dt++) acc[dt] = MFMA(mc_frag<D>(lkt, j, 32 * dt, lane), db, acc[dt]);
    }
  }
  if (qok) {
    uint16_t* op = a.dqkv + (rowbase + qpos) * a.ld + head * D;
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        int d = dt * 32 + 8 * q4 + 4 * g;
        u32x2 v = {pack_bf16x2(acc[dt][4 * q4] * a.scale, acc[dt][4 * q4 + 1] * a.scale),
                   pack_bf16x2(acc[dt][4 * q4 + 2] * a.scale, acc[dt][4 * q4 + 3] * a.scale)};
        *reinterpret_cast<u32x2*>(op + d) = v;
      }
  }
}

// =================================================================================================
// backward: dK, dV for a 128-key block; loops over the 64-query tiles that see it
// =================================================================================================
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_dkv_kernel(AttnArgs a) {
  using TQ = Tile<64, D>;
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) char lds[2 * (TQ::kc_bytes + TQ::mc_bytes) + 512];
  char* lq = lds;
  char* lqt = lq + TQ::kc_bytes;
  char* ldo = lqt + TQ::mc_bytes;
  char* ldot = ldo + TQ::kc_bytes;
  float* lstat = reinterpret_cast<float*>(ldot + TQ::mc_bytes);  // [64] lse2, [64] delta
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  const int sq = blockIdx.x / a.blocks, kb = blockIdx.x % a.blocks, head = blockIdx.y;
  const int seq_idx = a.seq0 + sq;
  const int k_begin = a.pos0 + kb * 128;
  const int k_end = min(a.pos0 + a.npos, k_begin + 128);
  const size_t rowbase = (size_t)seq_idx * a.seq;
  const uint16_t* Qp = a.qkv + rowbase * a.ld + head * D;
  const uint16_t* Kp = Qp + a.hp;
  const uint16_t* Vp = Qp + 2 * a.hp;
  const uint16_t* dOp = a.dout + rowbase * a.hp + head * D;
  const float* lsep = a.lse + ((size_t)seq_idx * a.heads + head) * a.seq;
  const float* dlp = a.delta + ((size_t)seq_idx * a.heads + head) * a.seq;
  const int kw = k_begin + 32 * wave;
  const int kpos = kw + (lane & 31);
  const bool kok = kpos < k_end;

  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    u32x4 v = {0u, 0u, 0u, 0u}, w = {0u, 0u, 0u, 0u};
    if (kok) {
      v = *reinterpret_cast<const u32x4*>(Kp + (size_t)kpos * a.ld + ks * 16 + 8 * g);
      w = *reinterpret_cast<const u32x4*>(Vp + (size_t)kpos * a.ld + ks * 16 + 8 * g);
    }
    kf[ks] = __builtin_bit_cast(bf16x8, v);
    vf[ks] = __builtin_bit_cast(bf16x8, w);
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int i = 0; i < DT; i++) { dk[i] = zero16(); dv[i] = zero16(); }

  const int qt0 = CAUSAL ? k_begin / 64 : 0;
  const int nqt = (a.seq + 63) / 64;
  u32x4 rq[TQ::per_thread], rdo[TQ::per_thread];
  float rstat = 0.f;
  auto fetch = [&](int t) {
    load_rows<64, D>(rq, Qp, a.ld, t * 64, a.seq, tid);
    load_rows<64, D>(rdo, dOp, a.hp, t * 64, a.seq, tid);
    if (tid < 128) {
      int qp = t * 64 + (tid & 63);
      rstat = 0.f;
      if (qp < a.seq) rstat = tid < 64 ? lsep[qp] * kLog2e : dlp[qp];
    }
  };
  if (qt0 < nqt) fetch(qt0);
  for (int t = qt0; t < nqt; t++) {
    const int q0 = t * 64;
    __syncthreads();
    store_kc<64, D>(rq, lq, tid);
    store_mc<64, D>(rq, lqt, tid);
    store_kc<64, D>(rdo, ldo, tid);
    store_mc<64, D>(rdo, ldot, tid);
    if (tid < 128) lstat[tid] = rstat;
    __syncthreads();
    if (t + 1 < nqt) fetch(t + 1);
    if (CAUSAL && q0 + 63 < kw) continue;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
      s[u] = zero16();
      dp[u] = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        s[u] = MFMA(kc_frag<D>(lq, 32 * u, ks, lane), kf[ks], s[u]);
        dp[u] = MFMA(kc_frag<D>(ldo, 32 * u, ks, lane), vf[ks], dp[u]);
      }
    }
    const bool need_mask = (q0 + 64 > a.seq) || (CAUSAL && q0 < kw + 31);
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
      for (int i4 = 0; i4 < 4; i4++) {
        const int ql = 32 * u + 8 * i4 + 4 * g;  // 4 consecutive queries
        f32x4 l4 = *reinterpret_cast<const f32x4*>(lstat + ql);
        f32x4 d4 = *reinterpret_cast<const f32x4*>(lstat + 64 + ql);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const int i = 4 * i4 + e;
          float p = __builtin_amdgcn_exp2f(s[u][i] * a.scale_log2 - l4[e]);
          if (need_mask) {
            int qp = q0 + ql + e;
            if (qp >= a.seq || (CAUSAL && kpos > qp)) p = 0.f;
          }
          s[u][i] = p;
          dp[u][i] = p * (dp[u][i] - d4[e]);
        }
      }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      bf16x8 pa = pack8(s[j >> 1], 8 * (j & 1));
      bf16x8 da = pack8(dp[j >> 1], 8 * (j & 1));
#pragma unroll
      for (int dt = 0; dt < DT; dt++) {
        dv[dt] = MFMA(pa, mc_frag<D>(ldot, j, 32 * dt, lane), dv[dt]);
        dk[dt] = MFMA(da, mc_frag<D>(lqt, j, 32 * dt, lane), dk[dt]);
      }
    }
  }
  // accumulator row = key 8*(i/4) + 4g + i%4 of this wave's 32, column = d = 32*dt + l%32
  uint16_t* dKp = a.dqkv + rowbase * a.ld + a.hp + head * D;
  uint16_t* dVp = dKp + a.hp;
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int i = 0; i < 16; i++) {
      int kp = kw + 8 * (i >> 2) + 4 * g + (i & 3);
      if (kp < k_end) {
        size_t o = (size_t)kp * a.ld + dt * 32 + (lane & 31);
        dKp[o] = (uint16_t)f32_to_bf16_bits(dk[dt][i] * a.scale);
        dVp[o] = (uint16_t)f32_to_bf16_bits(dv[dt][i]);
      }
    }
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
    a.blocks = (seq + 127) / 128;
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
  a.blocks = (rows + 127) / 128;
  return 1;
}

}  // namespace

int launch_attention_fwd(const void* qkv, void* out, float* lse, int batch, int seq, int heads, int head_dim, int causal,
                         int row0, int rows, hipStream_t s) {
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
  dim3 grid(nseq * a.blocks, heads), block(NT);
  if (head_dim == 64) {
    if (causal) hipLaunchKernelGGL((attn_fwd_kernel<64, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((attn_fwd_kernel<64, false>), grid, block, 0, s, a);
  } else {
    if (causal) hipLaunchKernelGGL((attn_fwd_kernel<128, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((attn_fwd_kernel<128, false>), grid, block, 0, s, a);
  }
  OASES_LAUNCH_CHECK("attn_fwd_kernel");
  return 0;
}

int launch_attention_bwd(const void* qkv, const void* out, const void* dout, const float* lse, float* delta, void* dqkv,
                         int batch, int seq, int heads, int head_dim, int causal, int row0, int rows, hipStream_t s) {
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
  dim3 dgrid((unsigned)((pairs + NT - 1) / NT)), block(NT), grid(nseq * a.blocks, heads);
  if (head_dim == 64) hipLaunchKernelGGL((attn_delta_kernel<64>), dgrid, block, 0, s, a, first_row, n_rows);
  else hipLaunchKernelGGL((attn_delta_kernel<128>), dgrid, block, 0, s, a, first_row, n_rows);
  OASES_LAUNCH_CHECK("attn_delta_kernel");
#define OASES_ATTN_BWD(DD, CC)                                                    \
  do {                                                                            \
    hipLaunchKernelGGL((attn_dkv_kernel<DD, CC>), grid, block, 0, s, a);          \
    hipLaunchKernelGGL((attn_dq_kernel<DD, CC>), grid, block, 0, s, a);           \
  } while (0)
  if (head_dim == 64) { if (causal) OASES_ATTN_BWD(64, true); else OASES_ATTN_BWD(64, false); }
  else { if (causal) OASES_ATTN_BWD(128, true); else OASES_ATTN_BWD(128, false); }
#undef OASES_ATTN_BWD
  OASES_LAUNCH_CHECK("attn_bwd kernels");
  return 0;
}

}  // namespace oases
