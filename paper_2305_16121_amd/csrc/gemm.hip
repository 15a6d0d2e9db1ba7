// bf16 MFMA GEMM family for gfx950: C = A*B with fp32 accumulation, LDS-staged tiles.
//
// One kernel template covers the three contractions of a linear map under Megatron's partition
// (paper Sec. II): forward (A k-contiguous, B n-contiguous), input gradient (both k-contiguous) and
// weight gradient (both stored with the contraction index as the row).  A k-contiguous operand tile
// is kept in LDS as [rows][64 k] with a 16-byte-chunk XOR swizzle (chunk ^ (row/2)%8: 16 consecutive rows of
// 128 bytes then cover all 64 banks once) and read with ds_read_b128; an
// operand stored with the contraction index as row is kept as [64 k][rows] (padded rows) and read
// with the LDS transpose read ds_read_b64_tr_b16, which hands each lane 4 consecutive k of one row.
// v_mfma_f32_32x32x16_bf16: A lane l holds row l%32, k = 8*(l/32)..+7; B the same with columns;
// accumulator element i of lane l is C[8*(i/4) + 4*(l/32) + i%4][l%32].
#include <type_traits>
#ifdef OASES_GEMM_TUNE_HOOK
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#endif

#include "common.h"

// This file is compiled once per contraction form (OASES_GEMM_PART = 0: NN and the host entry points, 1: NT, 2: TN), so
// that the three sets of kernel instantiations build in parallel; without the macro one object holds everything.
#ifndef OASES_GEMM_PART
#define OASES_GEMM_PART -1
#endif
#define OASES_GEMM_HAS(part) (OASES_GEMM_PART < 0 || OASES_GEMM_PART == (part))

namespace oases {

struct GemmArgs {
  const uint16_t* A;
  const uint16_t* B;
  void* C;
  const float* bias;
  uint16_t* aux;
  int M, N, K;
  int lda, ldb, ldc, ldaux;
  int tiles_m, tiles_n;
  int ksplit, k_per;  // split-K: slice s covers k in [s*k_per, min(K, (s+1)*k_per)) and writes partial s
};

// one launcher per contraction form, each defined in its own part
// choice_rows > 0: the kernel is chosen as if the launch had that many rows (see launch_gemm)
int launch_gemm_nn(const GemmArgs& g, int epi, float* ws, size_t ws_bytes, int forced_variant, int choice_rows, hipStream_t s);
int launch_gemm_nt(const GemmArgs& g, int epi, float* ws, size_t ws_bytes, int forced_variant, int choice_rows, hipStream_t s);
int launch_gemm_tn(const GemmArgs& g, float* ws, size_t ws_bytes, int forced_variant, hipStream_t s);

namespace {

constexpr int BK = 64;          // k extent of one LDS stage
constexpr int kMcPadBytes = 64; // row padding of a "contraction-major" tile (keeps transpose reads off the same banks)


template <int R, bool KC>
struct TileLayout {
  static constexpr int row_bytes = KC ? BK * 2 : R * 2 + kMcPadBytes;
  static constexpr int rows = KC ? R : BK;
  static constexpr int bytes = rows * row_bytes;
  static constexpr int chunks_per_row = KC ? BK / 8 : R / 8;
  static constexpr int chunks = rows * chunks_per_row;
};

// global -> registers for one operand tile.  FULL: the tile lies inside the matrix and the k range inside K,
// so no predicate is needed; otherwise addresses are clamped into the matrix and out-of-range chunks zeroed
// (no divergent branches either way).
template <int R, bool KC, int NT, bool FULL>
__device__ __forceinline__ void load_tile_global(u32x4* regs, const uint16_t* __restrict__ base, int ld, int r0, int k0,
                                                 int rmax, int kmax, int tid) {
  using L = TileLayout<R, KC>;
#pragma unroll
  for (int i = 0; i < L::chunks / NT; i++) {
    int c = tid + i * NT;
    int row = c / L::chunks_per_row, cc = c % L::chunks_per_row;
    int gr, gk;
    if (KC) { gr = r0 + row; gk = k0 + cc * 8; } else { gk = k0 + row; gr = r0 + cc * 8; }
    if (FULL) {
      // uniform base (scalar registers, advanced per k iteration) + one loop-invariant 32-bit lane offset
      static_assert(NT % L::chunks_per_row == 0, "row of a chunk must not depend on the pass");
      constexpr int rows_per_pass = NT / L::chunks_per_row;
      const char* sb = reinterpret_cast<const char*>(base) +
                       ((size_t)(KC ? r0 : k0) * ld + (KC ? k0 : r0) + (size_t)i * rows_per_pass * ld) * 2;
      const uint32_t voff = (uint32_t)(((tid / L::chunks_per_row) * ld + (tid % L::chunks_per_row) * 8) * 2);
      regs[i] = *reinterpret_cast<const u32x4*>(sb + voff);
    } else {
      const bool ok = (gr < rmax) && (gk < kmax);
      const int cr = min(gr, KC ? rmax - 1 : rmax - 8), ck = min(gk, KC ? kmax - 8 : kmax - 1);
      const uint16_t* p = KC ? base + (size_t)cr * ld + ck : base + (size_t)ck * ld + cr;
      u32x4 v = *reinterpret_cast<const u32x4*>(p);
      regs[i] = ok ? v : u32x4{0u, 0u, 0u, 0u};
    }
  }
}

template <int R, bool KC, int NT>
__device__ __forceinline__ void store_tile_lds(const u32x4* regs, char* lds, int tid) {
  using L = TileLayout<R, KC>;
#pragma unroll
  for (int i = 0; i < L::chunks / NT; i++) {
    int c = tid + i * NT;
    int row = c / L::chunks_per_row, cc = c % L::chunks_per_row;
    int off = KC ? row * L::row_bytes + ((cc ^ ((row >> 1) & 7)) << 4) : row * L::row_bytes + (cc << 4);
    *reinterpret_cast<u32x4*>(lds + off) = regs[i];
  }
}

// One 32(row) x 16(k) MFMA operand fragment out of an LDS tile.  r0: first row of the fragment in the
// tile (multiple of 32); kk: which 16-wide k step of the stage.
template <int R, bool KC>
__device__ __forceinline__ bf16x8 read_frag(const char* lds, int r0, int kk, int lane) {
  using L = TileLayout<R, KC>;
  if (KC) {
    int row = r0 + (lane & 31);
    int chunk = kk * 2 + (lane >> 5);
    const char* p = lds + row * L::row_bytes + ((chunk ^ ((lane >> 1) & 7)) << 4);
    return *reinterpret_cast<const bf16x8*>(p);
  } else {
    int krow = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
    int col = r0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const char* p = lds + krow * L::row_bytes + col * 2;
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((OASES_LDS short4v*)(p));
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((OASES_LDS short4v*)(p + 4 * L::row_bytes));
    typedef short short8v __attribute__((ext_vector_type(8)));
    short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

enum { EPI_F32 = 0, EPI_BF16 = 1, EPI_BIAS_BF16 = 2, EPI_BIAS_GELU = 3, EPI_DGELU = 4, EPI_ACC_F32 = 5, EPI_SWIGLU = 6, EPI_DSWIGLU = 7 };

// silu(z) = z * sigmoid(z) and its derivative, on the fast exp2 / rcp units
__device__ __forceinline__ float fast_sigmoid(float z) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z)); }
__device__ __forceinline__ float silu_f(float z) { return z * fast_sigmoid(z); }
__device__ __forceinline__ float silu_grad_f(float z) { const float sg = fast_sigmoid(z); return sg * (1.0f + z * (1.0f - sg)); }

// instruction-group hints for the machine scheduler (kinds: 0x8 MFMA, 0x20 VMEM read, 0x100 LDS read, 0x200 LDS write)
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// Epilogue of one 32 x 32 accumulator tile whose first element is C[row0][col0].  Transposed accumulator (every epilogue
// but the plain fp32 store): element e is C[row][col + (e&3)] with row = row0 + (lane & 31), col = col0 + 8 (e>>2) +
// 4 (lane>>5), so a lane owns 4 consecutive columns.
template <int EPI, bool FULL>
__device__ __forceinline__ void epilogue_tile(const GemmArgs& g, int row0, int col0, int lane, const f32x16& a) {
  if constexpr (EPI == EPI_F32) {
    // element e is C[row0 + 8 (e>>2) + 4 (lane>>5) + (e&3)][col], col = lane & 31 of the tile
    const int col = col0 + (lane & 31);
    if (!FULL && col >= g.N) return;
    float* cbase = reinterpret_cast<float*>(g.C) + col;
#pragma unroll
    for (int e = 0; e < 16; e++) {
      const int row = row0 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
      if (!FULL && row >= g.M) continue;
      float* p = cbase + (size_t)row * g.ldc;
      *p = a[e];
    }
    return;
  }
  const int row = row0 + (lane & 31);
  if (!FULL && row >= g.M) return;
#pragma unroll
  for (int q = 0; q < 4; q++) {
    const int col = col0 + 8 * q + 4 * (lane >> 5);
    if (!FULL && col >= g.N) continue;
    f32x4 v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
    const size_t o = (size_t)row * g.ldc + col;
    if (EPI == EPI_DSWIGLU) {
      // the accumulator holds dF for 4 columns of f; gate and up pre-activations of those columns sit in 32-column
      // blocks side by side in aux ([gate 32 | up 32] per block), and so do their gradients in C
      const size_t cg = (size_t)col + (col & ~31);
      const u32x2 gt = *reinterpret_cast<const u32x2*>(g.aux + (size_t)row * g.ldaux + cg);
      const u32x2 up = *reinterpret_cast<const u32x2*>(g.aux + (size_t)row * g.ldaux + cg + 32);
      float dg[4], du[4];
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const float ge = bf16_bits_to_f32((e & 1) ? gt[e >> 1] >> 16 : gt[e >> 1] & 0xffffu);
        const float ue = bf16_bits_to_f32((e & 1) ? up[e >> 1] >> 16 : up[e >> 1] & 0xffffu);
        dg[e] = v[e] * ue * silu_grad_f(ge);
        du[e] = v[e] * silu_f(ge);
      }
      uint16_t* cp = reinterpret_cast<uint16_t*>(g.C) + (size_t)row * g.ldc + cg;
      *reinterpret_cast<u32x2*>(cp) = u32x2{pack_bf16x2(dg[0], dg[1]), pack_bf16x2(dg[2], dg[3])};
      *reinterpret_cast<u32x2*>(cp + 32) = u32x2{pack_bf16x2(du[0], du[1]), pack_bf16x2(du[2], du[3])};
    } else if (EPI == EPI_F32) {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + o) = v;
    } else if (EPI == EPI_ACC_F32) {
      f32x4* p = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + o);
      *p = *p + v;
    } else {
      uint16_t* cp = reinterpret_cast<uint16_t*>(g.C) + o;
      if (EPI == EPI_BIAS_BF16 || EPI == EPI_BIAS_GELU) v += *reinterpret_cast<const f32x4*>(g.bias + col);
      if (EPI == EPI_BIAS_GELU) {
        *reinterpret_cast<u32x2*>(g.aux + (size_t)row * g.ldaux + col) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] = gelu_tanh(v[e]);
      } else if (EPI == EPI_DGELU) {
        u32x2 x = *reinterpret_cast<const u32x2*>(g.aux + (size_t)row * g.ldaux + col);
        v[0] *= gelu_tanh_grad(bf16_bits_to_f32(x[0] & 0xffffu));
        v[1] *= gelu_tanh_grad(bf16_bits_to_f32(x[0] >> 16));
        v[2] *= gelu_tanh_grad(bf16_bits_to_f32(x[1] & 0xffffu));
        v[3] *= gelu_tanh_grad(bf16_bits_to_f32(x[1] >> 16));
      }
      *reinterpret_cast<u32x2*>(cp) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
    }
  }
}

// SwiGLU: two neighbouring accumulator tiles, gate (first column col0 of the interleaved [gate 32 | up 32] layout) and up,
// hold the same 32 columns of f, element for element
template <bool FULL>
__device__ __forceinline__ void epilogue_tile_swiglu(const GemmArgs& g, int row0, int col0, int lane, const f32x16& ag, const f32x16& au) {
  const int row = row0 + (lane & 31);
  if (!FULL && row >= g.M) return;
#pragma unroll
  for (int q = 0; q < 4; q++) {
    const int cg = col0 + 8 * q + 4 * (lane >> 5);  // gate column in the interleaved [gate 32 | up 32] layout
    if (!FULL && cg >= g.N) continue;
    const int cf = col0 / 2 + 8 * q + 4 * (lane >> 5);
    uint16_t* ap = g.aux + (size_t)row * g.ldaux + cg;
    *reinterpret_cast<u32x2*>(ap) = u32x2{pack_bf16x2(ag[4 * q], ag[4 * q + 1]), pack_bf16x2(ag[4 * q + 2], ag[4 * q + 3])};
    *reinterpret_cast<u32x2*>(ap + 32) = u32x2{pack_bf16x2(au[4 * q], au[4 * q + 1]), pack_bf16x2(au[4 * q + 2], au[4 * q + 3])};
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; e++) f[e] = silu_f(ag[4 * q + e]) * au[4 * q + e];
    *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(g.C) + (size_t)row * g.ldc + cf) = u32x2{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3])};
  }
}

// Waves of a workgroup form a WGM x WGN x WGK grid: a wave owns a (BM/WGM) x (BN/WGN) part of the block tile and,
// when WGK > 1, every WGK-th pair of the 16-wide k steps of each stage; the WGK partial accumulators of a part are
// added through LDS after the k loop, in a fixed order.  Splitting k inside the workgroup instead of the tile keeps
// the wave tile at 128 x 128 for the rectangular block tiles, which is what bounds the LDS bytes read per MFMA.
template <int BM, int BN, int WGM, int WGN, int WGK, bool A_KC, bool B_KC, int EPI, bool FULL>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, char* lds, int m0, int n0) {
  constexpr int NT = 64 * WGM * WGN * WGK;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int KS = (BK / 16) / WGK;  // k steps of one stage that a wave multiplies
  static_assert(WGK == 1 || (KS == 2 && TM * TN >= 16), "k split inside the workgroup: two steps per wave, deep pipeline");
  using LA = TileLayout<BM, A_KC>;
  using LB = TileLayout<BN, B_KC>;
  constexpr int NA = LA::chunks / NT, NB = LB::chunks / NT;
  constexpr int kStage = LA::bytes + LB::bytes;  // stage s: A at lds + s*kStage, B behind it
  constexpr int NREAD = TM * (A_KC ? 1 : 2) + TN * (B_KC ? 1 : 2);  // LDS reads of one 16-wide k step
  constexpr int NMFMA = TM * TN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wk = wave / (WGM * WGN), wm = (wave / WGN) % WGM, wn = wave % WGN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  u32x4 ra[NA], rb[NB];
  bf16x8 fa[2][TM], fb[2][TN];
  const int nk = (g.K + BK - 1) / BK;

  auto fetch_a = [&](int kt) { load_tile_global<BM, A_KC, NT, FULL>(ra, g.A, g.lda, m0, kt * BK, g.M, g.K, tid); };
  auto fetch_b = [&](int kt) { load_tile_global<BN, B_KC, NT, FULL>(rb, g.B, g.ldb, n0, kt * BK, g.N, g.K, tid); };
  auto park_a = [&](int stage) { store_tile_lds<BM, A_KC, NT>(ra, lds + stage * kStage, tid); };
  auto park_b = [&](int stage) { store_tile_lds<BN, B_KC, NT>(rb, lds + stage * kStage + LA::bytes, tid); };
  auto frags = [&](int stage, int kk, int buf) {
    const char* la = lds + stage * kStage;
    const char* lb = la + LA::bytes;
#pragma unroll
    for (int i = 0; i < TM; i++) fa[buf][i] = read_frag<BM, A_KC>(la, wm * WTM + i * 32, wk * KS + kk, lane);
#pragma unroll
    for (int j = 0; j < TN; j++) fb[buf][j] = read_frag<BN, B_KC>(lb, wn * WTN + j * 32, wk * KS + kk, lane);
  };
  // the B fragment is the first MFMA operand: the accumulator then holds C^T, i.e. a lane owns 4 consecutive
  // columns of one row of C per group of four accumulator elements (16-byte stores in the epilogue)
  // ROWMAJ (plain fp32 output): the A fragment goes first instead and the accumulator holds C itself -- a lane owns
  // one column, 32 lanes one 128-byte row segment, so that every epilogue store writes whole cache lines (measured:
  // up to 18 % on short-k launches whose time is mostly the fp32 output).  Not for the accumulating epilogue, whose
  // read-modify-write wants the 16-byte accesses.
  constexpr bool ROWMAJ = EPI == EPI_F32;
  auto mma = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        if constexpr (ROWMAJ) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
        else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
      }
  };
  // one 16-wide k step: LDS reads of the next step interleaved one-for-one with this step's MFMAs
  auto hint_step = [&]() {
    constexpr int PER = (NREAD + NMFMA - 1) / NMFMA;
#pragma unroll
    for (int i = 0; i < NMFMA; i++) {
      SGB(0x008, 1);
      SGB(0x100, PER);
    }
  };

  if constexpr (TM * TN >= 16) {
    // Pipeline.  While tile kt is multiplied out of stage kt&1, tile kt+1 sits in the other stage.  One operand's half
    // of tile kt+2 is written into stage kt&1 right behind the barrier of iteration kt (which releases that stage),
    // the other's during the first k step of iteration kt+1; each half's registers are refilled from global memory
    // right behind its LDS store, a whole iteration ahead of the next store.  LDS stores and global loads are thus
    // spread over two k steps and never wait at the top of the loop.
    // "early" half: stored during the first k step, "late" half: stored behind the barrier, where it competes with the
    // first fragment reads of the next stage -- the smaller operand tile goes there.
    constexpr bool LATE_A = BM <= BN;
    constexpr int N_EARLY = LATE_A ? NB : NA, N_LATE = LATE_A ? NA : NB;
    auto fetch_early = [&](int kt) { if constexpr (LATE_A) fetch_b(kt); else fetch_a(kt); };
    auto fetch_late = [&](int kt) { if constexpr (LATE_A) fetch_a(kt); else fetch_b(kt); };
    auto park_early = [&](int stage) { if constexpr (LATE_A) park_b(stage); else park_a(stage); };
    auto park_late = [&](int stage) { if constexpr (LATE_A) park_a(stage); else park_b(stage); };
    fetch_a(0);
    fetch_b(0);
    park_a(0);
    park_b(0);
    if (nk > 1) { fetch_late(1); park_late(1); fetch_early(1); }
    if (nk > 2) fetch_late(2);
    __syncthreads();
    frags(0, 0, 0);

    // one 64-wide k iteration; M1/M2/M3: tile kt+1 / kt+2 / kt+3 exists.  The steady state (all true) is branch-free
    // so that the scheduler sees one block per iteration.
    auto iteration = [&](auto m1_c, auto m2_c, auto m3_c, int kt) {
      constexpr bool M1 = decltype(m1_c)::value, M2 = decltype(m2_c)::value, M3 = decltype(m3_c)::value;
      const int cur = kt & 1;
      if (M1) park_early(cur ^ 1);  // early half of tile kt+1 (the stage was released by the previous barrier)
      if (M2) fetch_early(kt + 2);
      frags(cur, 1, 1);
      mma(0);
  #pragma unroll
      for (int i = 0; i < NMFMA; i++) {
        SGB(0x008, 1);
        SGB(0x100, (NREAD + NMFMA - 1) / NMFMA);
        if (M1) SGB(0x200, (N_EARLY + NMFMA - 1) / NMFMA);
        if (M2) SGB(0x020, (N_EARLY + NMFMA - 1) / NMFMA);
      }
      if (KS == 4) {
        frags(cur, 2, 0);
        mma(1);
        hint_step();
        frags(cur, 3, 1);
        mma(0);
        hint_step();
      }
      // every wave has its last fragments of stage `cur` in registers, and stage cur^1 (tile kt+1) is complete
      __syncthreads();
      if (M1) frags(cur ^ 1, 0, 0);
      if (M2) park_late(cur);       // late half of tile kt+2 -> the stage just released
      if (M3) fetch_late(kt + 3);
      mma(1);
  #pragma unroll
      for (int i = 0; i < NMFMA; i++) {
        SGB(0x008, 1);
        if (M1) SGB(0x100, (NREAD + NMFMA - 1) / NMFMA);
        if (M2) SGB(0x200, (N_LATE + NMFMA - 1) / NMFMA);
        if (M3) SGB(0x020, (N_LATE + NMFMA - 1) / NMFMA);
      }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    int kt = 0;
    for (; kt + 3 < nk; kt++) iteration(T_{}, T_{}, T_{}, kt);
    if (kt + 2 < nk) { iteration(T_{}, T_{}, F_{}, kt); kt++; }
    if (kt + 1 < nk) { iteration(T_{}, F_{}, F_{}, kt); kt++; }
    iteration(F_{}, F_{}, F_{}, kt);
  } else {
    // Pipeline for the smaller tiles (their LDS traffic per MFMA is higher; a single burst of LDS stores at the top of
    // the iteration disturbs the fragment reads least): tile kt+1 waits in registers, is stored into the other stage
    // at the top of iteration kt, and the registers are refilled with tile kt+2 right behind.
    fetch_a(0);
    fetch_b(0);
    park_a(0);
    park_b(0);
    if (nk > 1) { fetch_a(1); fetch_b(1); }
    __syncthreads();
    frags(0, 0, 0);
    auto iteration = [&](auto m1_c, auto m2_c, int kt) {
      constexpr bool M1 = decltype(m1_c)::value, M2 = decltype(m2_c)::value;
      const int cur = kt & 1;
      if (M1) { park_a(cur ^ 1); park_b(cur ^ 1); }
      if (M2) { fetch_a(kt + 2); fetch_b(kt + 2); }
      frags(cur, 1, 1);
      mma(0);
      if (M1) SGB(0x200, NA + NB);
  #pragma unroll
      for (int i = 0; i < NMFMA; i++) {
        SGB(0x008, 1);
        if (M2) SGB(0x020, (NA + NB + NMFMA - 1) / NMFMA);
        SGB(0x100, (NREAD + NMFMA - 1) / NMFMA);
      }
      frags(cur, 2, 0);
      mma(1);
      hint_step();
      frags(cur, 3, 1);
      mma(0);
      hint_step();
      __syncthreads();
      if (M1) frags(cur ^ 1, 0, 0);
      mma(1);
      hint_step();
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    int kt = 0;
    for (; kt + 2 < nk; kt++) iteration(T_{}, T_{}, kt);
    if (kt + 1 < nk) { iteration(T_{}, F_{}, kt); kt++; }
    iteration(F_{}, F_{}, kt);
  }

  auto emit = [&](int i, int j, const f32x16& a) { epilogue_tile<EPI, FULL>(g, m0 + wm * WTM + i * 32, n0 + wn * WTN + j * 32, lane, a); };
  auto emit_pair = [&](int i, int jj, const f32x16& ag, const f32x16& au) {
    epilogue_tile_swiglu<FULL>(g, m0 + wm * WTM + i * 32, n0 + wn * WTN + jj * 64, lane, ag, au);
  };

  static_assert(TN % 2 == 0, "tiles of a wave are finished in pairs");
  if constexpr (WGK == 1) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
        if constexpr (EPI == EPI_SWIGLU) {
          emit_pair(i, j / 2, acc[i][j], acc[i][j + 1]);
        } else {
          emit(i, j, acc[i][j]);
          emit(i, j + 1, acc[i][j + 1]);
        }
      }
  } else {
    // The two waves that hold the k halves of one part each finish one half of its rows: a wave hands the
    // accumulator tiles of the other half over through LDS (lane-for-lane, 16 bytes per lane and store) and adds what
    // it receives to its own; the sum of two terms does not depend on which of them is "own".
    static_assert(WGK == 2 && TM % 2 == 0, "pairwise exchange");
    constexpr int HM = TM / 2;
    f32x4* xch = reinterpret_cast<f32x4*>(lds);
    const int mine = wave * (HM * TN * 4), theirs = (wave ^ (WGM * WGN)) * (HM * TN * 4);
    __syncthreads();  // every wave is done with the operand stages
    auto hand_over = [&](auto half_c) {  // half_c: which half of the tile rows leaves this wave
      constexpr int H = decltype(half_c)::value;
#pragma unroll
      for (int i = 0; i < HM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const f32x16& a = acc[H * HM + i][j];
            xch[(mine + (i * TN + j) * 4 + q) * 64 + lane] = f32x4{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
          }
    };
    auto finish = [&](auto half_c) {  // half_c: which half of the tile rows this wave keeps
      constexpr int H = decltype(half_c)::value;
#pragma unroll
      for (int i = 0; i < HM; i++)
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
          f32x16 a[2] = {acc[H * HM + i][j], acc[H * HM + i][j + 1]};
#pragma unroll
          for (int t = 0; t < 2; t++)
#pragma unroll
            for (int q = 0; q < 4; q++) {
              const f32x4 o = xch[(theirs + (i * TN + j + t) * 4 + q) * 64 + lane];
#pragma unroll
              for (int e = 0; e < 4; e++) a[t][4 * q + e] += o[e];
            }
          if constexpr (EPI == EPI_SWIGLU) {
            emit_pair(H * HM + i, j / 2, a[0], a[1]);
          } else {
            emit(H * HM + i, j, a[0]);
            emit(H * HM + i, j + 1, a[1]);
          }
        }
    };
    if (wk == 0) hand_over(std::integral_constant<int, 1>{}); else hand_over(std::integral_constant<int, 0>{});
    __syncthreads();
    if (wk == 0) finish(std::integral_constant<int, 0>{}); else finish(std::integral_constant<int, 1>{});
  }
}

// workgroup id within a launch of tiles_m x tiles_n tiles -> tile: undo the round-robin of workgroup ids over the 8 XCDs so
// that each XCD's L2 sees a contiguous range of tiles, then walk that range in groups of 8 tile rows
__device__ __forceinline__ void tile_of_workgroup(int pid, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  const int T = tiles_m * tiles_n;
  const int per = (T + 7) / 8, tall = (T % 8 == 0) ? 8 : T % 8;
  const int xcd = pid & 7, local = pid >> 3;
  const int logical = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
  constexpr int GM = 8;
  const int width = GM * tiles_n;
  const int group = logical / width, first_m = group * GM;
  const int gsz = min(tiles_m - first_m, GM);
  tile_m = first_m + (logical % width) % gsz;
  tile_n = (logical % width) / gsz;
}

template <int BM, int BN, int WGM, int WGN, int WGK, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN * WGK) void gemm_kernel(GemmArgs g) {  // g: by value, adjusted per k slice
  using LA = TileLayout<BM, A_KC>;
  using LB = TileLayout<BN, B_KC>;
  constexpr int kStages = 2 * (LA::bytes + LB::bytes);
  constexpr int kExchange = WGK > 1 ? BM * BN * 4 : 0;  // half of every wave's accumulator
  __shared__ __attribute__((aligned(16))) char lds[kStages > kExchange ? kStages : kExchange];

  // workgroup -> (k slice, tile)
  int tile_m, tile_n;
  const int T = g.tiles_m * g.tiles_n;
  const int slice = blockIdx.x / T;
  tile_of_workgroup(blockIdx.x - slice * T, g.tiles_m, g.tiles_n, tile_m, tile_n);
  if (g.ksplit > 1) {  // this workgroup's k range and partial-result plane
    const int k0 = slice * g.k_per;
    g.A += A_KC ? (size_t)k0 : (size_t)k0 * g.lda;
    g.B += B_KC ? (size_t)k0 : (size_t)k0 * g.ldb;
    g.K = min(g.K - k0, g.k_per);
    g.C = reinterpret_cast<float*>(g.C) + (size_t)slice * g.M * g.ldc;
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const bool full = (m0 + BM <= g.M) && (n0 + BN <= g.N) && (g.K % BK == 0);
  if (full) gemm_tile<BM, BN, WGM, WGN, WGK, A_KC, B_KC, EPI, true>(g, lds, m0, n0);
  else gemm_tile<BM, BN, WGM, WGN, WGK, A_KC, B_KC, EPI, false>(g, lds, m0, n0);
}

// =================================================================================================
// 256 x 256 tiles fed by direct-to-LDS loads (global_load_lds_dwordx4): no staging registers, four LDS stages of 32 k,
// three tiles (96 KB per CU) in flight.  The compiler would put s_waitcnt vmcnt(0) in front of every LDS read that
// might alias a pending LDS DMA, so the fragment reads are inline assembly and every wait is placed by hand:
//   vmcnt  -- DMA instructions complete in order, 8 per wave and tile: "tile t has landed" = at most 8 x (younger tiles
//             in flight) outstanding, then the workgroup barrier makes all four waves' parts visible;
//   lgkmcnt -- LDS reads return in order: fragments of the first k step are waited for with the second step's reads
//             still outstanding; the second step's are waited for before the barrier, so that a stage is never
//             refilled while a wave still reads it.
// K must be a whole number of 32-wide stages and there are no k slices; M and N may end inside a tile where the operand
// is row-indexed (see dtl_src); everything else runs on the kernels above.
// =================================================================================================
#ifndef OASES_DTL_STAGES
#define OASES_DTL_STAGES 4
#endif
constexpr int BKD = 32, NSD = OASES_DTL_STAGES;
constexpr int kDtlOperand = 256 * BKD * 2;  // bytes of one operand tile
constexpr int kDtlStage = 2 * kDtlOperand;

template <int OFF>
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ u32x2 lds_read_tr16_b64(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
// the eight fragments of one k step become valid: at most N younger LDS reads may still be outstanding
template <int N>
__device__ __forceinline__ void lds_wait(u32x4 (&a)[4], u32x4 (&b)[4]) {
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3])
               : "n"(N));
}

// Operand tile in LDS.  KC (k contiguous in memory): [256 rows][32 k] = 64-byte rows, 16-byte chunk c of row r at slot
// c ^ ((r/4)%4) (16 consecutive rows at one chunk then cover all 64 banks).  MC (row index contiguous in memory):
// [32 k][256 rows] = 512-byte k rows, chunk c of k row kr at slot c ^ 4*(kr%4) (the 4 k rows x 64 bytes that 32 lanes of
// a transpose read touch in one LDS cycle then fall on 16 different chunk positions mod 16).  One DMA instruction of a wave writes 1 KB
// of the tile, lane i the 16 bytes at i*16: the swizzle is applied to the global address the lane fetches.
// `extent`: rows of the operand's free dimension (M of A, N of B).  A row-indexed operand may end inside the tile
// (extent a multiple of 8, so whole 16-byte chunks): chunks beyond it are fetched from column 0 instead -- valid memory,
// and the rows / columns of C they feed are never stored.  A k-major operand must fill its tiles.
//
// The eight-wave kernels fetch the tiles with buffer loads (resource in SGPRs + 32-bit lane offset + SGPR tile offset)
// straight into LDS: no address arithmetic in the vector ALU and half the address registers; measured 5-10 % faster
// there than global_load_lds with 64-bit lane addresses (TN 2048 x 4096 x 8192: 1029 -> 1120 TFLOP/s, 4096 x 4096 x
// 8192: 1111 -> 1228).  An operand must span less than 2 GiB (gemm_span_fits, checked by the launcher).
typedef void OASES_LDS* lds_ptr_t;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ uint32_t lane_offset(const char* p, const void* base) { return (uint32_t)(p - reinterpret_cast<const char*>(base)); }
// 16 bytes per lane: lane i's go to dst + 16 i (dst is uniform over the wave)
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t tile_off, char* dst) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)dst, 16, (int)lane_off, (int)tile_off, 0, 0);
}

// the same through global_load_lds (64-bit lane address): what the four-wave kernels use -- they issue a tile's loads between
// MFMAs of the same wave, where the buffer form measured 5-10 % slower
__device__ __forceinline__ void dma16_global(const void* base, uint32_t lane_off, uint32_t tile_off, char* dst) {
  typedef const void __attribute__((address_space(1))) * gptr_t;
  __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char*>(base) + lane_off + (size_t)tile_off), (lds_ptr_t)dst, 16, 0, 0);
}

template <bool KC>
__device__ __forceinline__ const char* dtl_src(const uint16_t* base, int ld, int r0, int q, int lane, int extent) {
  if (KC) {
    const int row = 16 * q + (lane >> 2), chunk = (lane & 3) ^ ((row >> 2) & 3);
    return reinterpret_cast<const char*>(base + (size_t)(r0 + row) * ld + chunk * 8);
  }
  const int kr = 2 * q + (lane >> 5), cc = (lane & 31) ^ (4 * (kr & 3));
  int col = r0 + cc * 8;
  if (col >= extent) col = 0;
  return reinterpret_cast<const char*>(base + (size_t)kr * ld + col);
}
// per-lane LDS offsets of the fragment reads of a wave's 128-row part starting at tile row R0
template <bool KC>
__device__ __forceinline__ void dtl_frag_offsets(uint32_t* off, int R0, int lane) {
  if (KC) {  // off[kk]: fragment i adds 32 rows = 2048 bytes
#pragma unroll
    for (int kk = 0; kk < 2; kk++) {
      const int row = R0 + (lane & 31), chunk = kk * 2 + (lane >> 5);
      off[kk] = (uint32_t)(row * 64 + 16 * (chunk ^ ((row >> 2) & 3)));
    }
  } else {  // off[i]: k step kk adds 16 k rows = 8192 bytes, the second half of the fragment 4 k rows = 2048 bytes
    const int krow = 8 * (lane >> 5) + ((lane & 15) >> 2);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int col = R0 + 32 * i + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      off[i] = (uint32_t)(krow * 512 + (((col >> 3) ^ (4 * (krow & 3))) << 4) + (col & 7) * 2);
    }
  }
}
template <bool KC, int KK>
__device__ __forceinline__ void dtl_read_frags(u32x4 (&f)[4], uint32_t base, const uint32_t* off) {
  if constexpr (KC) {
    const uint32_t a = base + off[KK];
    f[0] = lds_read_b128<0>(a);
    f[1] = lds_read_b128<2048>(a);
    f[2] = lds_read_b128<4096>(a);
    f[3] = lds_read_b128<6144>(a);
  } else {
#define OASES_TR(i)                                                         \
  {                                                                         \
    const u32x2 lo = lds_read_tr16_b64<KK * 8192>(base + off[i]);           \
    const u32x2 hi = lds_read_tr16_b64<KK * 8192 + 2048>(base + off[i]);    \
    f[i] = u32x4{lo[0], lo[1], hi[0], hi[1]};                               \
  }
    OASES_TR(0) OASES_TR(1) OASES_TR(2) OASES_TR(3)
#undef OASES_TR
  }
}

template <bool A_KC, bool B_KC, int EPI, bool FULL>
__global__ __launch_bounds__(256) void gemm_dtl_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(1024))) char lds[NSD * kDtlStage];
  int tile_m, tile_n;
  tile_of_workgroup(blockIdx.x, g.tiles_m, g.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * 256, n0 = tile_n * 256;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;
  constexpr int WGM = 2, WGN = 2, WTM = 128, WTN = 128, TM = 4, TN = 4;
  const int nk = g.K / BKD;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // DMA sources of this lane: instruction j of this wave is instruction q = 4*wave + j of the operand tile
  // (the swizzle of an MC tile depends on the parity of q: one source pointer for even, one for odd instructions)
  const uint32_t srcA[2] = {lane_offset(dtl_src<A_KC>(g.A, g.lda, m0, 4 * wave, lane, g.M), g.A), lane_offset(dtl_src<A_KC>(g.A, g.lda, m0, 4 * wave + 1, lane, g.M), g.A)};
  const uint32_t srcB[2] = {lane_offset(dtl_src<B_KC>(g.B, g.ldb, n0, 4 * wave, lane, g.N), g.B), lane_offset(dtl_src<B_KC>(g.B, g.ldb, n0, 4 * wave + 1, lane, g.N), g.B)};
  const uint32_t stepA_q = A_KC ? 32u * g.lda * 2 : 4u * g.lda * 2;   // two instructions on: 32 rows resp. 4 k rows
  const uint32_t stepB_q = B_KC ? 32u * g.ldb * 2 : 4u * g.ldb * 2;
  const uint32_t stepA_k = A_KC ? (uint32_t)BKD * 2 : (uint32_t)BKD * g.lda * 2;          // next k tile
  const uint32_t stepB_k = B_KC ? (uint32_t)BKD * 2 : (uint32_t)BKD * g.ldb * 2;
  auto issue = [&](int t) {
    char* st = lds + (t % NSD) * kDtlStage + wave * 4096;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      dma16_global(g.A, srcA[j & 1], (uint32_t)t * stepA_k + (j >> 1) * stepA_q, st + j * 1024);
      dma16_global(g.B, srcB[j & 1], (uint32_t)t * stepB_k + (j >> 1) * stepB_q, st + kDtlOperand + j * 1024);
    }
  };

  uint32_t offA[4], offB[4];
  dtl_frag_offsets<A_KC>(offA, wm * WTM, lane);
  dtl_frag_offsets<B_KC>(offB, wn * WTN, lane);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(OASES_LDS char*)lds;
  u32x4 fa[2][4], fb[2][4];
  constexpr int NRA = A_KC ? 4 : 8, NRB = B_KC ? 4 : 8, NR = NRA + NRB > 15 ? 15 : NRA + NRB;  // reads of one k step (lgkmcnt saturates at 15)
  auto mma = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, fa[buf][i]), b = __builtin_bit_cast(bf16x8, fb[buf][j]);
        if constexpr (EPI == EPI_F32) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
        else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[i][j], 0, 0, 0);
      }
  };
  // s_waitcnt vmcnt(n) only.  Steady state: NSD-2 younger tiles of 8 DMA instructions each may still be in flight
  constexpr int kYoung = 8 * (NSD - 2);
  constexpr int kVm16 = ((kYoung >> 4) << 14) | (kYoung & 15) | (7 << 4) | (15 << 8), kVm0 = (7 << 4) | (15 << 8);

#pragma unroll
  for (int t = 0; t < NSD - 1; t++)
    if (t < nk) issue(t);
  if (nk > NSD - 2) __builtin_amdgcn_s_waitcnt(kVm16); else __builtin_amdgcn_s_waitcnt(kVm0);
  __builtin_amdgcn_s_barrier();
  dtl_read_frags<A_KC, 0>(fa[0], lds0, offA);
  dtl_read_frags<B_KC, 0>(fb[0], lds0 + kDtlOperand, offB);

  // one 32-wide k tile.  STEADY: tile kt+NSD-1 exists and is requested now (its stage held tile kt-1; a wave passes the
  // barrier of an iteration only after all its reads of that iteration's tile have returned), so NSD-2 younger tiles
  // are in flight when tile kt+1 must have landed; NEXT: tile kt+1 exists.
  uint32_t cur = lds0;
  auto iteration = [&](auto steady_c, auto next_c, int kt) {
    constexpr bool STEADY = decltype(steady_c)::value, NEXT = decltype(next_c)::value;
    const uint32_t nxt = cur + kDtlStage == lds0 + NSD * kDtlStage ? lds0 : cur + kDtlStage;
    dtl_read_frags<A_KC, 1>(fa[1], cur, offA);
    dtl_read_frags<B_KC, 1>(fb[1], cur + kDtlOperand, offB);
    lds_wait<NR>(fa[0], fb[0]);
    if (STEADY) issue(kt + NSD - 1);
    mma(0);
    lds_wait<0>(fa[1], fb[1]);  // requested before the MFMAs above; with it every read this wave makes of tile kt is complete
    if (NEXT) {
      if (STEADY) __builtin_amdgcn_s_waitcnt(kVm16); else __builtin_amdgcn_s_waitcnt(kVm0);  // own part of tile kt+1 has landed
      __builtin_amdgcn_s_barrier();  // tile kt+1 is visible to every wave, and no wave reads tile kt any more
      dtl_read_frags<A_KC, 0>(fa[0], nxt, offA);
      dtl_read_frags<B_KC, 0>(fb[0], nxt + kDtlOperand, offB);
    }
    mma(1);
    cur = nxt;
  };
  {
    using T_ = std::true_type;
    using F_ = std::false_type;
    int kt = 0;
    for (; kt + NSD - 1 < nk; kt++) iteration(T_{}, T_{}, kt);
    for (; kt + 1 < nk; kt++) iteration(F_{}, T_{}, kt);
    iteration(F_{}, F_{}, kt);
  }
  auto emit = [&](int i, int j, const f32x16& a) { epilogue_tile<EPI, FULL>(g, m0 + wm * WTM + i * 32, n0 + wn * WTN + j * 32, lane, a); };
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j += 2) {
      if constexpr (EPI == EPI_SWIGLU) {  // tiles j (gate) and j+1 (up) of the interleaved 64-column blocks
        epilogue_tile_swiglu<FULL>(g, m0 + wm * WTM + i * 32, n0 + wn * WTN + j * 32, lane, acc[i][j], acc[i][j + 1]);
      } else {
        emit(i, j, acc[i][j]);
        emit(i, j + 1, acc[i][j + 1]);
      }
    }
}

// =================================================================================================
// 128 x 256 tiles fed by direct-to-LDS loads.  Three LDS stages of 64 k (48 KB each); the two wave pairs split the four
// 16-wide k steps of a stage between them, so a wave keeps the 128 x 128 accumulator of the square kernel (same LDS
// bytes read per MFMA) while the launch has twice as many workgroups; the two partial sums of a part meet once,
// through LDS, after the k loop.  Waits as in the kernel above; a wave issues 12 DMA instructions per tile (4 of A,
// 8 of B).  K % 64 == 0; M and N may end inside a tile (see rect_src).
// Operand tile in LDS.  KC: [R rows][64 k] = 128-byte rows, chunk c of row r at slot c ^ ((r/2)%8) (16 consecutive
// rows at one chunk cover all 64 banks); one DMA instruction covers 8 rows.  MC: [64 k][R rows], k row = 2R bytes,
// chunk c of k row kr at slot c ^ 4*(kr%4); one DMA instruction covers 512/R k rows.  In both the swizzle of
// instruction q depends on the parity of q only.
// =================================================================================================
constexpr int BKR = 64, NSR = 3;
constexpr int kRectA = BKR * 128 * 2, kRectB = BKR * 256 * 2, kRectStage = kRectA + kRectB;

template <bool KC, int R>
__device__ __forceinline__ const char* rect_src(const uint16_t* base, int ld, int r0, int q, int lane, int extent) {
  if (KC) {  // rows beyond the operand's extent: the last row again (valid memory; what they feed is never stored)
    const int row = 8 * q + (lane >> 3), chunk = (lane & 7) ^ ((row >> 1) & 7);
    return reinterpret_cast<const char*>(base + (size_t)min(r0 + row, extent - 1) * ld + chunk * 8);
  }
  constexpr int CPR = R / 8, KPI = 64 / CPR;
  const int kr = KPI * q + lane / CPR, cc = (lane % CPR) ^ (4 * (kr & 3));
  int col = r0 + cc * 8;
  if (col >= extent) col = 0;  // beyond a row-indexed operand's extent: see dtl_src
  return reinterpret_cast<const char*>(base + (size_t)kr * ld + col);
}
// per-lane LDS offsets of the fragment reads of a wave's 128-row part starting at tile row R0, for the k half wk of a
// tile.  KC: off[kk], k step kk of the half (fragment i adds 32 rows = 4096 bytes); MC: off[i], fragment i (k step kk
// adds 16 k rows, the second half of a fragment 4 k rows).
template <bool KC, int R>
__device__ __forceinline__ void rect_frag_offsets(uint32_t* off, int R0, int wk, int lane) {
  if (KC) {
#pragma unroll
    for (int kk = 0; kk < 2; kk++) {
      const int row = R0 + (lane & 31), chunk = 4 * wk + 2 * kk + (lane >> 5);
      off[kk] = (uint32_t)(row * 128 + 16 * (chunk ^ ((row >> 1) & 7)));
    }
  } else {
    const int krow = 32 * wk + 8 * (lane >> 5) + ((lane & 15) >> 2);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int col = R0 + 32 * i + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      off[i] = (uint32_t)(krow * (2 * R) + (((col >> 3) ^ (4 * (krow & 3))) << 4) + (col & 7) * 2);
    }
  }
}
template <bool KC, int R, int KK>
__device__ __forceinline__ void rect_read_frags(u32x4 (&f)[4], uint32_t base, const uint32_t* off) {
  if constexpr (KC) {
    const uint32_t a = base + off[KK];
    f[0] = lds_read_b128<0>(a);
    f[1] = lds_read_b128<4096>(a);
    f[2] = lds_read_b128<8192>(a);
    f[3] = lds_read_b128<12288>(a);
  } else {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const u32x2 lo = lds_read_tr16_b64<KK * 16 * 2 * R>(base + off[i]);
      const u32x2 hi = lds_read_tr16_b64<KK * 16 * 2 * R + 4 * 2 * R>(base + off[i]);
      f[i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
    }
  }
}

constexpr int kRectExchange = 128 * 256 * 4;
constexpr int kRectLds = NSR * kRectStage > kRectExchange ? NSR * kRectStage : kRectExchange;

// one 128 x 256 tile: workgroup `pid` of the tiles_m x tiles_n tiles of problem g; lds: kRectLds bytes, 1024-byte aligned
template <bool A_KC, bool B_KC, int EPI, bool FULL>
__device__ __forceinline__ void dtl_rect_tile(const GemmArgs& g, int pid, char* lds) {
  int tile_m, tile_n;
  tile_of_workgroup(pid, g.tiles_m, g.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * 128, n0 = tile_n * 256;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wn = wave & 1, wk = wave >> 1;
  constexpr int TM = 4, TN = 4;
  const int nk = g.K / BKR;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // this wave's DMA instructions of a tile: A instructions 4*wave .. 4*wave+3, B instructions 8*wave .. 8*wave+7, one
  // source pointer each (rows or chunks beyond an operand's extent are redirected per instruction)
  uint32_t srcA[4], srcB[8];
#pragma unroll
  for (int j = 0; j < 4; j++) srcA[j] = lane_offset(rect_src<A_KC, 128>(g.A, g.lda, m0, 4 * wave + j, lane, g.M), g.A);
#pragma unroll
  for (int j = 0; j < 8; j++) srcB[j] = lane_offset(rect_src<B_KC, 256>(g.B, g.ldb, n0, 8 * wave + j, lane, g.N), g.B);
  const uint32_t stepA_k = A_KC ? (uint32_t)BKR * 2 : (uint32_t)BKR * g.lda * 2, stepB_k = B_KC ? (uint32_t)BKR * 2 : (uint32_t)BKR * g.ldb * 2;  // next k tile
  auto issue = [&](int t) {
    char* st = lds + (t % NSR) * kRectStage;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      dma16_global(g.A, srcA[j], (uint32_t)t * stepA_k, st + (4 * wave + j) * 1024);
      dma16_global(g.B, srcB[2 * j], (uint32_t)t * stepB_k, st + kRectA + (8 * wave + 2 * j) * 1024);
      dma16_global(g.B, srcB[2 * j + 1], (uint32_t)t * stepB_k, st + kRectA + (8 * wave + 2 * j + 1) * 1024);
    }
  };

  uint32_t offA[4], offB[4];
  rect_frag_offsets<A_KC, 128>(offA, 0, wk, lane);
  rect_frag_offsets<B_KC, 256>(offB, wn * 128, wk, lane);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(OASES_LDS char*)lds;
  u32x4 fa[2][4], fb[2][4];
  auto mma = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, fa[buf][i]), b = __builtin_bit_cast(bf16x8, fb[buf][j]);
        if constexpr (EPI == EPI_F32) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
        else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[i][j], 0, 0, 0);
      }
  };
  constexpr int kYoung = 12 * (NSR - 2);  // DMA instructions of the younger tiles that may still be in flight
  constexpr int kVmSteady = ((kYoung >> 4) << 14) | (kYoung & 15) | (7 << 4) | (15 << 8), kVm0 = (7 << 4) | (15 << 8);
  constexpr int NRA = A_KC ? 4 : 8, NRB = B_KC ? 4 : 8, NR = NRA + NRB > 15 ? 15 : NRA + NRB;  // reads of one k step (the counter saturates at 15)

#pragma unroll
  for (int t = 0; t < NSR - 1; t++)
    if (t < nk) issue(t);
  if (nk > NSR - 2) __builtin_amdgcn_s_waitcnt(kVmSteady); else __builtin_amdgcn_s_waitcnt(kVm0);
  __builtin_amdgcn_s_barrier();
  rect_read_frags<A_KC, 128, 0>(fa[0], lds0, offA);
  rect_read_frags<B_KC, 256, 0>(fb[0], lds0 + kRectA, offB);

  uint32_t cur = lds0;
  auto iteration = [&](auto steady_c, auto next_c, int kt) {
    constexpr bool STEADY = decltype(steady_c)::value, NEXT = decltype(next_c)::value;
    const uint32_t nxt = cur + kRectStage == lds0 + NSR * kRectStage ? lds0 : cur + kRectStage;
    rect_read_frags<A_KC, 128, 1>(fa[1], cur, offA);
    rect_read_frags<B_KC, 256, 1>(fb[1], cur + kRectA, offB);
    lds_wait<NR>(fa[0], fb[0]);
    if (STEADY) issue(kt + NSR - 1);  // into the stage of tile kt-1: its reads had returned before any wave passed the last barrier
    mma(0);
    lds_wait<0>(fa[1], fb[1]);  // requested before the MFMAs above; with it every read this wave makes of tile kt is complete
    if (NEXT) {
      if (STEADY) __builtin_amdgcn_s_waitcnt(kVmSteady); else __builtin_amdgcn_s_waitcnt(kVm0);  // own part of tile kt+1 has landed
      __builtin_amdgcn_s_barrier();  // tile kt+1 is visible to every wave, and no wave reads tile kt any more
      rect_read_frags<A_KC, 128, 0>(fa[0], nxt, offA);
      rect_read_frags<B_KC, 256, 0>(fb[0], nxt + kRectA, offB);
    }
    mma(1);
    cur = nxt;
  };
  {
    using T_ = std::true_type;
    using F_ = std::false_type;
    int kt = 0;
    for (; kt + NSR - 1 < nk; kt++) iteration(T_{}, T_{}, kt);
    for (; kt + 1 < nk; kt++) iteration(F_{}, T_{}, kt);
    iteration(F_{}, F_{}, kt);
  }

  // The two waves that hold the k halves of one 128 x 128 part each finish 64 of its rows: a wave hands the accumulator
  // tiles of the other 64 rows over through LDS (lane for lane) and adds what it receives to its own.
  constexpr int HM = TM / 2;
  f32x4* xch = reinterpret_cast<f32x4*>(lds);
  const int mine = wave * (HM * TN * 4), theirs = (wave ^ 2) * (HM * TN * 4);
  __syncthreads();  // every wave is done with the operand stages (all DMA has landed: the last tile was waited for)
  auto hand_over = [&](auto half_c) {
    constexpr int H = decltype(half_c)::value;
#pragma unroll
    for (int i = 0; i < HM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const f32x16& a = acc[H * HM + i][j];
          xch[(mine + (i * TN + j) * 4 + q) * 64 + lane] = f32x4{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
        }
  };
  auto finish = [&](auto half_c) {
    constexpr int H = decltype(half_c)::value;
#pragma unroll
    for (int i = 0; i < HM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        f32x16 a = acc[H * HM + i][j];
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const f32x4 o = xch[(theirs + (i * TN + j) * 4 + q) * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; e++) a[4 * q + e] += o[e];
        }
        epilogue_tile<EPI, FULL>(g, m0 + (H * HM + i) * 32, n0 + wn * 128 + j * 32, lane, a);
      }
  };
  if (wk == 0) hand_over(std::integral_constant<int, 1>{}); else hand_over(std::integral_constant<int, 0>{});
  __syncthreads();
  if (wk == 0) finish(std::integral_constant<int, 0>{}); else finish(std::integral_constant<int, 1>{});
}

template <bool A_KC, bool B_KC, int EPI, bool FULL>
__global__ __launch_bounds__(256) void gemm_dtl_rect_kernel(GemmArgs g) {  // g: by value, adjusted per k slice
  __shared__ __attribute__((aligned(1024))) char lds[kRectLds];
  int pid = blockIdx.x;
  if (g.ksplit > 1) {  // this workgroup's k range (k_per: a whole number of stages) and fp32 partial-result plane
    const int T = g.tiles_m * g.tiles_n, slice = pid / T, k0 = slice * g.k_per;
    pid -= slice * T;
    g.A += A_KC ? (size_t)k0 : (size_t)k0 * g.lda;
    g.B += B_KC ? (size_t)k0 : (size_t)k0 * g.ldb;
    g.K = g.k_per;
    g.C = reinterpret_cast<float*>(g.C) + (size_t)slice * g.M * g.ldc;
  }
  dtl_rect_tile<A_KC, B_KC, EPI, FULL>(g, pid, lds);
}

// =================================================================================================
// Eight-wave kernels: two waves on every SIMD, alternating between a memory phase and an MFMA phase.
// A wave's part of the block tile is 128 x 64 (128 accumulator registers), so two waves fit the register file of a SIMD.
// Waves 0-3 (one per SIMD) and waves 4-7 run the same loop one phase apart: group 1 passes one extra barrier before the
// loop and group 0 one behind it, so that every workgroup barrier ends a memory phase of one group and an MFMA phase of
// the other.  Memory phase of k tile kt: the 12 operand fragments of the tile are read from LDS into registers, the
// direct-to-LDS loads of tile kt+NS-1 are issued into the stage that held tile kt-1, and the wave waits until its own
// loads of tile kt+1 have landed.  MFMA phase: 16 MFMAs, nothing else.  While one wave of a SIMD multiplies, the other
// one's LDS reads, address arithmetic and waits cost the MFMA pipe nothing.
//   Why this is safe.  Number the barriers B0 (before the loop, all waves), B(2k+1) = {group 0 ends its memory phase k, group
//   1 ends its MFMA phase k-1 (k = 0: the extra barrier)}, B(2k+2) = {group 0 ends MFMA phase k, group 1 ends memory phase
//   k}.  Group 0 reads tile k between B(2k) and B(2k+1), group 1 between B(2k+1) and B(2k+2); every wave's reads have
//   returned (lgkmcnt(0)) before it reaches the barrier that ends the phase.  (a) Tile k is complete before it is read:
//   each wave waits for its own loads of tile k in its memory phase k-1, i.e. before B(2k-1) (group 0) or B(2k) (group
//   1); tile 0 before B0.  (b) A stage is refilled only after its last reader is done: tile k+NS-1 replaces tile k-1;
//   group 0 issues it behind B(2k), group 1 behind B(2k+1); the last reads of tile k-1 are group 1's, complete before
//   B(2k).
// 256 x 256 tiles (variant 301256256): waves 2 x 4, LDS stages and layouts of the four-wave direct-to-LDS kernel (four
// stages of 32 k).  128 x 256 tiles (301128256, over k slices 302128256 / 304128256): waves 1 x 4 x 2 -- the two groups
// split the four k steps of a 64-wide stage and add their accumulators through LDS after the loop -- three stages,
// layouts of the four-wave 128 x 256 kernel.  Shapes: as those kernels.
// =================================================================================================
// fragment I (of NF) of k step KK.  KC: off[KK] + I * FRAG bytes; MC: off[I] + KK * KSTEP bytes, second half HALF bytes on
template <bool KC, int KK, int I, int FRAG, int KSTEP, int HALF>
__device__ __forceinline__ u32x4 pp_read_frag(uint32_t base, const uint32_t* off) {
  if constexpr (KC) {
    return lds_read_b128<I * FRAG>(base + off[KK]);
  } else {
    const u32x2 lo = lds_read_tr16_b64<KK * KSTEP>(base + off[I]);
    const u32x2 hi = lds_read_tr16_b64<KK * KSTEP + HALF>(base + off[I]);
    return u32x4{lo[0], lo[1], hi[0], hi[1]};
  }
}
__device__ __forceinline__ void pp_wait_frags(u32x4 (&a)[2][4], u32x4 (&b)[2][2]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[0][2]), "+v"(a[0][3]), "+v"(a[1][0]), "+v"(a[1][1]), "+v"(a[1][2]), "+v"(a[1][3]),
                 "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]));
}

constexpr int kPpLds256 = NSD * kDtlStage;                                  // 128 KB
constexpr int kPpExchange = 8 * 2 * 2 * 4 * 64 * 16;                        // 128 x 256 tiles: half of every wave's accumulator
constexpr int kPpLds128 = NSR * kRectStage > kPpExchange ? NSR * kRectStage : kPpExchange;  // 144 KB

template <int BM, bool A_KC, bool B_KC, int EPI, bool FULL>
__device__ __forceinline__ void pp_tile(const GemmArgs& g, int pid, char* lds) {
  static_assert(BM == 256 || BM == 128, "block tiles 256 x 256 and 128 x 256");
  constexpr bool SQ = BM == 256;
  constexpr int NS = SQ ? NSD : NSR;                 // LDS stages
  constexpr int KT = SQ ? BKD : BKR;                 // k extent of a stage
  constexpr int kOpA = SQ ? kDtlOperand : kRectA;    // bytes of the A tile of a stage (B behind it)
  constexpr int kStage = SQ ? kDtlStage : kRectStage;
  constexpr int PER_A = 2, PER_B = SQ ? 2 : 4, PER = PER_A + PER_B;  // direct-to-LDS instructions of a wave per stage
  int tile_m, tile_n;
  tile_of_workgroup(pid, g.tiles_m, g.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * 256;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, wn = wave & 3;          // grp: phase group; 256 x 256: also the row half, 128 x 256: the k half
  const int nk = g.K / KT;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  const __amdgpu_buffer_rsrc_t rsA = operand_rsrc(g.A), rsB = operand_rsrc(g.B);
  uint32_t srcA[PER_A], srcB[PER_B];
#pragma unroll
  for (int j = 0; j < PER_A; j++)
    srcA[j] = lane_offset(SQ ? dtl_src<A_KC>(g.A, g.lda, m0, PER_A * wave + j, lane, g.M) : rect_src<A_KC, 128>(g.A, g.lda, m0, PER_A * wave + j, lane, g.M), g.A);
#pragma unroll
  for (int j = 0; j < PER_B; j++)
    srcB[j] = lane_offset(SQ ? dtl_src<B_KC>(g.B, g.ldb, n0, PER_B * wave + j, lane, g.N) : rect_src<B_KC, 256>(g.B, g.ldb, n0, PER_B * wave + j, lane, g.N), g.B);
#ifdef OASES_PP_SAMEK   // timing experiment: every k tile is tile 0 (all loads hit L2)
  const uint32_t stepA_k = 0, stepB_k = 0;
#else
  const uint32_t stepA_k = A_KC ? (uint32_t)KT * 2 : (uint32_t)KT * g.lda * 2, stepB_k = B_KC ? (uint32_t)KT * 2 : (uint32_t)KT * g.ldb * 2;  // next k tile
#endif
  auto issue = [&](int t) {
    char* st = lds + (t % NS) * kStage;
#pragma unroll
    for (int j = 0; j < PER_A; j++) dma16(rsA, srcA[j], (uint32_t)t * stepA_k, st + (PER_A * wave + j) * 1024);
#pragma unroll
    for (int j = 0; j < PER_B; j++) dma16(rsB, srcB[j], (uint32_t)t * stepB_k, st + kOpA + (PER_B * wave + j) * 1024);
  };

  uint32_t offA[4], offB[4];
  if constexpr (SQ) {
    dtl_frag_offsets<A_KC>(offA, grp * 128, lane);
    dtl_frag_offsets<B_KC>(offB, wn * 64, lane);
  } else {
    rect_frag_offsets<A_KC, 128>(offA, 0, grp, lane);
    rect_frag_offsets<B_KC, 256>(offB, wn * 64, grp, lane);
  }
  // strides of the LDS layouts: fragment to fragment (k-major operand), k step to k step and first to second half of a
  // fragment (row-indexed operand)
  constexpr int FRAG = SQ ? 2048 : 4096;
  constexpr int KSTEP_A = SQ ? 8192 : 16 * 2 * 128, HALF_A = SQ ? 2048 : 4 * 2 * 128;
  constexpr int KSTEP_B = SQ ? 8192 : 16 * 2 * 256, HALF_B = SQ ? 2048 : 4 * 2 * 256;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(OASES_LDS char*)lds;
  u32x4 fa[2][4], fb[2][2];
  auto read_stage = [&](uint32_t st) {
#define OASES_PP_A(KK, I) fa[KK][I] = pp_read_frag<A_KC, KK, I, FRAG, KSTEP_A, HALF_A>(st, offA);
#define OASES_PP_B(KK, I) fb[KK][I] = pp_read_frag<B_KC, KK, I, FRAG, KSTEP_B, HALF_B>(st + kOpA, offB);
    OASES_PP_A(0, 0) OASES_PP_A(0, 1) OASES_PP_A(0, 2) OASES_PP_A(0, 3) OASES_PP_B(0, 0) OASES_PP_B(0, 1)
    OASES_PP_A(1, 0) OASES_PP_A(1, 1) OASES_PP_A(1, 2) OASES_PP_A(1, 3) OASES_PP_B(1, 0) OASES_PP_B(1, 1)
#undef OASES_PP_A
#undef OASES_PP_B
  };
  auto mma = [&]() {
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, fa[kk][i]), b = __builtin_bit_cast(bf16x8, fb[kk][j]);
          if constexpr (EPI == EPI_F32) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
          else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[i][j], 0, 0, 0);
        }
  };
  constexpr int kYoung = PER * (NS - 2);  // direct-to-LDS instructions of the younger tiles that may still be in flight
  constexpr int kVmSteady = ((kYoung >> 4) << 14) | (kYoung & 15) | (7 << 4) | (15 << 8), kVm0 = (7 << 4) | (15 << 8);

#pragma unroll
  for (int t = 0; t < NS - 1; t++)
    if (t < nk) issue(t);
  if (nk > NS - 2) __builtin_amdgcn_s_waitcnt(kVmSteady); else __builtin_amdgcn_s_waitcnt(kVm0);  // own part of tile 0
  __builtin_amdgcn_s_barrier();                 // B0
  if (grp == 1) __builtin_amdgcn_s_barrier();   // group 1 runs one phase behind
  __builtin_amdgcn_sched_barrier(0);

  uint32_t cur = lds0;
  auto iteration = [&](auto steady_c, int kt) {
    constexpr bool STEADY = decltype(steady_c)::value;  // tile kt+NS-1 exists and is requested now
    // Timing experiments only (results are wrong with any bit set): -DOASES_PP_SKIP=bits switches parts of the loop off --
    // 1 the direct-to-LDS loads, 2 the fragment reads (tile 0's stay), 4 the priority changes, 8 the MFMAs, 16 the two
    // barriers (every wave still passes the same number of barriers); -DOASES_PP_SAMEK makes every k tile tile 0.
#ifndef OASES_PP_SKIP
#define OASES_PP_SKIP 0
#endif
    if (!(OASES_PP_SKIP & 2) || kt == 0) read_stage(cur);
    if (STEADY) {
      if (!(OASES_PP_SKIP & 1)) issue(kt + NS - 1);
      __builtin_amdgcn_s_waitcnt(kVmSteady);
    } else {
      __builtin_amdgcn_s_waitcnt(kVm0);
    }
    pp_wait_frags(fa, fb);
    __builtin_amdgcn_sched_barrier(0);
    if (!(OASES_PP_SKIP & 16)) __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (!(OASES_PP_SKIP & 4)) __builtin_amdgcn_s_setprio(1);
    if (!(OASES_PP_SKIP & 8)) mma();
    if (!(OASES_PP_SKIP & 4)) __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    if (!(OASES_PP_SKIP & 16)) __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    cur = cur + kStage == lds0 + NS * kStage ? lds0 : cur + kStage;
  };
  {
    int kt = 0;
    for (; kt + NS - 1 < nk; kt++) iteration(std::true_type{}, kt);
    for (; kt < nk; kt++) iteration(std::false_type{}, kt);
  }
  if (grp == 0) __builtin_amdgcn_s_barrier();   // group 0 catches up: both groups have passed the same number of barriers
  __builtin_amdgcn_sched_barrier(0);

  if constexpr (SQ) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if constexpr (EPI == EPI_SWIGLU) {  // the wave's 64 columns are one [gate 32 | up 32] block
        epilogue_tile_swiglu<FULL>(g, m0 + grp * 128 + i * 32, n0 + wn * 64, lane, acc[i][0], acc[i][1]);
      } else {
        epilogue_tile<EPI, FULL>(g, m0 + grp * 128 + i * 32, n0 + wn * 64, lane, acc[i][0]);
        epilogue_tile<EPI, FULL>(g, m0 + grp * 128 + i * 32, n0 + wn * 64 + 32, lane, acc[i][1]);
      }
    }
  } else {
    // The two waves that hold the k halves of one 128 x 64 part each finish 64 of its rows: a wave hands the accumulator
    // tiles of the other 64 rows over through LDS (lane for lane) and adds what it receives to its own (two terms: the
    // order of the addition does not matter).
    f32x4* xch = reinterpret_cast<f32x4*>(lds);
    const int mine = wave * 16, theirs = (wave ^ 4) * 16;  // 2 x 2 tiles x 4 quarters per wave
    __syncthreads();  // every wave has its last fragments in registers, and all direct-to-LDS loads have landed
    auto hand_over = [&](auto half_c) {
      constexpr int H = decltype(half_c)::value;
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const f32x16& a = acc[H * 2 + i][j];
            xch[(mine + (i * 2 + j) * 4 + q) * 64 + lane] = f32x4{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
          }
    };
    auto finish = [&](auto half_c) {
      constexpr int H = decltype(half_c)::value;
#pragma unroll
      for (int i = 0; i < 2; i++) {
        f32x16 a[2] = {acc[H * 2 + i][0], acc[H * 2 + i][1]};
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const f32x4 o = xch[(theirs + (i * 2 + j) * 4 + q) * 64 + lane];
#pragma unroll
            for (int e = 0; e < 4; e++) a[j][4 * q + e] += o[e];
          }
        if constexpr (EPI == EPI_SWIGLU) {
          epilogue_tile_swiglu<FULL>(g, m0 + (H * 2 + i) * 32, n0 + wn * 64, lane, a[0], a[1]);
        } else {
          epilogue_tile<EPI, FULL>(g, m0 + (H * 2 + i) * 32, n0 + wn * 64, lane, a[0]);
          epilogue_tile<EPI, FULL>(g, m0 + (H * 2 + i) * 32, n0 + wn * 64 + 32, lane, a[1]);
        }
      }
    };
    if (grp == 0) hand_over(std::integral_constant<int, 1>{}); else hand_over(std::integral_constant<int, 0>{});
    __syncthreads();
    if (grp == 0) finish(std::integral_constant<int, 0>{}); else finish(std::integral_constant<int, 1>{});
  }
}

template <int BM, bool A_KC, bool B_KC, int EPI, bool FULL>
__global__ __launch_bounds__(512) void gemm_pp_kernel(GemmArgs g) {  // g: by value, adjusted per k slice
  __shared__ __attribute__((aligned(1024))) char lds[BM == 256 ? kPpLds256 : kPpLds128];
  int pid = blockIdx.x;
  if (BM == 128 && g.ksplit > 1) {  // this workgroup's k range (k_per: a whole number of stages) and fp32 partial-result plane
    const int T = g.tiles_m * g.tiles_n, slice = pid / T, k0 = slice * g.k_per;
    pid -= slice * T;
    g.A += A_KC ? (size_t)k0 : (size_t)k0 * g.lda;
    g.B += B_KC ? (size_t)k0 : (size_t)k0 * g.ldb;
    g.K = g.k_per;
    g.C = reinterpret_cast<float*>(g.C) + (size_t)slice * g.M * g.ldc;
  }
  pp_tile<BM, A_KC, B_KC, EPI, FULL>(g, pid, lds);
}

// Two weight-gradient contractions over the same K rows in one launch: the tiles of the second problem follow those of
// the first, so that two launches that would each leave CUs idle (or need k slices to fill them) share one round.
__global__ __launch_bounds__(512) void gemm_pp_pair_kernel(GemmArgs g0, GemmArgs g1) {
  __shared__ __attribute__((aligned(1024))) char lds[kPpLds128];
  const int first = g0.tiles_m * g0.tiles_n;
  if ((int)blockIdx.x < first) pp_tile<128, false, false, EPI_ACC_F32, true>(g0, blockIdx.x, lds);
  else pp_tile<128, false, false, EPI_ACC_F32, true>(g1, blockIdx.x - first, lds);
}

// split-K second pass: C = epilogue(sum over slices of the fp32 partial planes), slices added in index order
template <int EPI>
__global__ __launch_bounds__(256) void splitk_fixup_kernel(const float* __restrict__ part, int S, GemmArgs g) {
  const int nc4 = g.N >> 2;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)g.M * nc4) return;
  const int row = (int)(idx / nc4), col = (int)(idx % nc4) * 4;
  const size_t plane = (size_t)g.M * g.N;
  f32x4 v = *reinterpret_cast<const f32x4*>(part + (size_t)row * g.N + col);
  for (int s2 = 1; s2 < S; s2++) v += *reinterpret_cast<const f32x4*>(part + s2 * plane + (size_t)row * g.N + col);
  const size_t o = (size_t)row * g.ldc + col;
  if (EPI == EPI_F32) {
    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + o) = v;
  } else if (EPI == EPI_ACC_F32) {
    f32x4* p = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + o);
    *p = *p + v;
  } else {
    uint16_t* cp = reinterpret_cast<uint16_t*>(g.C) + o;
    if (EPI == EPI_BIAS_BF16 || EPI == EPI_BIAS_GELU) v += *reinterpret_cast<const f32x4*>(g.bias + col);
    if (EPI == EPI_BIAS_GELU) {
      *reinterpret_cast<u32x2*>(g.aux + (size_t)row * g.ldaux + col) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
#pragma unroll
      for (int e = 0; e < 4; e++) v[e] = gelu_tanh(v[e]);
    } else if (EPI == EPI_DGELU) {
      u32x2 a = *reinterpret_cast<const u32x2*>(g.aux + (size_t)row * g.ldaux + col);
      v[0] *= gelu_tanh_grad(bf16_bits_to_f32(a[0] & 0xffffu));
      v[1] *= gelu_tanh_grad(bf16_bits_to_f32(a[0] >> 16));
      v[2] *= gelu_tanh_grad(bf16_bits_to_f32(a[1] & 0xffffu));
      v[3] *= gelu_tanh_grad(bf16_bits_to_f32(a[1] >> 16));
    }
    *reinterpret_cast<u32x2*>(cp) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
  }
}

template <int BM, int BN, int WGM, int WGN, int WGK, bool A_KC, bool B_KC, int EPI>
int launch_one(const GemmArgs& g0, int ksplit, float* ws, hipStream_t s) {
  GemmArgs g = g0;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = (g.N + BN - 1) / BN;
  g.ksplit = 1;
  g.k_per = g.K;
  dim3 block(64 * WGM * WGN * WGK);
  if (ksplit <= 1) {
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, WGK, A_KC, B_KC, EPI>), dim3(g.tiles_m * g.tiles_n), block, 0, s, g);
    OASES_LAUNCH_CHECK("gemm_kernel");
    return 0;
  }
  // first pass: fp32 partial planes [ksplit][M][N] in the workspace; second pass: sum + the real epilogue
  if (!ws) { set_error("gemm: split-K chosen without a workspace"); return OASES_ENULL; }
  if (EPI == EPI_SWIGLU || EPI == EPI_DSWIGLU) { set_error("gemm: the SwiGLU epilogues do not run over k slices"); return OASES_EINVAL; }
  GemmArgs p = g;
  p.ksplit = ksplit;
  p.k_per = ((g.K + ksplit - 1) / ksplit + BK - 1) / BK * BK;
  p.C = ws;
  p.ldc = g.N;
  hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, WGK, A_KC, B_KC, EPI_F32>), dim3(g.tiles_m * g.tiles_n * ksplit), block, 0, s, p);
  OASES_LAUNCH_CHECK("gemm_kernel (split-K)");
  const long n4 = (long)g.M * (g.N / 4);
  hipLaunchKernelGGL((splitk_fixup_kernel<EPI>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, ws, ksplit, g);
  OASES_LAUNCH_CHECK("splitk_fixup_kernel");
  return 0;
}

// Tile and split-K choice by a small time model.  Bigger tiles run closer to the MFMA rate (fewer LDS bytes per flop)
// but a launch only uses the chip well if its workgroup count is near a multiple of the 256 CUs; splitting K multiplies
// the workgroup count at the price of a second pass over fp32 partial planes.  Rates measured on this part.
struct TileChoice { int bm, bn, ksplit; bool wave_ksplit; bool dtl = false; bool pp = false; };  // pp: the eight-wave kernel of a direct-to-LDS tile shape
// per kind of contraction (0: NN, 1: NT, 2: TN, 3: NN with the bias+GeLU epilogue): whether the rectangular tiles
// split k between waves, and the sustained rates of the four block tiles
// Shapes the direct-to-LDS kernels cover, per kind of contraction (0, 3: NN, 1: NT, 2: TN): whole k tiles; in the
// 256 x 256 kernel a k-major operand must fill its tiles and a row-indexed one (A of TN; B of NN and TN) may end inside
// its last tile; in the 128 x 256 kernel both may.
bool dtl_fits(int kind, int M, int N, int K) {
  return (kind == 2 || M % 256 == 0) && (kind != 1 || N % 256 == 0) && M % 8 == 0 && N % 8 == 0 && K % BKD == 0 && K >= BKD;
}
bool dtl_rect_fits(int kind, int M, int N, int K) {  // the 128 x 256 kernel redirects rows of a k-major operand too
  (void)kind;
  return M % 8 == 0 && N % 8 == 0 && K % BKR == 0 && K >= BKR;
}
bool dtl_rect_whole(int M, int N, int K) { return M % 128 == 0 && N % 256 == 0 && K % BKR == 0 && K >= BKR; }
struct KindTable { bool wave_ksplit; float r256x256, r128x256, r256x128, r128x128; };
const KindTable g_kinds[4] = {{true, 1200.f, 1080.f, 960.f, 740.f}, {true, 1200.f, 1080.f, 960.f, 740.f},
                        {true, 1200.f, 1080.f, 960.f, 740.f}, {false, 1200.f, 1080.f, 900.f, 740.f}};
TileChoice pick_tile(int kind, int epi, int M, int N, int K, size_t ws_bytes) {
  const KindTable& kt = g_kinds[kind];
  const struct { int bm, bn; float tflops; } cand[] = {{256, 256, kt.r256x256}, {128, 256, kt.r128x256}, {256, 128, kt.r256x128}, {128, 128, kt.r128x128}};
  TileChoice best{128, 128, 1, kt.wave_ksplit};
  double best_t = 1e30;
  for (auto& c : cand) {
    const long tm = (M + c.bm - 1) / c.bm, tn = (N + c.bn - 1) / c.bn;
    for (int S = 1; S <= 8; S *= 2) {
      if (S > 1 && ((size_t)S * M * N * 4 > ws_bytes || K / S < 512)) break;
      const long wgs = tm * tn * S, rounds = (wgs + 255) / 256;
      // time of one workgroup's tile slice at the tile's rate (one workgroup per CU), times the number of rounds
      double t = (double)rounds * (2.0 * c.bm * c.bn * ((double)K / S) + 3.0e6) / (c.tflops * 1e12 / 256.0);
      if (S > 1) t += ((double)(2 * S + 1) * M * N * 4.0) / 3.0e12 + 4e-6;
      if (t < best_t) { best_t = t; best = TileChoice{c.bm, c.bn, S, kt.wave_ksplit}; }
    }
  }
  // Whole tiles without k slices: the eight-wave direct-to-LDS kernels, which measure faster than the four-wave and the
  // register-staged kernels of the same tile on every shape of the two full-size workloads (cold operands, 3-15 %).
  if (best.ksplit == 1) {
    if (best.bm == 256 && best.bn == 256 && dtl_fits(kind, M, N, K)) best.dtl = best.pp = true;
    if (best.bm == 128 && best.bn == 256 && dtl_rect_fits(kind, M, N, K)) best = TileChoice{128, 256, 1, true, true, true};
    // Few rows, long k (a sub-batch of 1024 rows against K = 8192): 128 x 128 tiles fill the chip but run at the small
    // tile's rate; the 128 x 256 direct-to-LDS kernel over two k slices fills it too, and is faster even with its second
    // pass (measured on cold operands: 87-93 us against 108-116 us).
    const long rtiles = (long)((M + 127) / 128) * ((N + 255) / 256);
    if (best.bm == 128 && best.bn == 128 && epi != EPI_SWIGLU && epi != EPI_DSWIGLU && 2 * rtiles >= 192 && 2 * rtiles <= 256 && K >= 4096 &&
        K % (2 * BKR) == 0 && dtl_rect_fits(kind, M, N, K / 2) && (size_t)2 * M * N * 4 <= ws_bytes)
      best = TileChoice{128, 256, 2, true, true, true};
  } else if (best.bm == 128 && best.bn == 256 && (best.ksplit == 2 || best.ksplit == 4) && epi != EPI_SWIGLU && epi != EPI_DSWIGLU &&
             K % (best.ksplit * BKR) == 0 && dtl_rect_fits(kind, M, N, K / best.ksplit)) {
    best = TileChoice{128, 256, best.ksplit, true, true, true};  // k slices of whole stages: the eight-wave kernel
  }
  return best;
}

int encode_variant(const TileChoice& t) {
  const bool rect = t.bm != t.bn;
  return (t.dtl ? (t.pp ? 300000000 : 200000000) : rect && t.wave_ksplit ? 100000000 : 0) + t.ksplit * 1000000 + t.bm * 1000 + t.bn;
}
// variant -> TileChoice; false if no such instantiation exists or the k slices do not fit the problem / workspace
bool decode_variant(int variant, int kind, int M, int N, int K, size_t ws_bytes, TileChoice* t) {
  if (variant <= 0) return false;
  const int wk = variant / 100000000, S = variant / 1000000 % 100, bm = variant / 1000 % 1000, bn = variant % 1000;
  const bool square = (bm == 256 && bn == 256) || (bm == 128 && bn == 128), rect = (bm == 256 && bn == 128) || (bm == 128 && bn == 256);
  if ((wk == 2 || wk == 3) && S == 1) {  // direct-to-LDS kernels (3: eight waves), one k slice
    if (bm == 256 && bn == 256 && dtl_fits(kind, M, N, K)) { *t = TileChoice{256, 256, 1, false, true, wk == 3}; return true; }
    if (bm == 128 && bn == 256 && dtl_rect_fits(kind, M, N, K)) { *t = TileChoice{128, 256, 1, true, true, wk == 3}; return true; }
    return false;
  }
  if ((wk == 2 || wk == 3) && bm == 128 && bn == 256 && (S == 2 || S == 4)) {  // the 128 x 256 kernels over k slices of whole stages
    if (K % (S * BKR) || !dtl_rect_fits(kind, M, N, K / S) || (size_t)S * M * N * 4 > ws_bytes) return false;
    *t = TileChoice{128, 256, S, true, true, wk == 3};
    return true;
  }
  if (wk > 1 || !(square || rect) || (wk == 1 && !rect) || S < 1 || S > 8) return false;
  if (S > 1) {
    const int k_per = ((K + S - 1) / S + BK - 1) / BK * BK;
    if ((size_t)S * M * N * 4 > ws_bytes || (long)(S - 1) * k_per >= K) return false;
  }
  *t = TileChoice{bm, bn, S, wk == 1};
  return true;
}

template <bool A_KC, bool B_KC, int EPI>
int launch_shape(const GemmArgs& g, float* ws, size_t ws_bytes, int forced_variant, int choice_rows, hipStream_t s) {
  constexpr int kind = !A_KC ? 2 : B_KC ? 1 : (EPI == EPI_BIAS_GELU || EPI == EPI_SWIGLU) ? 3 : 0;
  if (EPI == EPI_SWIGLU || EPI == EPI_DSWIGLU) ws_bytes = 0;  // their epilogues pair columns: no second pass over partial planes
  TileChoice t;
  if (forced_variant == 0) {
    // Pinned choice: the number of k slices and whether waves split k -- the two things that set the order in which the
    // fp32 terms of an output element are added -- come from (choice_rows, N, K, epilogue), so every launch over a part of
    // those rows adds in the same order.  The 256 x 256 direct-to-LDS kernels need whole row tiles; a part that has none
    // runs the staged kernel of the same tile, which adds in the same order.
    const bool pinned = kind != 2 && choice_rows > g.M;
    t = pick_tile(kind, EPI, pinned ? choice_rows : g.M, g.N, g.K, ws ? ws_bytes : 0);
    if (pinned && t.dtl && t.bm == 256 && !dtl_fits(kind, g.M, g.N, g.K)) t.dtl = t.pp = false;
    const int rows = pinned ? choice_rows : g.M;
    if (t.dtl && !(gemm_span_fits(A_KC ? rows : g.K, g.lda) && gemm_span_fits(B_KC ? g.N : g.K, g.ldb))) t.dtl = t.pp = false;
#ifdef OASES_GEMM_TUNE_HOOK
    {  // tuning aid (not compiled into the library): OASES_GEMM_TUNE="kind:epi:M:N:K=variant;..." overrides the choice
      static const char* tune = getenv("OASES_GEMM_TUNE");
      if (tune) {
        char key[96];
        snprintf(key, sizeof key, "%d:%d:%d:%d:%d=", kind, (int)EPI, g.M, g.N, g.K);
        const char* hit = strstr(tune, key);
        TileChoice tt;
        if (hit && decode_variant(atoi(hit + strlen(key)), kind, g.M, g.N, g.K, ws ? ws_bytes : 0, &tt)) t = tt;
      }
    }
#endif
  } else if (!decode_variant(forced_variant, kind, g.M, g.N, g.K, ws ? ws_bytes : 0, &t)) {
    set_error("gemm: variant %d does not exist or does not fit M=%d N=%d K=%d with %zu workspace bytes", forced_variant, g.M, g.N, g.K, ws ? ws_bytes : (size_t)0);
    return OASES_EINVAL;
  } else if (t.dtl && !(gemm_span_fits(A_KC ? g.M : g.K, g.lda) && gemm_span_fits(B_KC ? g.N : g.K, g.ldb))) {
    set_error("gemm: variant %d (direct-to-LDS) needs operands that span less than 2 GiB (lda=%d ldb=%d)", forced_variant, g.lda, g.ldb);
    return OASES_EINVAL;
  }
  if (t.dtl && t.pp) {
    constexpr bool kCanBeRagged = !A_KC || !B_KC;
    const int bm = t.bm;
    GemmArgs d = g;
    d.tiles_m = (g.M + bm - 1) / bm;
    d.tiles_n = (g.N + 255) / 256;
    const bool whole = g.M % bm == 0 && g.N % 256 == 0;
    if (!whole && bm == 256 && !kCanBeRagged) { set_error("gemm: direct-to-LDS kernel on a shape it does not cover"); return OASES_EINVAL; }
    if (bm == 128 && t.ksplit > 1) {
      if constexpr (EPI == EPI_SWIGLU || EPI == EPI_DSWIGLU) {
        set_error("gemm: the SwiGLU epilogues do not run over k slices");
        return OASES_EINVAL;
      } else {
        if (!ws) { set_error("gemm: split-K chosen without a workspace"); return OASES_ENULL; }
        GemmArgs p = d;
        p.ksplit = t.ksplit;
        p.k_per = g.K / t.ksplit;
        p.C = ws;
        p.ldc = g.N;
        const dim3 sgrid(d.tiles_m * d.tiles_n * t.ksplit);
        if (whole) hipLaunchKernelGGL((gemm_pp_kernel<128, A_KC, B_KC, EPI_F32, true>), sgrid, dim3(512), 0, s, p);
        else hipLaunchKernelGGL((gemm_pp_kernel<128, A_KC, B_KC, EPI_F32, false>), sgrid, dim3(512), 0, s, p);
        OASES_LAUNCH_CHECK("gemm_pp_kernel (split-K)");
        const long n4 = (long)g.M * (g.N / 4);
        hipLaunchKernelGGL((splitk_fixup_kernel<EPI>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, ws, t.ksplit, d);
        OASES_LAUNCH_CHECK("splitk_fixup_kernel");
        return 0;
      }
    }
    const dim3 grid(d.tiles_m * d.tiles_n);
    if (bm == 128) {
      if (whole) hipLaunchKernelGGL((gemm_pp_kernel<128, A_KC, B_KC, EPI, true>), grid, dim3(512), 0, s, d);
      else hipLaunchKernelGGL((gemm_pp_kernel<128, A_KC, B_KC, EPI, false>), grid, dim3(512), 0, s, d);
    } else {
      if (whole) hipLaunchKernelGGL((gemm_pp_kernel<256, A_KC, B_KC, EPI, true>), grid, dim3(512), 0, s, d);
      else if constexpr (kCanBeRagged) hipLaunchKernelGGL((gemm_pp_kernel<256, A_KC, B_KC, EPI, false>), grid, dim3(512), 0, s, d);
    }
    OASES_LAUNCH_CHECK("gemm_pp_kernel");
    return 0;
  }
  if (t.dtl) {
    if (EPI == EPI_SWIGLU && t.bm == 128) {
      set_error("gemm: the 128x256 direct-to-LDS kernel has no SwiGLU epilogue");
      return OASES_EINVAL;
    } else {
      // the 256 x 256 instantiation with bounds checks in the epilogue exists only where a tile can be ragged
      constexpr bool kCanBeRagged = !A_KC || !B_KC;
      const int bm = t.bm;  // 128 or 256; both kernels have 256-column tiles
      GemmArgs d = g;
      d.tiles_m = (g.M + bm - 1) / bm;
      d.tiles_n = (g.N + 255) / 256;
      const dim3 grid(d.tiles_m * d.tiles_n);
      const bool whole = g.M % bm == 0 && g.N % 256 == 0;
      if (!whole && bm == 256 && !kCanBeRagged) { set_error("gemm: direct-to-LDS kernel on a shape it does not cover"); return OASES_EINVAL; }
      if (bm == 128 && t.ksplit > 1) {
        // k slices: fp32 partial planes [slices][M][N] in the workspace, then the sum and the real epilogue
        if constexpr (EPI == EPI_SWIGLU || EPI == EPI_DSWIGLU) {
          set_error("gemm: the SwiGLU epilogues do not run over k slices");
          return OASES_EINVAL;
        } else {
          if (!ws) { set_error("gemm: split-K chosen without a workspace"); return OASES_ENULL; }
          GemmArgs p = d;
          p.ksplit = t.ksplit;
          p.k_per = g.K / t.ksplit;
          p.C = ws;
          p.ldc = g.N;
          const dim3 sgrid(d.tiles_m * d.tiles_n * t.ksplit);
          if (whole) hipLaunchKernelGGL((gemm_dtl_rect_kernel<A_KC, B_KC, EPI_F32, true>), sgrid, dim3(256), 0, s, p);
          else hipLaunchKernelGGL((gemm_dtl_rect_kernel<A_KC, B_KC, EPI_F32, false>), sgrid, dim3(256), 0, s, p);
          OASES_LAUNCH_CHECK("gemm_dtl_rect_kernel (split-K)");
          const long n4 = (long)g.M * (g.N / 4);
          hipLaunchKernelGGL((splitk_fixup_kernel<EPI>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, ws, t.ksplit, d);
          OASES_LAUNCH_CHECK("splitk_fixup_kernel");
          return 0;
        }
      } else if (bm == 128) {
        if constexpr (EPI != EPI_SWIGLU) {
          if (whole) hipLaunchKernelGGL((gemm_dtl_rect_kernel<A_KC, B_KC, EPI, true>), grid, dim3(256), 0, s, d);
          else hipLaunchKernelGGL((gemm_dtl_rect_kernel<A_KC, B_KC, EPI, false>), grid, dim3(256), 0, s, d);
        }
      } else {
        if (whole) hipLaunchKernelGGL((gemm_dtl_kernel<A_KC, B_KC, EPI, true>), grid, dim3(256), 0, s, d);
        else if constexpr (kCanBeRagged) hipLaunchKernelGGL((gemm_dtl_kernel<A_KC, B_KC, EPI, false>), grid, dim3(256), 0, s, d);
      }
      OASES_LAUNCH_CHECK("gemm direct-to-LDS kernel");
      return 0;
    }
  }
  if (t.bm == 256 && t.bn == 256) return launch_one<256, 256, 2, 2, 1, A_KC, B_KC, EPI>(g, t.ksplit, ws, s);
  if (!t.wave_ksplit) {
    if (t.bm == 256 && t.bn == 128) return launch_one<256, 128, 2, 2, 1, A_KC, B_KC, EPI>(g, t.ksplit, ws, s);
    if (t.bm == 128 && t.bn == 256) return launch_one<128, 256, 2, 2, 1, A_KC, B_KC, EPI>(g, t.ksplit, ws, s);
  }
  if (t.bm == 256 && t.bn == 128) return launch_one<256, 128, 2, 1, 2, A_KC, B_KC, EPI>(g, t.ksplit, ws, s);
  if (t.bm == 128 && t.bn == 256) return launch_one<128, 256, 1, 2, 2, A_KC, B_KC, EPI>(g, t.ksplit, ws, s);
  return launch_one<128, 128, 2, 2, 1, A_KC, B_KC, EPI>(g, t.ksplit, ws, s);
}

}  // namespace

#if OASES_GEMM_HAS(0)
int launch_gemm_nn(const GemmArgs& g, int epi, float* ws, size_t ws_bytes, int forced_variant, int choice_rows, hipStream_t s) {
  switch (epi) {
    case EPI_F32: return launch_shape<true, false, EPI_F32>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_BF16: return launch_shape<true, false, EPI_BF16>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_BIAS_BF16: return launch_shape<true, false, EPI_BIAS_BF16>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_BIAS_GELU: return launch_shape<true, false, EPI_BIAS_GELU>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_DGELU: return launch_shape<true, false, EPI_DGELU>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_SWIGLU: return launch_shape<true, false, EPI_SWIGLU>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    default: set_error("gemm: unknown epilogue %d", epi); return OASES_EINVAL;
  }
}
#endif
#if OASES_GEMM_HAS(1)
int launch_gemm_nt(const GemmArgs& g, int epi, float* ws, size_t ws_bytes, int forced_variant, int choice_rows, hipStream_t s) {
  switch (epi) {
    case EPI_F32: return launch_shape<true, true, EPI_F32>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_BF16: return launch_shape<true, true, EPI_BF16>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_BIAS_BF16: return launch_shape<true, true, EPI_BIAS_BF16>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_BIAS_GELU: return launch_shape<true, true, EPI_BIAS_GELU>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_DGELU: return launch_shape<true, true, EPI_DGELU>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    case EPI_DSWIGLU: return launch_shape<true, true, EPI_DSWIGLU>(g, ws, ws_bytes, forced_variant, choice_rows, s);
    default: set_error("gemm: unknown epilogue %d", epi); return OASES_EINVAL;
  }
}
#endif
#if OASES_GEMM_HAS(2)
int launch_gemm_tn(const GemmArgs& g, float* ws, size_t ws_bytes, int forced_variant, hipStream_t s) {
  return launch_shape<false, false, EPI_ACC_F32>(g, ws, ws_bytes, forced_variant, 0, s);
}

bool gemm_tn_pair_wins(int K, int M0, int N0, int M1, int N1) {
  if (M0 <= 0 || N0 <= 0 || M1 <= 0 || N1 <= 0 || !dtl_rect_whole(M0, N0, K) || !dtl_rect_whole(M1, N1, K)) return false;
  const long t0 = (long)(M0 / 128) * (N0 / 256), t1 = (long)(M1 / 128) * (N1 / 256);
  // enough tiles to be worth whole 128 x 256 tiles at all, and fewer rounds of 256 workgroups together than apart
  return t0 + t1 > 128 && (t0 + t1 + 255) / 256 < (t0 + 255) / 256 + (t1 + 255) / 256;
}

int launch_gemm_tn_pair(int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0, void* C0, int ldc0, int M1, int N1,
                        const void* A1, int lda1, const void* B1, int ldb1, void* C1, int ldc1, hipStream_t s) {
  if (K <= 0 || M0 <= 0 || N0 <= 0 || M1 <= 0 || N1 <= 0 || !dtl_rect_whole(M0, N0, K) || !dtl_rect_whole(M1, N1, K)) {
    set_error("gemm_tn_pair: needs M %% 128 == 0, N %% 256 == 0, K %% 64 == 0 for both problems (got K=%d, %dx%d and %dx%d)", K, M0, N0, M1, N1);
    return OASES_EINVAL;
  }
  if ((lda0 % 8) || (ldb0 % 8) || (ldc0 % 4) || (lda1 % 8) || (ldb1 % 8) || (ldc1 % 4) || lda0 < M0 || ldb0 < N0 || ldc0 < N0 || lda1 < M1 ||
      ldb1 < N1 || ldc1 < N1) {
    set_error("gemm_tn_pair: leading dimension too small or not a multiple of 8 (A, B) / 4 (C)");
    return OASES_EINVAL;
  }
  if (!gemm_span_fits(K, lda0) || !gemm_span_fits(K, ldb0) || !gemm_span_fits(K, lda1) || !gemm_span_fits(K, ldb1)) {
    set_error("gemm_tn_pair: an operand spans 2 GiB or more (K=%d rows)", K);
    return OASES_EINVAL;
  }
  if (!A0 || !B0 || !C0 || !A1 || !B1 || !C1) { set_error("gemm_tn_pair: NULL operand"); return OASES_ENULL; }
  if (!aligned16(A0) || !aligned16(B0) || !aligned16(C0) || !aligned16(A1) || !aligned16(B1) || !aligned16(C1)) {
    set_error("gemm_tn_pair: operand not 16-byte aligned");
    return OASES_EALIGN;
  }
  GemmArgs g0{(const uint16_t*)A0, (const uint16_t*)B0, C0, nullptr, nullptr, M0, N0, K, lda0, ldb0, ldc0, 0, M0 / 128, N0 / 256, 1, K};
  GemmArgs g1{(const uint16_t*)A1, (const uint16_t*)B1, C1, nullptr, nullptr, M1, N1, K, lda1, ldb1, ldc1, 0, M1 / 128, N1 / 256, 1, K};
  hipLaunchKernelGGL(gemm_pp_pair_kernel, dim3(g0.tiles_m * g0.tiles_n + g1.tiles_m * g1.tiles_n), dim3(512), 0, s, g0, g1);
  OASES_LAUNCH_CHECK("gemm_pp_pair_kernel");
  return 0;
}

#endif  // TN part
#if OASES_GEMM_HAS(0)
int gemm_variant(int op, int epi, int M, int N, int K, size_t ws_bytes) {
  const int kind = op == OASES_GEMM_TN ? 2 : op == OASES_GEMM_NT ? 1 : (epi == EPI_BIAS_GELU || epi == EPI_SWIGLU) ? 3 : 0;
  if (epi == EPI_SWIGLU || epi == EPI_DSWIGLU) ws_bytes = 0;
  return encode_variant(pick_tile(kind, op == OASES_GEMM_TN ? EPI_ACC_F32 : epi, M, N, K, ws_bytes));
}

int launch_gemm(int op, int epi, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C,
                int ldc, const float* bias, void* aux, int ldaux, void* splitk_ws, size_t splitk_ws_bytes, int forced_variant,
                hipStream_t s, int choice_rows) {
  float* ws = reinterpret_cast<float*>(splitk_ws);
  const size_t wsb = splitk_ws_bytes;
  if (M <= 0 || N <= 0 || K <= 0 || (M % 8) || (N % 8) || (K % 8) || (lda % 8) || (ldb % 8) || (ldc % 4) || (aux && ldaux % 4)) {
    set_error("gemm: M,N,K,lda,ldb must be positive multiples of 8, ldc/ldaux of 4 (got M=%d N=%d K=%d lda=%d ldb=%d ldc=%d)", M, N, K, lda, ldb, ldc);
    return OASES_EINVAL;
  }
  if (!A || !B || !C) { set_error("gemm: NULL operand"); return OASES_ENULL; }
  if (!aligned16(A) || !aligned16(B) || !aligned16(C) || !aligned16(bias) || !aligned16(aux)) { set_error("gemm: operand not 16-byte aligned"); return OASES_EALIGN; }
  GemmArgs g{(const uint16_t*)A, (const uint16_t*)B, C, bias, (uint16_t*)aux, M, N, K, lda, ldb, ldc, ldaux, 0, 0, 1, K};
  if (op == OASES_GEMM_TN) {
    if (lda < M || ldb < N || ldc < N) { set_error("gemm TN: leading dimension too small"); return OASES_EINVAL; }
    return launch_gemm_tn(g, ws, wsb, forced_variant, s);
  }
  const bool nn = op == OASES_GEMM_NN;
  if (!nn && op != OASES_GEMM_NT) { set_error("gemm: unknown op %d", op); return OASES_EINVAL; }
  const int c_cols = epi == EPI_SWIGLU ? N / 2 : epi == EPI_DSWIGLU ? 2 * N : N;  // SwiGLU: C is [M, N/2]; its gradient: [M, 2N]
  if (lda < K || (nn ? ldb < N : ldb < K) || ldc < c_cols) { set_error("gemm: leading dimension too small"); return OASES_EINVAL; }
  if (epi == EPI_SWIGLU && (!nn || N % 64 || !aux || ldaux < N)) { set_error("gemm: SwiGLU epilogue needs the NN form, N %% 64 == 0 and aux [M,N]"); return OASES_EINVAL; }
  if (epi == EPI_DSWIGLU && (nn || N % 32 || !aux || ldaux < 2 * N)) { set_error("gemm: SwiGLU-gradient epilogue needs the NT form, N %% 32 == 0 and aux [M,2N]"); return OASES_EINVAL; }
  if ((epi == OASES_EPI_BIAS_BF16 || epi == OASES_EPI_BIAS_GELU) && !bias) { set_error("gemm: bias epilogue without bias"); return OASES_ENULL; }
  if ((epi == OASES_EPI_BIAS_GELU || epi == OASES_EPI_DGELU) && (!aux || ldaux < N)) { set_error("gemm: GeLU epilogue without aux"); return OASES_ENULL; }
  if ((nn && epi == EPI_DSWIGLU) || (!nn && epi == EPI_SWIGLU) || epi < 0 || epi > EPI_DSWIGLU || epi == EPI_ACC_F32) {
    set_error("gemm: unknown epilogue %d", epi);
    return OASES_EINVAL;
  }
  return nn ? launch_gemm_nn(g, epi, ws, wsb, forced_variant, choice_rows, s) : launch_gemm_nt(g, epi, ws, wsb, forced_variant, choice_rows, s);
}
#endif  // NN part and host entry points

}  // namespace oases
