// Shared device/host helpers of the HIP path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/oases.h"

namespace oases {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define OASES_LDS __attribute__((address_space(3)))

// ---- error plumbing (host) -------------------------------------------------------------------
void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);
#define OASES_HIP(call)                                     \
  do {                                                      \
    hipError_t e__ = (call);                                \
    if (e__ != hipSuccess) return hip_fail(e__, #call);     \
  } while (0)
#define OASES_LAUNCH_CHECK(name)                            \
  do {                                                      \
    hipError_t e__ = hipGetLastError();                     \
    if (e__ != hipSuccess) return hip_fail(e__, name);      \
  } while (0)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- bf16 conversions (round to nearest even; v_cvt_pk_bf16_f32 on gfx950) -------------------------
typedef float f32x2_ __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_ __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_ v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) {
  return __builtin_bit_cast(float, b << 16);
}

// ---- Philox4x32-10 (Salmon et al., SC'11) ------------------------------------------------------
struct Philox4 {
  uint32_t v[4];
};
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; r++) {
    uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += W0; k1 += W1;
  }
  return Philox4{{c0, c1, c2, c3}};
}

// Keep decisions of the 4 elements e = 4q .. 4q+3 of the unsharded [M,h] activation.
struct DropCfg {
  uint32_t k0, k1;      // seed lo / hi
  uint32_t site, layer; // counter words 2, 3
  uint32_t thresh;      // drop iff (word >> 8) < thresh; 0 disables dropout
  float scale;          // 1/(1-p)
};
__device__ __forceinline__ void dropout_keep4(const DropCfg& d, uint64_t q, bool keep[4]) {
  if (d.thresh == 0) {
    keep[0] = keep[1] = keep[2] = keep[3] = true;
    return;
  }
  Philox4 w = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), d.site, d.layer, d.k0, d.k1);
#pragma unroll
  for (int j = 0; j < 4; j++) keep[j] = (w.v[j] >> 8) >= d.thresh;
}
DropCfg make_drop_cfg(uint64_t seed, int layer, int site, float p);

// ---- tanh-form GeLU ----------------------------------------------------------------------------
__device__ __forceinline__ float fast_tanh(float x) {
  // tanh(x) = 1 - 2/(exp(2x)+1); exp via exp2
  float e = __builtin_amdgcn_exp2f(x * 2.885390081777927f);  // exp(2x)
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}
__device__ __forceinline__ float gelu_tanh(float x) {
  const float c0 = 0.7978845608028654f, c1 = 0.044715f;
  float t = fast_tanh(c0 * (x + c1 * x * x * x));
  return 0.5f * x * (1.0f + t);
}
__device__ __forceinline__ float gelu_tanh_grad(float x) {
  const float c0 = 0.7978845608028654f, c1 = 0.044715f;
  float t = fast_tanh(c0 * (x + c1 * x * x * x));
  return 0.5f * (1.0f + t) + 0.5f * x * (1.0f - t * t) * c0 * (1.0f + 3.0f * c1 * x * x);
}

// ---- two-stage column reductions (bias and LayerNorm-parameter gradients) ------------------------------------
// First stage: the kernel that walks the rows leaves one partial row per row group in a scratch array [groups][cols].
// Second stage: out[c] += sum over the partial rows, in a fixed order.  The second stage either follows at once, or --
// with a ColsumSink -- is put on a list, so that all column reductions of a pass share one launch at its end and the
// partial rows of one output from all sub-batches are added up together.
struct ColsumJob {
  const float* src;  // [groups][cols] partial rows
  float* out;        // [cols], accumulated into; NULL: no job
  int groups, cols;
};
constexpr int kMaxColsumJobs = 48;  // jobs of one second-stage launch
struct ColsumSink {
  // layout of the caller's arena for one first-stage call: its partial rows start at row `first_row` of `rows_total` rows
  // per output array, the arrays of a call with several outputs lie `kstride` floats apart
  int first_row = 0, rows_total = 0;
  size_t kstride = 0;
  ColsumJob* jobs = nullptr;  // list being built (capacity cap)
  int n = 0, cap = 0;
  bool overflow = false;
  void add(float* out, const float* base, int groups, int cols) {  // one job per output array: the same array is added only once
    for (int i = 0; i < n; i++)
      if (jobs[i].out == out && jobs[i].src == base) return;
    if (n >= cap) { overflow = true; return; }
    jobs[n++] = ColsumJob{base, out, groups, cols};
  }
};
int colsum_groups(int rows);  // row groups (partial rows) the first stage makes for `rows` rows
int launch_colsum_finalize(const ColsumJob* jobs, int n, hipStream_t s);

// ---- kernel launchers (one per .hip file), all enqueue-only, return 0 or OASES_E* ---------------
int launch_dropout_mask(uint8_t* mask, const DropCfg& d, int64_t row0, int rows, int h, hipStream_t s);
// rms = true: RMSNorm (no mean, no beta; mu / beta unused and may be NULL); bias may be NULL with rms
int launch_layernorm_fwd(const float* x, const float* gamma, const float* beta, void* out, float* mu,
                         float* rstd, int rows, int h, float eps, hipStream_t s, bool rms = false);
int launch_bdr_ln(const float* part, const float* peer, const float* bias, const float* xin, float* xo,
                  const float* gamma, const float* beta, void* ln_out, float* mu, float* rstd, int rows,
                  int h, float eps, const DropCfg& d, int64_t row0, hipStream_t s, bool rms = false, float* ln_f32 = nullptr);
// post-LN layers: out (bf16) = x (fp32), n elements; out = a + b (+ c) fp32
int launch_cast_bf16(const float* x, void* out, int64_t n, hipStream_t s);
int launch_add3(const float* a, const float* b, const float* c, float* out, int64_t n, hipStream_t s);
// rotary embedding: table [seq][head_dim/2] of (cos, sin) fp32; rotation in place on the Q and K parts of qkv
int launch_rope_table(float* tab, int seq, int head_dim, float theta, hipStream_t s);
int launch_rope(void* qkv, int ld, int rows, int64_t row0, int seq, int heads, int head_dim, const float* tab, int inverse,
                hipStream_t s);
// sink (dropout_bwd, layernorm_bwd, colsum_bf16): nullptr = the second stage of the column sums follows at once
int launch_dropout_bwd(const float* dyin, void* dz, float* dbias, int rows, int h, const DropCfg& d,
                       int64_t row0, float* scratch, hipStream_t s, ColsumSink* sink = nullptr);
int launch_layernorm_bwd(const float* part, const float* peer, const float* dres, const float* x,
                         const float* mu, const float* rstd, const float* gamma, float* dxo, float* dgamma,
                         float* dbeta, void* dz, float* dbias, int rows, int h, const DropCfg& d,
                         int64_t row0, float* scratch, hipStream_t s, bool rms = false, bool post = false, ColsumSink* sink = nullptr);
int launch_colsum_bf16(const void* a, int ld, int rows, int cols, float* out, float* scratch, hipStream_t s, ColsumSink* sink = nullptr);
// splitk_ws: optional fp32 scratch for split-K partial planes (NULL: never split); forced_variant: 0 = choose, else
// the instantiation to launch, encoded as gemm_variant() returns it
// choice_rows > M (NN / NT): the kernel is chosen as for a launch of that many rows, so that launches over parts of those rows
// (sub-batches) add the fp32 terms of an element in one order whatever the part
int launch_gemm(int op, int epi, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C,
                int ldc, const float* bias, void* aux, int ldaux, void* splitk_ws, size_t splitk_ws_bytes, int forced_variant,
                hipStream_t s, int choice_rows = 0);
// the direct-to-LDS kernels address an operand with 32-bit byte offsets: its rows x ld bf16 elements must span less than
// 2 GiB, or the launcher takes the register-staged kernel of the same tile
inline bool gemm_span_fits(long rows, long ld) { return rows * ld * 2 < (1L << 31); }
int gemm_variant(int op, int epi, int M, int N, int K, size_t ws_bytes);  // 1e8*[waves split k] + 1e6*slices + 1e3*BM + BN
// two TN contractions C_i += A_i^T B_i over the same K rows in one launch of the 128x256 direct-to-LDS kernel, and the
// host rule that says when that beats two launches (both fit whole tiles, fewer rounds of workgroups together)
int launch_gemm_tn_pair(int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0, void* C0, int ldc0, int M1, int N1,
                        const void* A1, int lda1, const void* B1, int ldb1, void* C1, int ldc1, hipStream_t s);
bool gemm_tn_pair_wins(int K, int M0, int N0, int M1, int N1);
constexpr size_t kSplitKWorkspaceBytes = 256u << 20;
// p_attn > 0: dropout on the probabilities (mask keyed by seed, layer, sequence, global head = head0 + local head, q, k)
int launch_attention_fwd(const void* qkv, void* out, float* lse, int batch, int seq, int heads, int head_dim,
                         int causal, int row0, int rows, hipStream_t s, uint64_t seed = 0, int layer = 0, float p_attn = 0.f,
                         int head0 = 0, int heads_total = 0);
int launch_attention_bwd(const void* qkv, const void* out, const void* dout, const float* lse, float* delta,
                         void* dqkv, int batch, int seq, int heads, int head_dim, int causal, int row0,
                         int rows, hipStream_t s, uint64_t seed = 0, int layer = 0, float p_attn = 0.f, int head0 = 0,
                         int heads_total = 0);

constexpr int kColPartials = 1024;  // row-groups of the two-stage column reductions

}  // namespace oases
