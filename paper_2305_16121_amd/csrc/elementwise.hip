// HBM-bound kernels of the layer: LayerNorm forward/backward, the fused
// reduction-point + bias + dropout + residual (+ LayerNorm) step, dropout backward, and the
// two-stage (deterministic) column reductions that give bias / LayerNorm-parameter gradients.
// One 256-thread workgroup walks whole rows with 16-byte accesses; a row stays in registers
// between its reduction and its write, so every tensor is read once and written once.
#include "common.h"

namespace oases {

namespace {

constexpr int NT = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// sum over the NW*64 threads of the workgroup, result in every thread; red: 2 x NW floats of LDS
template <int NW = 4>
__device__ __forceinline__ void block_sum2(float& a, float& b, float* red) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();  // red may still be read by the previous use
  if (lane == 0) { red[w] = a; red[NW + w] = b; }
  __syncthreads();
  a = 0.f;
  b = 0.f;
#pragma unroll
  for (int i = 0; i < NW; i++) { a += red[i]; b += red[NW + i]; }
}

__device__ __forceinline__ void store_bf16x4(uint16_t* p, float a, float b, float c, float d) {
  u32x2 v = {pack_bf16x2(a, b), pack_bf16x2(c, d)};
  *reinterpret_cast<u32x2*>(p) = v;
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void dropout_mask_kernel(uint8_t* mask, DropCfg d, uint64_t q0, int64_t nq) {
  int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= nq) return;
  bool k[4];
  dropout_keep4(d, q0 + (uint64_t)i, k);
  uint32_t v = (uint32_t)k[0] | ((uint32_t)k[1] << 8) | ((uint32_t)k[2] << 16) | ((uint32_t)k[3] << 24);
  reinterpret_cast<uint32_t*>(mask)[i] = v;
}

// ------------------------------------------------------------------------------------------------
// xo = xin + keep * (part + peer + bias) * scale   (if part != nullptr; else the row is xin itself; bias may be NULL)
// ln_out = gamma * (xo - mu) * rstd + beta          (if ln_out != nullptr; bf16), the same in fp32 to ln_f32 if given
// RMS: ln_out = gamma * xo * rstd with rstd = 1/sqrt(mean(xo^2) + eps) (RMSNorm: no mean, no beta, mu_out unused)
template <int NC, bool RMS>
__global__ __launch_bounds__(NT) void bdr_ln_kernel(const float* __restrict__ part, const float* __restrict__ peer,
                                                    const float* __restrict__ bias, const float* __restrict__ xin,
                                                    float* __restrict__ xo, const float* __restrict__ gamma,
                                                    const float* __restrict__ beta, uint16_t* __restrict__ ln_out,
                                                    float* __restrict__ mu_out, float* __restrict__ rstd_out, int h,
                                                    float eps, DropCfg d, int64_t row0, float* __restrict__ ln_f32) {
  __shared__ float red[8];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int nc = h >> 2;
  const size_t base = (size_t)row * h;
  f32x4 v[NC];
  // mean and variance in ONE reduction: moments of (x - shift) with shift = first element of the row that is
  // normalised (a value within a few standard deviations of the mean, so E[d^2] - E[d]^2 does not cancel).  Every
  // thread rebuilds that element itself, so the statistics are the same function of the row whether the row was
  // just produced here (fused reduction point) or is read back later (LayerNorm alone, recomputation).
  float shift = RMS ? 0.f : xin[base];
  if (!RMS && part) {
    float z0 = part[base] + (bias ? bias[0] : 0.f);
    if (peer) z0 += peer[base];
    bool k0[4];
    dropout_keep4(d, (uint64_t)(row0 + row) * h >> 2, k0);
    if (k0[0]) shift += z0 * d.scale;
  }
  float s = 0.f, q = 0.f;
#pragma unroll
  for (int i = 0; i < NC; i++) {
    const int c = tid + i * NT;
    v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (c < nc) {
      f32x4 x = *reinterpret_cast<const f32x4*>(xin + base + 4 * c);
      if (part) {
        f32x4 z = *reinterpret_cast<const f32x4*>(part + base + 4 * c);
        if (peer) z += *reinterpret_cast<const f32x4*>(peer + base + 4 * c);
        if (bias) z += *reinterpret_cast<const f32x4*>(bias + 4 * c);
        bool k[4];
        dropout_keep4(d, ((uint64_t)(row0 + row) * h >> 2) + c, k);
#pragma unroll
        for (int j = 0; j < 4; j++) x[j] = k[j] ? x[j] + z[j] * d.scale : x[j];
        *reinterpret_cast<f32x4*>(xo + base + 4 * c) = x;
      }
      v[i] = x;
#pragma unroll
      for (int j = 0; j < 4; j++) { float t = x[j] - shift; s += t; q += t * t; }
    }
  }
  if (!ln_out && !ln_f32) return;
  block_sum2(s, q, red);
  const float ms = RMS ? 0.f : s / h;
  const float mu = shift + ms;
  const float rstd = rsqrtf(fmaxf(q / h - ms * ms, 0.f) + eps);
  if (tid == 0) {
    if (!RMS) mu_out[row] = mu;
    rstd_out[row] = rstd;
  }
#pragma unroll
  for (int i = 0; i < NC; i++) {
    const int c = tid + i * NT;
    if (c < nc) {
      f32x4 gm = *reinterpret_cast<const f32x4*>(gamma + 4 * c);
      f32x4 bt = f32x4{0.f, 0.f, 0.f, 0.f};
      if (!RMS) bt = *reinterpret_cast<const f32x4*>(beta + 4 * c);
      f32x4 o;
#pragma unroll
      for (int j = 0; j < 4; j++) o[j] = gm[j] * ((v[i][j] - mu) * rstd) + bt[j];
      if (ln_out) store_bf16x4(ln_out + base + 4 * c, o[0], o[1], o[2], o[3]);
      if (ln_f32) *reinterpret_cast<f32x4*>(ln_f32 + base + 4 * c) = o;   // post-LN layers: the normalised row is the residual stream
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dz = keep * dyin * scale (bf16); partial column sums of the unrounded dz into scratch[group][h]
template <int NC, int NT>
__global__ __launch_bounds__(NT) void dropout_bwd_kernel(const float* __restrict__ dyin, uint16_t* __restrict__ dz,
                                                         float* __restrict__ scratch, int rows, int h, DropCfg d,
                                                         int64_t row0) {
  const int tid = threadIdx.x, nc = h >> 2;
  f32x4 acc[NC];
#pragma unroll
  for (int i = 0; i < NC; i++) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int row = blockIdx.x; row < rows; row += gridDim.x) {
    const size_t base = (size_t)row * h;
#pragma unroll
    for (int i = 0; i < NC; i++) {
      const int c = tid + i * NT;
      if (c < nc) {
        f32x4 g = *reinterpret_cast<const f32x4*>(dyin + base + 4 * c);
        bool k[4];
        dropout_keep4(d, ((uint64_t)(row0 + row) * h >> 2) + c, k);
#pragma unroll
        for (int j = 0; j < 4; j++) g[j] = k[j] ? g[j] * d.scale : 0.f;
        store_bf16x4(dz + base + 4 * c, g[0], g[1], g[2], g[3]);
        acc[i] += g;
      }
    }
  }
  if (scratch) {
#pragma unroll
    for (int i = 0; i < NC; i++) {
      const int c = tid + i * NT;
      if (c < nc) *reinterpret_cast<f32x4*>(scratch + (size_t)blockIdx.x * h + 4 * c) = acc[i];
    }
  }
}

// out[c] += sum over the partial rows src[g][c], g < groups, for every job of the list
struct FinalizeArgs {
  ColsumJob job[kMaxColsumJobs];
  int n;
};
__global__ __launch_bounds__(NT) void colsum_finalize_kernel(FinalizeArgs a) {
  // one job (blockIdx.y) and 64 columns per workgroup: 16 lanes x 16 bytes cover the 64 columns of a partial row, the 16
  // groups of lanes take the partial rows 16 apart; fixed summation order and tree, so the result does not depend on timing
  __shared__ f32x4 red[16][17];
  const ColsumJob& jb = a.job[blockIdx.y];
  const int cols = jb.cols, groups = jb.groups;
  if (!jb.out || (int)blockIdx.x * 64 >= cols) return;
  const int cx = threadIdx.x & 15, gy = threadIdx.x >> 4;
  const int c = blockIdx.x * 64 + 4 * cx;   // cols is a multiple of 8: a group of four columns is inside or outside
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  if (c < cols) {
    const float* p = jb.src + c;
    int g = gy;
    for (; g + 48 < groups; g += 64) {
      const f32x4 v0 = *reinterpret_cast<const f32x4*>(p + (size_t)g * cols), v1 = *reinterpret_cast<const f32x4*>(p + (size_t)(g + 16) * cols),
                  v2 = *reinterpret_cast<const f32x4*>(p + (size_t)(g + 32) * cols), v3 = *reinterpret_cast<const f32x4*>(p + (size_t)(g + 48) * cols);
      s += (v0 + v1) + (v2 + v3);
    }
    for (; g < groups; g += 16) s += *reinterpret_cast<const f32x4*>(p + (size_t)g * cols);
  }
  red[gy][cx] = s;
  __syncthreads();
  if (gy == 0 && c < cols) {
    f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 16; i++) t += red[i][cx];
    f32x4* o = reinterpret_cast<f32x4*>(jb.out + c);
    *o = *o + t;
  }
}

// ------------------------------------------------------------------------------------------------
// g = part + peer;  dxo = dres + rstd * (g*gamma - mean(g*gamma) - xhat * mean(g*gamma*xhat))
// partials: scratch[0] dgamma = sum g*xhat, scratch[1] dbeta = sum g, scratch[2] dbias = sum dz
// RMS: xhat = x * rstd, dxo = dres + rstd * (g*gamma - xhat * mean(g*gamma*xhat)), no dbeta
// POST (post-LN layers): the residual gradient passes through the LayerNorm too: g = part + peer + dres (dres may be
// NULL), dxo = rstd * (g*gamma - mean(g*gamma) - xhat * mean(g*gamma*xhat))
template <int NC, int NT, bool RMS, bool POST>
__global__ __launch_bounds__(NT) void layernorm_bwd_kernel(const float* __restrict__ part, const float* __restrict__ peer,
                                                           const float* __restrict__ dres, const float* __restrict__ x,
                                                           const float* __restrict__ mu, const float* __restrict__ rstd,
                                                           const float* __restrict__ gamma, float* __restrict__ dxo,
                                                           uint16_t* __restrict__ dz, float* __restrict__ scratch, int rows,
                                                           int h, DropCfg d, int64_t row0, int want_dbias, size_t gstride) {
  __shared__ float red[2 * (NT / 64)];
  const int tid = threadIdx.x, nc = h >> 2;
  f32x4 ag[NC], ab[NC], az[NC];
#pragma unroll
  for (int i = 0; i < NC; i++) ag[i] = ab[i] = az[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int row = blockIdx.x; row < rows; row += gridDim.x) {
    const size_t base = (size_t)row * h;
    const float m = RMS ? 0.f : mu[row], rs = rstd[row];
    f32x4 gg[NC], xh[NC], dr[NC];
    uint32_t kb[NC];  // keep bits of the row's dropout mask: integer work done while the row's loads are in flight
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NC; i++) {
      const int c = tid + i * NT;
      gg[i] = xh[i] = dr[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      kb[i] = 0u;
      if (c < nc) {
        f32x4 g = *reinterpret_cast<const f32x4*>(part + base + 4 * c);
        if (peer) g += *reinterpret_cast<const f32x4*>(peer + base + 4 * c);
        f32x4 xv = *reinterpret_cast<const f32x4*>(x + base + 4 * c);
        if (!POST || dres) dr[i] = *reinterpret_cast<const f32x4*>(dres + base + 4 * c);   // pre-LN: needed only after the reduction, fetched now
        if (POST) g += dr[i];
        f32x4 gm = *reinterpret_cast<const f32x4*>(gamma + 4 * c);
        if (dz) {
          bool k[4];
          dropout_keep4(d, ((uint64_t)(row0 + row) * h >> 2) + c, k);
          kb[i] = (uint32_t)k[0] | ((uint32_t)k[1] << 1) | ((uint32_t)k[2] << 2) | ((uint32_t)k[3] << 3);
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
          xh[i][j] = (xv[j] - m) * rs;
          ag[i][j] += g[j] * xh[i][j];
          ab[i][j] += g[j];
          gg[i][j] = g[j] * gm[j];
          s1 += gg[i][j];
          s2 += gg[i][j] * xh[i][j];
        }
      }
    }
    block_sum2<NT / 64>(s1, s2, red);
    const float m1 = RMS ? 0.f : s1 / h, m2 = s2 / h;
#pragma unroll
    for (int i = 0; i < NC; i++) {
      const int c = tid + i * NT;
      if (c < nc) {
        f32x4 o = POST ? f32x4{0.f, 0.f, 0.f, 0.f} : dr[i];
#pragma unroll
        for (int j = 0; j < 4; j++) o[j] += rs * (gg[i][j] - m1 - xh[i][j] * m2);
        *reinterpret_cast<f32x4*>(dxo + base + 4 * c) = o;
        if (dz) {
#pragma unroll
          for (int j = 0; j < 4; j++) o[j] = ((kb[i] >> j) & 1u) ? o[j] * d.scale : 0.f;
          store_bf16x4(dz + base + 4 * c, o[0], o[1], o[2], o[3]);
          az[i] += o;
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NC; i++) {
    const int c = tid + i * NT;
    if (c < nc) {
      float* p = scratch + (size_t)blockIdx.x * h + 4 * c;
      *reinterpret_cast<f32x4*>(p) = ag[i];
      if (!RMS) *reinterpret_cast<f32x4*>(p + gstride) = ab[i];
      if (dz && want_dbias) *reinterpret_cast<f32x4*>(p + 2 * gstride) = az[i];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// partial column sums of a bf16 matrix; each thread owns 8 columns
__global__ __launch_bounds__(NT) void colsum_bf16_kernel(const uint16_t* __restrict__ a, int ld, int rows, int cols,
                                                         float* __restrict__ scratch) {
  const int c = blockIdx.y * NT + threadIdx.x;  // 8-column chunk
  if (c * 8 >= cols) return;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int row = blockIdx.x; row < rows; row += gridDim.x) {
    u32x4 v = *reinterpret_cast<const u32x4*>(a + (size_t)row * ld + 8 * c);
#pragma unroll
    for (int j = 0; j < 4; j++) {
      acc[2 * j] += bf16_bits_to_f32(v[j] & 0xffffu);
      acc[2 * j + 1] += bf16_bits_to_f32(v[j] >> 16);
    }
  }
  float* p = scratch + (size_t)blockIdx.x * cols + 8 * c;
  *reinterpret_cast<f32x4*>(p) = f32x4{acc[0], acc[1], acc[2], acc[3]};
  *reinterpret_cast<f32x4*>(p + 4) = f32x4{acc[4], acc[5], acc[6], acc[7]};
}

// ------------------------------------------------------------------------------------------------
// Rotary position embedding.  tab[pos][i] = (cos, sin) of pos * theta^(-2i/d), i < d/2, built in fp64.
__global__ __launch_bounds__(NT) void rope_table_kernel(float2* __restrict__ tab, int seq, int half, double log2_theta) {
  const int idx = blockIdx.x * NT + threadIdx.x;
  if (idx >= seq * half) return;
  const int pos = idx / half, i = idx % half;
  const double ang = (double)pos * exp2(-(double)i / (double)half * log2_theta);
  tab[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

// In place on the Q and K parts of qkv [rows, ld] = [Q heads | K heads | V heads]: the pair (i, i + d/2) of every head
// turns by the token's angle (sign = +1), or back (sign = -1: the transpose, which is what a gradient needs).
// One thread owns 8 consecutive i of one head of one row: two 16-byte loads, two 16-byte stores.
__global__ __launch_bounds__(NT) void rope_kernel(uint16_t* __restrict__ qkv, int ld, int rows, int64_t row0, int seq, int heads,
                                                  int d, const float2* __restrict__ tab, float sign) {
  const int half = d >> 1, cpw = half >> 3;  // 8-element chunks per half head
  const int64_t idx = (int64_t)blockIdx.x * NT + threadIdx.x;
  const int64_t per_row = (int64_t)2 * heads * cpw;
  if (idx >= (int64_t)rows * per_row) return;
  const int row = (int)(idx / per_row), r = (int)(idx % per_row);
  const int hd = r / cpw, c = r % cpw;  // hd < 2*heads runs over the Q heads, then the K heads
  const int pos = (int)((row0 + row) % seq);
  uint16_t* p = qkv + (size_t)row * ld + (size_t)hd * d + 8 * c;
  const u32x4 a = *reinterpret_cast<const u32x4*>(p), b = *reinterpret_cast<const u32x4*>(p + half);
  const float2* t = tab + (size_t)pos * half + 8 * c;
  float o1[8], o2[8];
#pragma unroll
  for (int j = 0; j < 8; j++) {
    const float x1 = bf16_bits_to_f32((j & 1) ? a[j >> 1] >> 16 : a[j >> 1] & 0xffffu);
    const float x2 = bf16_bits_to_f32((j & 1) ? b[j >> 1] >> 16 : b[j >> 1] & 0xffffu);
    const float cs = t[j].x, sn = sign * t[j].y;
    o1[j] = x1 * cs - x2 * sn;
    o2[j] = x2 * cs + x1 * sn;
  }
  *reinterpret_cast<u32x4*>(p) = u32x4{pack_bf16x2(o1[0], o1[1]), pack_bf16x2(o1[2], o1[3]), pack_bf16x2(o1[4], o1[5]), pack_bf16x2(o1[6], o1[7])};
  *reinterpret_cast<u32x4*>(p + half) = u32x4{pack_bf16x2(o2[0], o2[1]), pack_bf16x2(o2[2], o2[3]), pack_bf16x2(o2[4], o2[5]), pack_bf16x2(o2[6], o2[7])};
}

// ------------------------------------------------------------------------------------------------
// out (bf16) = x (fp32); n4 groups of 4 elements
__global__ __launch_bounds__(NT) void cast_bf16_kernel(const float* __restrict__ x, uint16_t* __restrict__ out, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n4) return;
  const f32x4 v = *reinterpret_cast<const f32x4*>(x + 4 * i);
  store_bf16x4(out + 4 * i, v[0], v[1], v[2], v[3]);
}
// out = a + b (+ c), fp32
__global__ __launch_bounds__(NT) void add3_kernel(const float* __restrict__ a, const float* __restrict__ b, const float* __restrict__ c,
                                                  float* __restrict__ out, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n4) return;
  f32x4 v = *reinterpret_cast<const f32x4*>(a + 4 * i) + *reinterpret_cast<const f32x4*>(b + 4 * i);
  if (c) v += *reinterpret_cast<const f32x4*>(c + 4 * i);
  *reinterpret_cast<f32x4*>(out + 4 * i) = v;
}

// row groups of a two-stage column reduction: about sixteen rows per group (few partial rows to write and to add up:
// measured faster than eight), but at least one group per CU when the rows allow it, at most kColPartials groups
int col_groups(int rows) {
  int g = rows / 16;
  if (g < 256) g = rows / 2 < 256 ? rows / 2 : 256;
  return g < 1 ? 1 : (g > kColPartials ? kColPartials : g);
}

int pick_nc(int h) {
  const int nc = (h / 4 + NT - 1) / NT;
  for (int c = 1; c <= 16; c *= 2)
    if (nc <= c) return c;
  return 0;
}

bool check_h(int rows, int h, const char* who) {
  if (rows <= 0 || h <= 0 || (h % 8) != 0 || pick_nc(h) == 0) {
    set_error("%s: rows=%d h=%d unsupported (h must be a multiple of 8, at most 16384)", who, rows, h);
    return false;
  }
  return true;
}

// backward kernels: 1024-thread workgroups for wide rows (more bytes in flight per row, fewer registers per thread)
#define OASES_BWD_DISPATCH(H, ...)                                                   \
  if ((H) >= 4096) {                                                                 \
    constexpr int NTHR = 1024;                                                       \
    switch (((H) / 4 + NTHR - 1) / NTHR) {                                           \
      case 1: { constexpr int NC = 1; __VA_ARGS__; break; }                          \
      case 2: { constexpr int NC = 2; __VA_ARGS__; break; }                          \
      default: { constexpr int NC = 4; __VA_ARGS__; break; }                         \
    }                                                                                \
  } else {                                                                           \
    constexpr int NTHR = 256;                                                        \
    switch (pick_nc(H)) {                                                            \
      case 1: { constexpr int NC = 1; __VA_ARGS__; break; }                          \
      case 2: { constexpr int NC = 2; __VA_ARGS__; break; }                          \
      default: { constexpr int NC = 4; __VA_ARGS__; break; }                         \
    }                                                                                \
  }

#define OASES_NC_DISPATCH(NCV, ...)          \
  switch (NCV) {                             \
    case 1: { constexpr int NC = 1; __VA_ARGS__; break; }   \
    case 2: { constexpr int NC = 2; __VA_ARGS__; break; }   \
    case 4: { constexpr int NC = 4; __VA_ARGS__; break; }   \
    case 8: { constexpr int NC = 8; __VA_ARGS__; break; }   \
    default: { constexpr int NC = 16; __VA_ARGS__; break; } \
  }

}  // namespace

DropCfg make_drop_cfg(uint64_t seed, int layer, int site, float p) {
  DropCfg d;
  d.k0 = (uint32_t)seed;
  d.k1 = (uint32_t)(seed >> 32);
  d.site = (uint32_t)site;
  d.layer = (uint32_t)layer;
  double t = (double)p * 16777216.0;
  d.thresh = p > 0.f ? (uint32_t)__builtin_rint(t) : 0u;
  d.scale = (float)(1.0 / (1.0 - (double)p));
  return d;
}

int launch_dropout_mask(uint8_t* mask, const DropCfg& d, int64_t row0, int rows, int h, hipStream_t s) {
  if (!mask) { set_error("dropout_mask: NULL"); return OASES_ENULL; }
  if (rows <= 0 || h <= 0 || h % 4) { set_error("dropout_mask: bad shape"); return OASES_EINVAL; }
  int64_t nq = (int64_t)rows * h / 4;
  hipLaunchKernelGGL(dropout_mask_kernel, dim3((unsigned)((nq + NT - 1) / NT)), dim3(NT), 0, s, mask, d,
                     (uint64_t)row0 * h / 4, nq);
  OASES_LAUNCH_CHECK("dropout_mask_kernel");
  return 0;
}

int launch_bdr_ln(const float* part, const float* peer, const float* bias, const float* xin, float* xo,
                  const float* gamma, const float* beta, void* ln_out, float* mu, float* rstd, int rows, int h,
                  float eps, const DropCfg& d, int64_t row0, hipStream_t s, bool rms, float* ln_f32) {
  if (!check_h(rows, h, "bias_dropout_residual_ln")) return OASES_EINVAL;
  if (!xin || (part && !xo) || (part && !rms && !bias) || ((ln_out || ln_f32) && (!gamma || !rstd || (!rms && (!beta || !mu))))) {
    set_error("bias_dropout_residual_ln: NULL argument");
    return OASES_ENULL;
  }
  if (rms) {
    OASES_NC_DISPATCH(pick_nc(h), hipLaunchKernelGGL((bdr_ln_kernel<NC, true>), dim3(rows), dim3(NT), 0, s, part, peer, bias, xin, xo,
                                                     gamma, beta, (uint16_t*)ln_out, mu, rstd, h, eps, d, row0, ln_f32));
  } else {
    OASES_NC_DISPATCH(pick_nc(h), hipLaunchKernelGGL((bdr_ln_kernel<NC, false>), dim3(rows), dim3(NT), 0, s, part, peer, bias, xin, xo,
                                                     gamma, beta, (uint16_t*)ln_out, mu, rstd, h, eps, d, row0, ln_f32));
  }
  OASES_LAUNCH_CHECK("bdr_ln_kernel");
  return 0;
}

int launch_layernorm_fwd(const float* x, const float* gamma, const float* beta, void* out, float* mu, float* rstd,
                         int rows, int h, float eps, hipStream_t s, bool rms) {
  DropCfg d = make_drop_cfg(0, 0, 0, 0.f);
  if (!out) { set_error("layernorm_fwd: NULL output"); return OASES_ENULL; }
  return launch_bdr_ln(nullptr, nullptr, nullptr, x, nullptr, gamma, beta, out, mu, rstd, rows, h, eps, d, 0, s, rms, nullptr);
}

int colsum_groups(int rows) { return col_groups(rows); }

int launch_colsum_finalize(const ColsumJob* jobs, int n, hipStream_t s) {
  for (int first = 0; first < n; first += kMaxColsumJobs) {
    FinalizeArgs a;
    a.n = n - first < kMaxColsumJobs ? n - first : kMaxColsumJobs;
    int cols = 0;
    for (int i = 0; i < a.n; i++) {
      a.job[i] = jobs[first + i];
      if (a.job[i].out && a.job[i].cols > cols) cols = a.job[i].cols;
    }
    if (cols == 0) continue;
    hipLaunchKernelGGL(colsum_finalize_kernel, dim3((cols + 63) / 64, a.n), dim3(NT), 0, s, a);
    OASES_LAUNCH_CHECK("colsum_finalize_kernel");
  }
  return 0;
}

// the second pass of a column reduction: now (sink == nullptr), or later with the jobs of other reductions in one launch
static int finish_colsums(ColsumSink* sink, float* scratch, size_t kstride, float* o0, float* o1, float* o2, int groups, int cols, hipStream_t s) {
  ColsumJob jobs[3] = {{scratch, o0, groups, cols}, {scratch + kstride, o1, groups, cols}, {scratch + 2 * kstride, o2, groups, cols}};
  if (!sink) return launch_colsum_finalize(jobs, 3, s);
  for (const ColsumJob& j : jobs)
    if (j.out) sink->add(j.out, j.src - (size_t)sink->first_row * cols, sink->rows_total, cols);
  return 0;
}

int launch_dropout_bwd(const float* dyin, void* dz, float* dbias, int rows, int h, const DropCfg& d, int64_t row0,
                       float* scratch, hipStream_t s, ColsumSink* sink) {
  if (!check_h(rows, h, "dropout_bwd")) return OASES_EINVAL;
  if (!dyin || !dz || (dbias && !scratch)) { set_error("dropout_bwd: NULL argument"); return OASES_ENULL; }
  const int groups = col_groups(rows);
  OASES_BWD_DISPATCH(h, hipLaunchKernelGGL((dropout_bwd_kernel<NC, NTHR>), dim3(groups), dim3(NTHR), 0, s, dyin, (uint16_t*)dz,
                                           dbias ? scratch : nullptr, rows, h, d, row0));
  OASES_LAUNCH_CHECK("dropout_bwd_kernel");
  if (dbias) return finish_colsums(sink, scratch, 0, dbias, nullptr, nullptr, groups, h, s);
  return 0;
}

int launch_layernorm_bwd(const float* part, const float* peer, const float* dres, const float* x, const float* mu,
                         const float* rstd, const float* gamma, float* dxo, float* dgamma, float* dbeta, void* dz,
                         float* dbias, int rows, int h, const DropCfg& d, int64_t row0, float* scratch, hipStream_t s, bool rms,
                         bool post, ColsumSink* sink) {
  if (!check_h(rows, h, "layernorm_bwd")) return OASES_EINVAL;
  if (rms && post) { set_error("layernorm_bwd: no post-norm RMS variant"); return OASES_EINVAL; }
  if (!part || (!dres && !post) || !x || !rstd || !gamma || !dxo || !dgamma || !scratch || (!rms && (!mu || !dbeta || (dz && !dbias)))) {
    set_error("layernorm_bwd: NULL argument");
    return OASES_ENULL;
  }
  const int groups = col_groups(rows);
  const int want_dbias = dz && dbias;
  // distance between the three arrays of partial rows: behind one another for this call alone, or as the sink lays them out
  const size_t kstride = sink ? sink->kstride : (size_t)groups * h;
  if (rms) {
    OASES_BWD_DISPATCH(h, hipLaunchKernelGGL((layernorm_bwd_kernel<NC, NTHR, true, false>), dim3(groups), dim3(NTHR), 0, s, part, peer, dres, x,
                                             mu, rstd, gamma, dxo, (uint16_t*)dz, scratch, rows, h, d, row0, want_dbias, kstride));
  } else if (post) {
    OASES_BWD_DISPATCH(h, hipLaunchKernelGGL((layernorm_bwd_kernel<NC, NTHR, false, true>), dim3(groups), dim3(NTHR), 0, s, part, peer, dres, x,
                                             mu, rstd, gamma, dxo, (uint16_t*)dz, scratch, rows, h, d, row0, want_dbias, kstride));
  } else {
    OASES_BWD_DISPATCH(h, hipLaunchKernelGGL((layernorm_bwd_kernel<NC, NTHR, false, false>), dim3(groups), dim3(NTHR), 0, s, part, peer, dres, x,
                                             mu, rstd, gamma, dxo, (uint16_t*)dz, scratch, rows, h, d, row0, want_dbias, kstride));
  }
  OASES_LAUNCH_CHECK("layernorm_bwd_kernel");
  return finish_colsums(sink, scratch, kstride, dgamma, rms ? nullptr : dbeta, want_dbias ? dbias : nullptr, groups, h, s);
}

int launch_cast_bf16(const float* x, void* out, int64_t n, hipStream_t s) {
  if (!x || !out) { set_error("cast_bf16: NULL argument"); return OASES_ENULL; }
  if (n <= 0 || n % 4 || !aligned16(x) || (reinterpret_cast<uintptr_t>(out) & 7u)) { set_error("cast_bf16: n must be a positive multiple of 4, pointers aligned"); return OASES_EINVAL; }
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)((n / 4 + NT - 1) / NT)), dim3(NT), 0, s, x, (uint16_t*)out, n / 4);
  OASES_LAUNCH_CHECK("cast_bf16_kernel");
  return 0;
}

int launch_add3(const float* a, const float* b, const float* c, float* out, int64_t n, hipStream_t s) {
  if (!a || !b || !out) { set_error("add3: NULL argument"); return OASES_ENULL; }
  if (n <= 0 || n % 4 || !aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(out)) { set_error("add3: n must be a positive multiple of 4, pointers 16-byte aligned"); return OASES_EINVAL; }
  hipLaunchKernelGGL(add3_kernel, dim3((unsigned)((n / 4 + NT - 1) / NT)), dim3(NT), 0, s, a, b, c, out, n / 4);
  OASES_LAUNCH_CHECK("add3_kernel");
  return 0;
}

int launch_rope_table(float* tab, int seq, int head_dim, float theta, hipStream_t s) {
  if (!tab) { set_error("rope_table: NULL"); return OASES_ENULL; }
  if (seq <= 0 || head_dim <= 0 || head_dim % 16 || !(theta > 1.f)) { set_error("rope_table: bad argument (head_dim %% 16, theta > 1)"); return OASES_EINVAL; }
  const int n = seq * (head_dim / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + NT - 1) / NT), dim3(NT), 0, s, reinterpret_cast<float2*>(tab), seq, head_dim / 2,
                     log2((double)theta));
  OASES_LAUNCH_CHECK("rope_table_kernel");
  return 0;
}

int launch_rope(void* qkv, int ld, int rows, int64_t row0, int seq, int heads, int head_dim, const float* tab, int inverse,
                hipStream_t s) {
  if (!qkv || !tab) { set_error("rope: NULL argument"); return OASES_ENULL; }
  if (rows <= 0 || seq <= 0 || heads <= 0 || head_dim % 16 || ld % 8 || ld < 3 * heads * head_dim || row0 < 0 || !aligned16(qkv)) {
    set_error("rope: bad shape (head_dim %% 16, ld %% 8, ld >= 3*heads*head_dim)");
    return OASES_EINVAL;
  }
  const int64_t n = (int64_t)rows * 2 * heads * (head_dim / 16);
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((n + NT - 1) / NT)), dim3(NT), 0, s, (uint16_t*)qkv, ld, rows, row0, seq, heads,
                     head_dim, reinterpret_cast<const float2*>(tab), inverse ? -1.f : 1.f);
  OASES_LAUNCH_CHECK("rope_kernel");
  return 0;
}

int launch_colsum_bf16(const void* a, int ld, int rows, int cols, float* out, float* scratch, hipStream_t s, ColsumSink* sink) {
  if (!a || !out || !scratch) { set_error("colsum_bf16: NULL argument"); return OASES_ENULL; }
  if (rows <= 0 || cols <= 0 || cols % 8 || ld % 8 || ld < cols) { set_error("colsum_bf16: bad shape"); return OASES_EINVAL; }
  const int groups = col_groups(rows);
  hipLaunchKernelGGL(colsum_bf16_kernel, dim3(groups, (cols / 8 + NT - 1) / NT), dim3(NT), 0, s, (const uint16_t*)a, ld, rows,
                     cols, scratch);
  OASES_LAUNCH_CHECK("colsum_bf16_kernel");
  return finish_colsums(sink, scratch, 0, out, nullptr, nullptr, groups, cols, s);
}

}  // namespace oases
