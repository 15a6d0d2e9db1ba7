// Measurement helper: the rate at which this part sustains v_mfma_f32_32x32x16_bf16 from registers, with no memory traffic
// at all -- the ceiling that any GEMM on it sits under.  On a power-capped part the rate depends on the operand VALUES
// (the clock drops when many bits toggle), so the operands are either all zero or pseudo-random, roughly normal values.
#include "common.h"

namespace oases {
namespace {

template <int NACC>
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* out, int iters, int random_operands) {
  f32x16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
  // operand registers of this lane: a sum of four 16-bit uniforms, centred and scaled to unit variance, as bf16
  u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
  if (random_operands) {
    const uint32_t id = blockIdx.x * 256u + threadIdx.x;
    Philox4 wa = philox4x32_10(id, 0u, 1u, 0u, 0x1234u, 0x5678u), wb = philox4x32_10(id, 0u, 2u, 0u, 0x1234u, 0x5678u);
    Philox4 wc = philox4x32_10(id, 0u, 3u, 0u, 0x1234u, 0x5678u), wd = philox4x32_10(id, 0u, 4u, 0u, 0x1234u, 0x5678u);
    auto normalish = [](uint32_t w0, uint32_t w1) {
      const float s = (float)(w0 & 0xffffu) + (float)(w0 >> 16) + (float)(w1 & 0xffffu) + (float)(w1 >> 16);
      return (s * (1.0f / 65536.0f) - 2.0f) * 1.7320508f;
    };
#pragma unroll
    for (int j = 0; j < 4; j++) {
      a[j] = pack_bf16x2(normalish(wa.v[j], wb.v[j]), normalish(wb.v[j], wc.v[j]));
      b[j] = pack_bf16x2(normalish(wc.v[j], wd.v[j]), normalish(wd.v[j], wa.v[j]));
    }
  }
  const bf16x8 fa = __builtin_bit_cast(bf16x8, a), fb = __builtin_bit_cast(bf16x8, b);
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < NACC; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) s += acc[i][e];
  if (out) out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;   // keeps the loop alive
}

// Rate at which one workgroup per CU pulls L2-resident data straight into LDS (global_load_lds_dwordx4, 1 KB per wave
// instruction): the ceiling under which the operand streams of the GEMMs sit.  Workgroup b sweeps its own 64 KB of `src`
// (16 rows of 4 KB; resident in its XCD's L2 after the first sweep) iters times; the data is never read.
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void lds_load_rate_kernel(const char* __restrict__ src, int iters, float* out) {
  __shared__ __attribute__((aligned(1024))) char lds[WAVES * 8192];
  typedef const void __attribute__((address_space(1))) * gptr_t;
  typedef void OASES_LDS* lptr_t;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const char* base = src + (size_t)blockIdx.x * 65536 + lane * 16;
  char* my = lds + wave * 8192;
  uint32_t p = wave * 8;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int j = 0; j < 8; j++) __builtin_amdgcn_global_load_lds((gptr_t)(base + ((p + j) & 63u) * 1024u), (lptr_t)(my + j * 1024), 16, 0, 0);
    p += WAVES * 8;
    __builtin_amdgcn_s_waitcnt(8 | (7 << 4) | (15 << 8));   // vmcnt(8): the previous batch of eight has landed
  }
  __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));
  __syncthreads();
  if (out && reinterpret_cast<const uint32_t*>(lds)[threadIdx.x] == 0x12345678u) out[threadIdx.x] = 1.f;   // keeps the loads alive
}

}  // namespace
}  // namespace oases

using namespace oases;

extern "C" int oases_probe_lds_load_rate(int waves, int iters, int workgroups, const void* src, size_t src_bytes, void* out, void* stream) {
  if ((waves != 4 && waves != 8) || iters <= 0 || workgroups <= 0) { set_error("oases_probe_lds_load_rate: waves must be 4 or 8, iters and workgroups positive"); return OASES_EINVAL; }
  if (!src || !out) { set_error("oases_probe_lds_load_rate: NULL argument"); return OASES_ENULL; }
  if (src_bytes < (size_t)workgroups * 65536) { set_error("oases_probe_lds_load_rate: src holds less than 64 KiB per workgroup"); return OASES_EINVAL; }
  if (!aligned16(src)) { set_error("oases_probe_lds_load_rate: src not 16-byte aligned"); return OASES_EALIGN; }
  if (waves == 4) hipLaunchKernelGGL((lds_load_rate_kernel<4>), dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (const char*)src, iters, (float*)out);
  else hipLaunchKernelGGL((lds_load_rate_kernel<8>), dim3(workgroups), dim3(512), 0, (hipStream_t)stream, (const char*)src, iters, (float*)out);
  OASES_LAUNCH_CHECK("lds_load_rate_kernel");
  return 0;
}

extern "C" int oases_probe_mfma_rate(int random_operands, int iters, int workgroups, void* out, void* stream) {
  if (iters <= 0 || workgroups <= 0) { set_error("oases_probe_mfma_rate: iters and workgroups must be positive"); return OASES_EINVAL; }
  if (!out) { set_error("oases_probe_mfma_rate: NULL output"); return OASES_ENULL; }
  hipLaunchKernelGGL((mfma_rate_kernel<8>), dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (float*)out, iters, random_operands);
  OASES_LAUNCH_CHECK("mfma_rate_kernel");
  return 0;
}
