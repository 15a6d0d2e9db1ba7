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

}  // namespace
}  // namespace oases

using namespace oases;

extern "C" int oases_probe_mfma_rate(int random_operands, int iters, int workgroups, void* out, void* stream) {
  if (iters <= 0 || workgroups <= 0) { set_error("oases_probe_mfma_rate: iters and workgroups must be positive"); return OASES_EINVAL; }
  if (!out) { set_error("oases_probe_mfma_rate: NULL output"); return OASES_ENULL; }
  hipLaunchKernelGGL((mfma_rate_kernel<8>), dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (float*)out, iters, random_operands);
  OASES_LAUNCH_CHECK("mfma_rate_kernel");
  return 0;
}
