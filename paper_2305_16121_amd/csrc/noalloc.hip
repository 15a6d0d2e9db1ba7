// Allocation-free variant of the bf16 column sum (bias gradients): the partial-sum rows that the two-stage reduction
// keeps between its kernels live in a file-scope device array instead of a caller-provided scratch buffer, for callers
// that can neither allocate device memory nor carry a workspace (code under HIP graph capture, tight serving loops).
#include <mutex>

#include "common.h"

namespace oases {
namespace {

// [kColPartials row groups][kStaticColsumMaxCols columns] fp32 partial sums = 16 MiB, held by every GPU the library runs
// on until the process ends.
constexpr int kStaticColsumMaxCols = 4096;
constexpr size_t kStaticScratchFloats = (size_t)kColPartials * kStaticColsumMaxCols;
static __device__ __attribute__((used)) __align__(256) float scratch[kStaticScratchFloats];

// Device address of `scratch` per GPU: the array's name is only a host-side stand-in, so the address is asked for once
// per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int static_scratch(float** out) {
  int dev = -1;
  OASES_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) { set_error("colsum_bf16_static: device index %d unsupported (max %d)", dev, kMaxDevices - 1); return OASES_EINVAL; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    OASES_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) { set_error("colsum_bf16_static: hipGetSymbolAddress returned a NULL address"); return OASES_EHIP; }
    g_scratch_ptr[dev] = reinterpret_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

}  // namespace
}  // namespace oases

using namespace oases;

extern "C" int oases_op_colsum_bf16_static(const void* a, int ld, int rows, int cols, void* out, void* stream) {
  if (cols > kStaticColsumMaxCols) {
    set_error("colsum_bf16_static: %d columns exceed the static scratch (at most %d)", cols, kStaticColsumMaxCols);
    return OASES_EWORKSPACE;
  }
  float* ptr = nullptr;
  const int rc = static_scratch(&ptr);
  if (rc) return rc;
  // the kernels take the device address, exactly as they take the caller's scratch in oases_op_colsum_bf16; every partial
  // row that the second kernel reads is written by the first one of the same call, so nothing has to be cleared
  return launch_colsum_bf16(a, ld, rows, cols, (float*)out, ptr, (hipStream_t)stream);
}
