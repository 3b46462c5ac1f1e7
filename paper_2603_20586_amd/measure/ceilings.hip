// Measured ceilings of the part, to quote beside the vendor peaks: a pure 32x32x16 bf16 MFMA
// loop (no memory traffic) and a streaming read of a large buffer with 16-byte non-temporal
// loads.  Neither is part of the method; they size the rooflines that the attention kernels
// are held against (sustained clocks under matrix load sit below the datasheet figure).
#include <hip/hip_runtime.h>

#include "../../include/mka.h"
#include "mka_dev.h"

namespace mka {
namespace {

// 8 waves per workgroup, 4 independent accumulator chains per wave
__global__ __launch_bounds__(512) void ceiling_mfma_kernel(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (bf16)(float)((threadIdx.x + e) & 3);
    b[e] = (bf16)(float)((threadIdx.x * 3 + e) & 1);
  }
  f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = mfma32(a, b, acc[k]);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  if (out) out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void ceiling_read_kernel(const uint4* __restrict__ src,
                                                           unsigned* out, long n_chunks) {
  constexpr int U = 8;
  long i = (long)blockIdx.x * 256 * U + threadIdx.x;
  const long stride = (long)gridDim.x * 256 * U;
  unsigned acc = 0;
  for (; i + 256 * (U - 1) < n_chunks; i += stride) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load16_stream(src + i + 256 * u);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u && out) out[0] = acc;  // keeps the loads alive, practically never taken
}

}  // namespace
}  // namespace mka

extern "C" mka_status mka_ceiling_mfma(float* out, int32_t workgroups, int32_t iters,
                                        double* flops, void* stream) {
  if (workgroups <= 0 || iters <= 0 || !out) return MKA_ERR_SHAPE;
  hipLaunchKernelGGL(mka::ceiling_mfma_kernel, dim3((unsigned)workgroups), dim3(512), 0,
                     static_cast<hipStream_t>(stream), out, iters);
  if (flops) *flops = (double)workgroups * 8.0 * iters * 4.0 * 32768.0;  // 2*32*32*16 per MFMA
  return hipGetLastError() == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

extern "C" mka_status mka_ceiling_read(const void* src, size_t bytes, uint32_t* out, void* stream) {
  if (!src || bytes < 16 * 256 * 8) return MKA_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(src) & 15) return MKA_ERR_ALIGN;
  hipLaunchKernelGGL(mka::ceiling_read_kernel, dim3(8192), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), out,
                     (long)(bytes / 16));
  return hipGetLastError() == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}
