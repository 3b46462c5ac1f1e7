// Reference micro-benchmarks of the part, to quote beside the vendor peaks: a pure 32x32x16 bf16
// MFMA loop (no memory traffic) and a streaming read of a large buffer.  Neither is part of the
// method and neither is linked into libmka.so: they form libmka_measure.so, which only bench.py
// loads (sustained clocks under matrix load sit below the datasheet figure, and HBM delivers
// less than its pin rate, so the rooflines are quoted against both).
#include <hip/hip_runtime.h>

#include "../../include/mka_measure.h"
#include "../csrc/mka_dev.h"

namespace mka {
namespace {

// 8 waves per workgroup, 4 independent accumulator chains per wave
__global__ __launch_bounds__(512) void measure_mfma_kernel(float* out, int iters) {
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

// The same loop on operands that change from MFMA to MFMA: every wave holds eight A and eight B
// fragments out of `frags` (the caller fills it with the value distribution of its workload)
// and walks through all pairings.  The board's power limit, not the issue rate, sets the clock
// under matrix load, and the power an MFMA draws depends on how many operand bits toggle: this
// is what the matrix pipe alone sustains on data like the attention kernels'.
__global__ __launch_bounds__(512) void measure_mfma_data_kernel(float* out, const uint4* __restrict__ frags,
                                                                int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = __builtin_bit_cast(bf16x8, frags[(j * 2) * 512 + threadIdx.x]);
    b[j] = __builtin_bit_cast(bf16x8, frags[(j * 2 + 1) * 512 + threadIdx.x]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[k] = mfma32(a[j], b[(j + k) & 7], acc[k]);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  if (out) out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Six streams (the buffer cut in six equal parts), each workgroup walks its slice of all six at
// once: per trip a lane issues 4 x 6 independent 16-byte non-temporal loads before the first use,
// 16 lanes cover 256 consecutive bytes - the decode kernel's traffic without its arithmetic.
__global__ __launch_bounds__(256) void measure_read_kernel(const uint4* __restrict__ src,
                                                           unsigned* out, long per_stream,
                                                           long chunk) {
  constexpr int U = 4, NS = 6;
  const long lo = (long)blockIdx.x * chunk;
  const long hi = lo + chunk < per_stream ? lo + chunk : per_stream;
  unsigned acc = 0;
  for (long i = lo + threadIdx.x; i + 256 * (U - 1) < hi; i += 256 * U) {
    uint4 v[U][NS];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s = 0; s < NS; ++s) v[u][s] = load16_stream(src + s * per_stream + i + 256 * u);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s = 0; s < NS; ++s) acc ^= v[u][s].x ^ v[u][s].y ^ v[u][s].z ^ v[u][s].w;
  }
  if (acc == 0x9e3779b9u && out) out[0] = acc;  // keeps the loads alive, practically never taken
}

}  // namespace
}  // namespace mka

extern "C" int32_t mka_measure_mfma_loop(float* out, int32_t workgroups, int32_t iters,
                                         double* flops, void* stream) {
  if (workgroups <= 0 || iters <= 0 || !out) return 2;
  hipLaunchKernelGGL(mka::measure_mfma_kernel, dim3((unsigned)workgroups), dim3(512), 0,
                     static_cast<hipStream_t>(stream), out, iters);
  if (flops) *flops = (double)workgroups * 8.0 * iters * 4.0 * 32768.0;  // 2*32*32*16 per MFMA
  return hipGetLastError() == hipSuccess ? 0 : 7;
}

extern "C" int32_t mka_measure_mfma_loop_data(float* out, const void* frags, int32_t workgroups,
                                              int32_t iters, double* flops, void* stream) {
  if (workgroups <= 0 || iters <= 0 || !out || !frags) return 2;
  if (reinterpret_cast<uintptr_t>(frags) & 15) return 4;
  hipLaunchKernelGGL(mka::measure_mfma_data_kernel, dim3((unsigned)workgroups), dim3(512), 0,
                     static_cast<hipStream_t>(stream), out, static_cast<const uint4*>(frags), iters);
  if (flops) *flops = (double)workgroups * 8.0 * iters * 32.0 * 32768.0;
  return hipGetLastError() == hipSuccess ? 0 : 7;
}

extern "C" int32_t mka_measure_stream_read(const void* src, size_t bytes, uint32_t* out,
                                           void* stream) {
  if (!src || bytes < (1u << 20)) return 2;
  if (reinterpret_cast<uintptr_t>(src) & 15) return 4;
  // whole 1024-chunk trips per stream (a tail of < 96 KiB is not read), 2048 workgroups
  const long per_stream = (long)(bytes / 16 / 6) / 1024 * 1024;
  const int wgs = 2048;
  long chunk = (per_stream + wgs - 1) / wgs;
  chunk = (chunk + 1023) / 1024 * 1024;
  hipLaunchKernelGGL(mka::measure_read_kernel, dim3(wgs), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), out,
                     per_stream, chunk);
  return hipGetLastError() == hipSuccess ? 0 : 7;
}
