// Symbolic (full) MKA, Alg. 1 of the paper - the three-path variant that FastMKA replaces - and
// the causal prefix-mean summary that produces its L2 memory.
//
//   a_l = softmax(tau Q K_l^T) V_l  (one attention per memory),   O[t] = sum_l lam[t,l] a_l[t]
//
// The three attentions are launches of the plain attention kernel (the gated-mixture kernel with
// one memory and no gates) into a workspace; this file holds the combine step, which is bound
// by reading the three partial outputs once, and the summary M[t] = mean(X[0..t]), a scan along
// the sequence in three small memory-bound kernels (chunk sums, prefix over the chunks, scan
// inside the chunks).  Because the K / V projections are linear, the L2 keys / values of Alg. 1
// are the prefix mean of the L1 keys / values, which is how the summary is applied here.
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

// ------------------------------------------------------------------ combine
// item = (row, 16-byte chunk); absent levels have a null pointer and contribute nothing
template <int D>
__global__ __launch_bounds__(256) void full_combine_kernel(const bf16* __restrict__ A0,
                                                           const bf16* __restrict__ A1,
                                                           const bf16* __restrict__ A2,
                                                           const float* __restrict__ G,
                                                           bf16* __restrict__ O, long rows) {
  constexpr int CPR = D / 8;
  const long item = (long)blockIdx.x * 256 + threadIdx.x;
  const long row = item / CPR;
  const int cc = (int)(item % CPR);
  if (row >= rows) return;
  const bf16* A[3] = {A0, A1, A2};
  uint4 raw[3];
#pragma unroll
  for (int l = 0; l < 3; ++l)
    raw[l] = A[l] ? *reinterpret_cast<const uint4*>(A[l] + row * D + cc * 8) : make_uint4(0, 0, 0, 0);
  const float g[3] = {G[row * 3 + 0], G[row * 3 + 1], G[row * 3 + 2]};
  float o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
  for (int l = 0; l < 3; ++l) {
    if (!A[l]) continue;
    float f[8];
    unpack8(raw[l], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = fmaf(g[l], f[e], o[e]);
  }
  *reinterpret_cast<uint4*>(O + row * D + cc * 8) = pack8(o);
}

// ------------------------------------------------------------------ prefix mean
constexpr int PM_C = 64;  // rows per chunk

// column sums of one chunk.  Thread = (16-byte chunk cc, row group rg of 4 rows)
template <int D>
__global__ __launch_bounds__(256) void pm_chunk_sum_kernel(const bf16* __restrict__ X,
                                                           float* __restrict__ csum, int S,
                                                           int nchunks) {
  constexpr int CPR = D / 8, RG = 256 / CPR, RPG = PM_C / RG;  // row groups, rows per group
  __shared__ float part[RG][D + 4];
  const int tid = threadIdx.x, cc = tid % CPR, rg = tid / CPR;
  const long bh = blockIdx.x / nchunks;
  const int ch = blockIdx.x % nchunks;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
  for (int u = 0; u < RPG; ++u) {
    const int t = ch * PM_C + rg * RPG + u;
    if (t < S) {
      float f[8];
      unpack8(*reinterpret_cast<const uint4*>(X + (bh * S + t) * D + cc * 8), f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += f[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][cc * 8 + e] = acc[e];
  __syncthreads();
  for (int k = tid; k < D; k += 256) {
    float s = 0.f;
    for (int r = 0; r < RG; ++r) s += part[r][k];  // fixed order
    csum[((long)bh * nchunks + ch) * D + k] = s;
  }
}

// exclusive prefix over the chunk sums of one (batch, head), in place; thread = column
__global__ __launch_bounds__(128) void pm_chunk_prefix_kernel(float* __restrict__ csum, int nchunks,
                                                              int D) {
  const long bh = blockIdx.x;
  for (int k = threadIdx.x; k < D; k += 128) {
    float run = 0.f;
    for (int ch = 0; ch < nchunks; ++ch) {
      float* p = csum + (bh * nchunks + ch) * D + k;
      const float v = *p;
      *p = run;
      run += v;
    }
  }
}

// scan inside a chunk on top of the chunk's offset, divide by the row count, round once
template <int D>
__global__ __launch_bounds__(256) void pm_scan_kernel(const bf16* __restrict__ X,
                                                      const float* __restrict__ coff,
                                                      bf16* __restrict__ M, int S, int nchunks) {
  constexpr int CPR = D / 8, RG = 256 / CPR, RPG = PM_C / RG;
  __shared__ float part[RG][D + 4];
  const int tid = threadIdx.x, cc = tid % CPR, rg = tid / CPR;
  const long bh = blockIdx.x / nchunks;
  const int ch = blockIdx.x % nchunks;
  float run[RPG][8];
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
  for (int u = 0; u < RPG; ++u) {
    const int t = ch * PM_C + rg * RPG + u;
    if (t < S) {
      float f[8];
      unpack8(*reinterpret_cast<const uint4*>(X + (bh * S + t) * D + cc * 8), f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += f[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) run[u][e] = acc[e];  // inclusive inside the row group
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][cc * 8 + e] = acc[e];
  __syncthreads();
  float base[8];
  const float* off = coff + ((long)bh * nchunks + ch) * D + cc * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float s = off[e];
    for (int r = 0; r < rg; ++r) s += part[r][cc * 8 + e];  // row groups before this one
    base[e] = s;
  }
#pragma unroll
  for (int u = 0; u < RPG; ++u) {
    const int t = ch * PM_C + rg * RPG + u;
    if (t < S) {
      const float inv = 1.0f / (float)(t + 1);
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (base[e] + run[u][e]) * inv;
      *reinterpret_cast<uint4*>(M + (bh * S + t) * D + cc * 8) = pack8(o);
    }
  }
}

}  // namespace

hipError_t launch_full_combine(const void* const A[3], const float* G, void* O, long rows, int d,
                               hipStream_t st) {
  if (rows == 0) return hipSuccess;
  const int cpr = d / 8;
  const unsigned grid = (unsigned)((rows * cpr + 255) / 256);
  if (d == 128)
    hipLaunchKernelGGL((full_combine_kernel<128>), dim3(grid), dim3(256), 0, st, (const bf16*)A[0],
                       (const bf16*)A[1], (const bf16*)A[2], G, (bf16*)O, rows);
  else
    hipLaunchKernelGGL((full_combine_kernel<64>), dim3(grid), dim3(256), 0, st, (const bf16*)A[0],
                       (const bf16*)A[1], (const bf16*)A[2], G, (bf16*)O, rows);
  return hipGetLastError();
}

size_t prefix_mean_workspace_bytes(int BH, int S, int d) {
  const size_t nchunks = (size_t)(S + PM_C - 1) / PM_C;
  return ((size_t)BH * nchunks * d * sizeof(float) + 255) & ~(size_t)255;
}

hipError_t launch_prefix_mean(const void* X, void* M, int BH, int S, int d, void* workspace,
                              hipStream_t st) {
  if (BH == 0 || S == 0) return hipSuccess;
  const int nchunks = (S + PM_C - 1) / PM_C;
  float* cs = static_cast<float*>(workspace);
  const unsigned grid = (unsigned)((long)BH * nchunks);
  if (d == 128)
    hipLaunchKernelGGL((pm_chunk_sum_kernel<128>), dim3(grid), dim3(256), 0, st, (const bf16*)X, cs, S, nchunks);
  else
    hipLaunchKernelGGL((pm_chunk_sum_kernel<64>), dim3(grid), dim3(256), 0, st, (const bf16*)X, cs, S, nchunks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(pm_chunk_prefix_kernel, dim3((unsigned)BH), dim3(128), 0, st, cs, nchunks, d);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (d == 128)
    hipLaunchKernelGGL((pm_scan_kernel<128>), dim3(grid), dim3(256), 0, st, (const bf16*)X, cs, (bf16*)M, S, nchunks);
  else
    hipLaunchKernelGGL((pm_scan_kernel<64>), dim3(grid), dim3(256), 0, st, (const bf16*)X, cs, (bf16*)M, S, nchunks);
  return hipGetLastError();
}

}  // namespace mka
