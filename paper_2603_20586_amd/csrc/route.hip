// Router kernel: Alg. 2 step 5 of the paper — gates lam = softmax_3(Q W_r + b_r), one triple
// per token, plus the argmax of the logits; also the routing variants of the paper's ablation
// (section "Routing Mechanism Ablation": fixed 1/3, hard top-2, hard top-1).
//
// One lane owns one query row.  The logits are an fp64 fma chain in ascending k that starts
// from the bias; every product bf16*f32 or f32*f32 is exact in fp64 and each fma is correctly
// rounded, so the logits (hence the argmax) are reproducible bit for bit by any other
// implementation that uses the same chain.  A wave stages its 64 rows through LDS so that the
// global reads are coalesced 16-byte loads; the kernel is bound by reading Q once.
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

template <typename T, int D>
__global__ __launch_bounds__(64) void route_kernel(const T* __restrict__ Q,
                                                   const float* __restrict__ W_r,
                                                   const float* __restrict__ b_r,
                                                   float* __restrict__ G, int32_t* __restrict__ idx,
                                                   long rows, int Tq, int S, int mode) {
  constexpr int ROWB = D * (int)sizeof(T);   // bytes per row
  constexpr int STR = ROWB + 16;             // padded LDS row stride (bytes)
  constexpr int CPR = ROWB / 16;             // 16-byte chunks per row
  constexpr int EPC = 16 / (int)sizeof(T);   // elements per chunk
  __shared__ __attribute__((aligned(16))) unsigned char sq[64 * STR];
  __shared__ double sw[D * 3];
  const int lane = threadIdx.x;
  const long row0 = (long)blockIdx.x * 64;
  for (int i = lane; i < D * 3; i += 64) sw[i] = (double)W_r[i];
  // coalesced copy of up to 64 rows into LDS
  const unsigned char* src = reinterpret_cast<const unsigned char*>(Q) + row0 * ROWB;
  const long nrows = (rows - row0) < 64 ? (rows - row0) : 64;
  for (int c = lane; c < 64 * CPR; c += 64) {
    const int r = c / CPR, cc = c % CPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < nrows) v = *reinterpret_cast<const uint4*>(src + (long)r * ROWB + cc * 16);
    *reinterpret_cast<uint4*>(&sq[r * STR + cc * 16]) = v;
  }
  __syncthreads();
  const long row = row0 + lane;
  if (row >= rows) return;
  double g0 = b_r ? (double)b_r[0] : 0.0;
  double g1 = b_r ? (double)b_r[1] : 0.0;
  double g2 = b_r ? (double)b_r[2] : 0.0;
  const unsigned char* myrow = &sq[lane * STR];
#pragma unroll 2
  for (int cc = 0; cc < CPR; ++cc) {
    const uint4 u = *reinterpret_cast<const uint4*>(myrow + cc * 16);
    float f[8];
    if constexpr (sizeof(T) == 2) {
      unpack8(u, f);
    } else {
      f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
      f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      const int k = cc * EPC + e;
      const double q = (double)f[e];
      g0 = fma(q, sw[k * 3 + 0], g0);
      g1 = fma(q, sw[k * 3 + 1], g1);
      g2 = fma(q, sw[k * 3 + 2], g2);
    }
  }
  float lam[3];
  const int best = gates_variant(g0, g1, g2, mode, lam);
  if (idx) idx[row] = best;
  if (G) {
    const long bh = row / Tq;
    const int t = (int)(row - bh * Tq);
    float* out = G + (bh * S + (S - Tq) + t) * 3;
    out[0] = lam[0];
    out[1] = lam[1];
    out[2] = lam[2];
  }
}

hipError_t launch_route(const RouteArgs& a, hipStream_t st) {
  const long rows = (long)a.BH * a.Tq;
  if (rows == 0) return hipSuccess;
  const unsigned grid = (unsigned)((rows + 63) / 64);
#define MKA_ROUTE(T, D)                                                                        \
  hipLaunchKernelGGL((route_kernel<T, D>), dim3(grid), dim3(64), 0, st, (const T*)a.Q, a.W_r, \
                     a.b_r, a.G, a.idx, rows, a.Tq, a.S, a.mode)
  if (a.bf16) {
    if (a.d == 128) MKA_ROUTE(bf16, 128); else MKA_ROUTE(bf16, 64);
  } else {
    if (a.d == 128) MKA_ROUTE(float, 128); else MKA_ROUTE(float, 64);
  }
#undef MKA_ROUTE
  return hipGetLastError();
}

}  // namespace mka
