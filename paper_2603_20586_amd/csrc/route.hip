// Router kernel: Alg. 2 step 5 of the paper — gates lam = softmax_3(Q W_r + b_r), one triple
// per token, plus the argmax of the logits; also the routing variants of the paper's ablation
// (section "Routing Mechanism Ablation": fixed 1/3, hard top-2, hard top-1).
//
// One lane owns one query row.  The logits are an fp64 fma chain in ascending k that starts
// from the bias; every product bf16*f32 or f32*f32 is exact in fp64 and each fma is correctly
// rounded, so the logits (hence the argmax) are reproducible bit for bit by any other
// implementation that uses the same chain.  A lane reads its row straight from global memory,
// 16 bytes at a time and four chunks ahead (a wave instruction touches 64 rows; the four
// instructions that share a 64-byte sector hit in the vector cache), and W_r through scalar
// loads (a uniform address), widened to fp64 on the way into the fma: no LDS, no barrier, so
// the waves of a compute unit overlap their loads and chains freely.  Measured against the
// earlier version (64 rows staged through LDS per single-wave workgroup, W_r as an fp64 table in
// LDS, 8-9 waves per compute unit): 29 us instead of 43 us for the 524 288 rows of the training
// config in a loop of back-to-back launches (4.6 TB/s of Q; unroll 2 / 8 and 64 / 256 rows per
// workgroup measured, this is the best).
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

constexpr int RT_WG = 128;  // rows (threads) per workgroup

template <typename T, int D>
__global__ __launch_bounds__(RT_WG) void route_kernel(const T* __restrict__ Q,
                                                      const float* __restrict__ W_r,
                                                      const float* __restrict__ b_r,
                                                      float* __restrict__ G,
                                                      int32_t* __restrict__ idx, long rows, int Tq,
                                                      int S, int mode) {
  constexpr int ROWB = D * (int)sizeof(T);   // bytes per row
  constexpr int CPR = ROWB / 16;             // 16-byte chunks per row
  constexpr int EPC = 16 / (int)sizeof(T);   // elements per chunk
  const long row = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= rows) return;
  double g0 = b_r ? (double)b_r[0] : 0.0;
  double g1 = b_r ? (double)b_r[1] : 0.0;
  double g2 = b_r ? (double)b_r[2] : 0.0;
  const unsigned char* myrow = reinterpret_cast<const unsigned char*>(Q) + row * ROWB;
#pragma unroll 4
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
      // W_r at a uniform address: scalar loads, widened to fp64 on the way into the fma
      g0 = fma(q, (double)W_r[k * 3 + 0], g0);
      g1 = fma(q, (double)W_r[k * 3 + 1], g1);
      g2 = fma(q, (double)W_r[k * 3 + 2], g2);
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
  const unsigned grid = (unsigned)((rows + RT_WG - 1) / RT_WG);
#define MKA_ROUTE(T, D)                                                                        \
  hipLaunchKernelGGL((route_kernel<T, D>), dim3(grid), dim3(RT_WG), 0, st, (const T*)a.Q, a.W_r, \
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
