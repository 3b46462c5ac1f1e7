// Route-fused attention forward, f32 accuracy path (paper: Alg. 2 steps 6-7 and 9, Eq. (1),
// max-shift recursion over KV tiles).  No matrix cores: this path exists for the 1e-5
// relative-error contract, not for throughput.
//
// A workgroup owns 64 query rows; each row is shared by 4 lanes that split the head dimension
// in interleaved 4-float groups.  Per KV tile of 32 slots the workgroup fuses the three K and
// three V tiles in f32 into LDS; each lane then accumulates its part of the 32 dot products,
// two xor-butterflies complete them, and the online softmax update is done per tile with an
// accurate expf.
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

template <int D>
__global__ __launch_bounds__(256) void fwd_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K0, const float* __restrict__ K1,
    const float* __restrict__ K2, const float* __restrict__ V0, const float* __restrict__ V1,
    const float* __restrict__ V2, const float* __restrict__ G, float* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S, int len0, int len1, int len2, int causal, float tau,
    int n_qtiles) {
  constexpr int BR = 64, BCF = 32, NT = 256;
  constexpr int DL = D / 4;   // floats per lane
  constexpr int NG = DL / 4;  // float4 groups per lane
  constexpr int CPR = D / 4;  // float4 chunks per row
  __shared__ __attribute__((aligned(16))) float sK[BCF * D];
  __shared__ __attribute__((aligned(16))) float sV[BCF * D];

  const int tid = threadIdx.x, part = tid & 3;
  const int qt = n_qtiles - 1 - (int)(blockIdx.x % n_qtiles);
  const long bh = blockIdx.x / n_qtiles;
  const int off = S - Tq;
  const int tq = qt * BR + (tid >> 2);
  const long kvbase = bh * (long)S * D;
  const float* Gb = G + bh * (long)S * 3;

  float4 q[NG];
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    q[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (tq < Tq)
      q[i] = *reinterpret_cast<const float4*>(Q + (bh * (long)Tq + tq) * D + 4 * (part + 4 * i));
  }
  float4 acc[NG];
#pragma unroll
  for (int i = 0; i < NG; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  float m = -INFINITY, lsum = 0.f;

  int t_last = qt * BR + BR - 1;
  if (t_last > Tq - 1) t_last = Tq - 1;
  int j_end = S;
  if (causal && t_last + off + 1 < S) j_end = t_last + off + 1;
  const int ntiles = (j_end + BCF - 1) / BCF;
  const int jmax = causal ? (tq + off < S - 1 ? tq + off : S - 1) : S - 1;

  for (int jt = 0; jt < ntiles; ++jt) {
    const int j0 = jt * BCF;
    __syncthreads();
    for (int it = tid; it < BCF * CPR; it += NT) {
      const int row = it / CPR, cc = it % CPR;
      const int j = j0 + row;
      float4 kf = make_float4(0.f, 0.f, 0.f, 0.f), vf = kf;
      if (j < S) {
        const long eoff = kvbase + (long)j * D + cc * 4;
        const float g[3] = {Gb[j * 3 + 0], Gb[j * 3 + 1], Gb[j * 3 + 2]};
        const float* Kp[3] = {K0, K1, K2};
        const float* Vp[3] = {V0, V1, V2};
        const int len[3] = {len0, len1, len2};
#pragma unroll
        for (int l = 0; l < 3; ++l) {
          if (j < len[l]) {
            const float4 a = *reinterpret_cast<const float4*>(Kp[l] + eoff);
            const float4 b = *reinterpret_cast<const float4*>(Vp[l] + eoff);
            kf.x = fmaf(g[l], a.x, kf.x); kf.y = fmaf(g[l], a.y, kf.y);
            kf.z = fmaf(g[l], a.z, kf.z); kf.w = fmaf(g[l], a.w, kf.w);
            vf.x = fmaf(g[l], b.x, vf.x); vf.y = fmaf(g[l], b.y, vf.y);
            vf.z = fmaf(g[l], b.z, vf.z); vf.w = fmaf(g[l], b.w, vf.w);
          }
        }
      }
      *reinterpret_cast<float4*>(&sK[row * D + cc * 4]) = kf;
      *reinterpret_cast<float4*>(&sV[row * D + cc * 4]) = vf;
    }
    __syncthreads();

    float s[BCF];
    float mx = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < BCF; ++jj) {
      float d0 = 0.f;
#pragma unroll
      for (int i = 0; i < NG; ++i) {
        const float4 k4 = *reinterpret_cast<const float4*>(&sK[jj * D + 4 * (part + 4 * i)]);
        d0 = fmaf(q[i].x, k4.x, d0); d0 = fmaf(q[i].y, k4.y, d0);
        d0 = fmaf(q[i].z, k4.z, d0); d0 = fmaf(q[i].w, k4.w, d0);
      }
      d0 += __shfl_xor(d0, 1, 64);
      d0 += __shfl_xor(d0, 2, 64);
      s[jj] = (j0 + jj <= jmax) ? d0 * tau : -INFINITY;
      mx = fmaxf(mx, s[jj]);
    }
    const float m_new = fmaxf(m, mx);  // finite: slot 0 is visible to every row
    const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
    lsum *= alpha;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      acc[i].x *= alpha; acc[i].y *= alpha; acc[i].z *= alpha; acc[i].w *= alpha;
    }
#pragma unroll
    for (int jj = 0; jj < BCF; ++jj) {
      const float p = (s[jj] == -INFINITY) ? 0.f : expf(s[jj] - m_new);
      lsum += p;
#pragma unroll
      for (int i = 0; i < NG; ++i) {
        const float4 v4 = *reinterpret_cast<const float4*>(&sV[jj * D + 4 * (part + 4 * i)]);
        acc[i].x = fmaf(p, v4.x, acc[i].x); acc[i].y = fmaf(p, v4.y, acc[i].y);
        acc[i].z = fmaf(p, v4.z, acc[i].z); acc[i].w = fmaf(p, v4.w, acc[i].w);
      }
    }
    m = m_new;
  }
  if (tq < Tq) {
    const float inv = 1.f / lsum;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      float4 o = make_float4(acc[i].x * inv, acc[i].y * inv, acc[i].z * inv, acc[i].w * inv);
      *reinterpret_cast<float4*>(O + (bh * (long)Tq + tq) * D + 4 * (part + 4 * i)) = o;
    }
    if (LSE && part == 0) LSE[bh * (long)Tq + tq] = m + logf(lsum);
  }
}

}  // namespace

hipError_t launch_fwd_f32(const FwdArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  const int n_qtiles = (a.Tq + 63) / 64;
  const long nblocks = (long)n_qtiles * a.BH;
#define MKA_FWD32(D)                                                                            \
  hipLaunchKernelGGL((fwd_f32_kernel<D>), dim3((unsigned)nblocks), dim3(256), 0, st,           \
                     (const float*)a.Q, (const float*)a.K[0], (const float*)a.K[1],             \
                     (const float*)a.K[2], (const float*)a.V[0], (const float*)a.V[1],          \
                     (const float*)a.V[2], a.G, (float*)a.O, a.LSE, a.Tq, a.S, a.len[0],        \
                     a.len[1], a.len[2], a.causal, a.scale, n_qtiles)
  if (a.d == 128) MKA_FWD32(128); else MKA_FWD32(64);
#undef MKA_FWD32
  return hipGetLastError();
}

}  // namespace mka
