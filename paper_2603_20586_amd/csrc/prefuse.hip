// Pre-fusion of the three K/V memories into ONE bf16 K/V stream (paper: Alg. 2 steps 6-7,
// Kf[j] = sum_l G[j,l] K_l[j], Vf likewise; "route-fusion creates a single fused KV tensor"):
// the materialised alternative to folding the fusion into the attention kernel's tile loads.
// The fused stream is what the paper caches; attention over it is plain softmax attention
// (mka_mixture_attn_fwd with one memory and no gates), decode over it reads a third of the bytes.
//
// One thread = one 16-byte chunk of two slots: the slots' gates, then up to twelve 16-byte
// streaming loads issued at once, f32 mix, one rounding to bf16, four 16-byte stores.  Bound by HBM: 6 reads + 2 writes of S*d*2
// bytes per (batch, head).
#include "fuse_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int PF_U = 2;  // slots per thread

template <int D>
__global__ __launch_bounds__(256) void prefuse_kernel(
    const bf16* __restrict__ K0, const bf16* __restrict__ K1, const bf16* __restrict__ K2,
    const bf16* __restrict__ V0, const bf16* __restrict__ V1, const bf16* __restrict__ V2,
    const float* __restrict__ G, bf16* __restrict__ Kf, bf16* __restrict__ Vf, long rows, int S,
    int len0, int len1, int len2) {
  constexpr int CPR = D / 8, RPW = 256 / CPR;  // rows per workgroup and pass
  const int cc = threadIdx.x % CPR;
  const long row0 = (long)blockIdx.x * (RPW * PF_U) + threadIdx.x / CPR;
  const bf16* Kp[3] = {K0, K1, K2};
  const bf16* Vp[3] = {V0, V1, V2};
  const int len[3] = {len0, len1, len2};
  // the gates of the thread's slots first, then all raw chunks that count (read once: streaming
  // loads); an absent entry is zeros
  uint4 rk[PF_U][3], rv[PF_U][3];
  float g[PF_U][3];
  // a level whose gate is exactly zero (hard routing, section "Routing Mechanism Ablation")
  // cannot contribute and is not loaded: top-1 gates halve the traffic (2 reads + 2 writes per
  // element instead of 6 + 2); with soft gates the dependent gate load costs nothing measurable
#pragma unroll
  for (int u = 0; u < PF_U; ++u) {
    const long row = row0 + (long)u * RPW;
    const long rc = row < rows ? row : rows - 1;
#pragma unroll
    for (int l = 0; l < 3; ++l) g[u][l] = G[rc * 3 + l];
  }
#pragma unroll
  for (int u = 0; u < PF_U; ++u) {
    const long row = row0 + (long)u * RPW;
    const long rc = row < rows ? row : rows - 1;
    const int j = (int)(rc % S);
#pragma unroll
    for (int l = 0; l < 3; ++l) {
      rk[u][l] = make_uint4(0, 0, 0, 0);
      rv[u][l] = make_uint4(0, 0, 0, 0);
      if (j < len[l] && g[u][l] != 0.f) {
        const long o = rc * D + cc * 8;
        rk[u][l] = load16_stream(Kp[l] + o);
        rv[u][l] = load16_stream(Vp[l] + o);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < PF_U; ++u) {
    const long row = row0 + (long)u * RPW;
    if (row >= rows) continue;
    const int j = (int)(row % S);
    const uint4 z = make_uint4(0, 0, 0, 0);
    Raw3 k3, v3;
    k3.a = j < len0 ? rk[u][0] : z;  v3.a = j < len0 ? rv[u][0] : z;
    k3.b = j < len1 ? rk[u][1] : z;  v3.b = j < len1 ? rv[u][1] : z;
    k3.c = j < len2 ? rk[u][2] : z;  v3.c = j < len2 ? rv[u][2] : z;
    float kf[8], vf[8];
    fuse8(k3, g[u][0], g[u][1], g[u][2], kf);
    fuse8(v3, g[u][0], g[u][1], g[u][2], vf);
    const long eoff = row * D + cc * 8;
    *reinterpret_cast<uint4*>(Kf + eoff) = pack8(kf);
    *reinterpret_cast<uint4*>(Vf + eoff) = pack8(vf);
  }
}

}  // namespace

hipError_t launch_prefuse(const PrefuseArgs& a, hipStream_t st) {
  const long rows = (long)a.BH * a.S;
  if (rows == 0) return hipSuccess;
  // a level without memory borrows another level's buffer and has length 0 (never used)
  const void* anyK = a.K[0] ? a.K[0] : (a.K[1] ? a.K[1] : a.K[2]);
  const void* anyV = a.V[0] ? a.V[0] : (a.V[1] ? a.V[1] : a.V[2]);
  if (!anyK || !anyV) return hipErrorInvalidValue;
  const void* Kp[3];
  const void* Vp[3];
  int len[3];
  for (int l = 0; l < 3; ++l) {
    const bool has = a.K[l] && a.V[l];
    Kp[l] = has ? a.K[l] : anyK;
    Vp[l] = has ? a.V[l] : anyV;
    len[l] = has ? a.len[l] : 0;
  }
  const int rows_per_wg = 256 / (a.d / 8) * PF_U;
  const unsigned grid = (unsigned)((rows + rows_per_wg - 1) / rows_per_wg);
#define MKA_PREFUSE(D)                                                                          \
  hipLaunchKernelGGL((prefuse_kernel<D>), dim3(grid), dim3(256), 0, st, (const bf16*)Kp[0],     \
                     (const bf16*)Kp[1], (const bf16*)Kp[2], (const bf16*)Vp[0],                \
                     (const bf16*)Vp[1], (const bf16*)Vp[2], a.G, (bf16*)a.Kf, (bf16*)a.Vf,     \
                     rows, a.S, len[0], len[1], len[2])
  if (a.d == 128) MKA_PREFUSE(128); else MKA_PREFUSE(64);
#undef MKA_PREFUSE
  return hipGetLastError();
}

}  // namespace mka
