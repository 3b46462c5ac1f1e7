// Pre-fusion of the three K/V memories into ONE bf16 K/V stream (paper: Alg. 2 steps 6-7,
// Kf[j] = sum_l G[j,l] K_l[j], Vf likewise; "route-fusion creates a single fused KV tensor"):
// the materialised alternative to folding the fusion into the attention kernel's tile loads.
// The fused stream is what the paper caches; attention over it is plain softmax attention
// (mka_mixture_attn_fwd with one memory and no gates), decode over it reads a third of the bytes.
//
// One thread = one 16-byte chunk of one slot: six 16-byte loads, the slot's three gates, f32
// mix, one rounding to bf16, two 16-byte stores.  Bound by HBM: 6 reads + 2 writes of S*d*2
// bytes per (batch, head).
#include "fuse_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

template <int D>
__global__ __launch_bounds__(256) void prefuse_kernel(
    const bf16* __restrict__ K0, const bf16* __restrict__ K1, const bf16* __restrict__ K2,
    const bf16* __restrict__ V0, const bf16* __restrict__ V1, const bf16* __restrict__ V2,
    const float* __restrict__ G, bf16* __restrict__ Kf, bf16* __restrict__ Vf, long rows, int S,
    int len0, int len1, int len2) {
  constexpr int CPR = D / 8;
  const long item = (long)blockIdx.x * 256 + threadIdx.x;
  const long row = item / CPR;  // (b,h,slot) flattened
  const int cc = (int)(item % CPR);
  if (row >= rows) return;
  const int j = (int)(row % S);
  const long base = row - j;  // first row of the (b,h) block: always exists
  const bool p0 = j < len0, p1 = j < len1, p2 = j < len2;
  const long eoff = row * D + cc * 8, boff = base * D + cc * 8;
  const Raw3 rk = load_raw3<false, long>(K0, K1, K2, boff, eoff, p0, p1, p2);
  const Raw3 rv = load_raw3<false, long>(V0, V1, V2, boff, eoff, p0, p1, p2);
  const float g0 = G[row * 3 + 0], g1 = G[row * 3 + 1], g2 = G[row * 3 + 2];
  float kf[8], vf[8];
  fuse8(rk, g0, g1, g2, kf);
  fuse8(rv, g0, g1, g2, vf);
  *reinterpret_cast<uint4*>(Kf + eoff) = pack8(kf);
  *reinterpret_cast<uint4*>(Vf + eoff) = pack8(vf);
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
  const int cpr = a.d / 8;
  const unsigned grid = (unsigned)((rows * cpr + 255) / 256);
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
