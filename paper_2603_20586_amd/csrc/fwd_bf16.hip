// Route-fused attention forward, bf16 MFMA path (paper: Alg. 2 steps 6-7 and 9; attention as
// Eq. (1) with the scale of Eq. (3); online softmax by the max-shift recursion of the section
// "Numerical Stability via Max-Shift", applied over KV tiles with one running max per row).
//
// One workgroup = NW waves x 32 query rows.  Per KV tile of 64 slots:
//   1. the workgroup reads the three raw K tiles, the three raw V tiles and the slots' gates
//      with coalesced 16-byte loads, mixes them in f32 (Kf = sum_l G_l K_l), rounds once to
//      bf16 and writes Kf row-major and Vf TRANSPOSED into LDS — the fused K/V stream exists
//      only there;
//   2. each wave computes S^T = Kf Q^T (slots x rows) with 32x32x16 MFMAs: A = Kf from LDS,
//      B = Q^T held in registers for the whole kernel.  In the S^T accumulator layout a lane
//      owns ONE query row (column l%32) and 16 slots per 32-slot block, so the row max and row
//      sum are in-lane reductions plus a single exchange with lane^32;
//   3. P^T = exp2(c S^T - c m) is rounded to bf16 in registers and is already the B operand
//      of O^T += Vf^T P^T (A = Vf^T from LDS); every O^T accumulator of a lane belongs to the
//      lane's row, so the rescale by exp2(c (m_old - m_new)) is a per-lane scalar.
// The rows of the Kf tile are fed to the MFMA in an order that swaps bits 2 and 3 of the row
// index; this makes the 8 P values a lane packs for one PV k-step belong to 8 consecutive
// slots, i.e. one 16-byte LDS read of Vf^T.
#include "fuse_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int BC = 64;  // slots per KV tile

__device__ __forceinline__ int swap23(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}


// Fuse one KV tile of BC slots into LDS: Kf row-major (row stride KSTR), Vf transposed (row
// stride VSTR).  K work item = (row, 16-byte chunk); V work item = (4 consecutive slots, chunk),
// so that a thread can emit 8-byte transposed writes.  All global loads of a thread are issued
// before the first use.
template <int D, int NT, bool FULL>
__device__ __forceinline__ void fuse_tile(const bf16* __restrict__ K0, const bf16* __restrict__ K1,
                                          const bf16* __restrict__ K2, const bf16* __restrict__ V0,
                                          const bf16* __restrict__ V1, const bf16* __restrict__ V2,
                                          const float* __restrict__ Gb, long kvbase, int j0, int S,
                                          int len0, int len1, int len2, bf16* sK, bf16* sVT) {
  constexpr int KSTR = D + 8, VSTR = BC + 8, CPR = D / 8;
  constexpr int KITEMS = BC * CPR, VITEMS = (BC / 4) * CPR;
  constexpr int KPT = (KITEMS + NT - 1) / NT, VPT = (VITEMS + NT - 1) / NT;
  const int tid = threadIdx.x;
  Raw3 kr[KPT];
  float kg[KPT][3];
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const int it = tid + i * NT;
    const int row = (it / CPR) % BC, cc = it % CPR;  // % BC keeps a surplus thread in range
    const int j = j0 + row;
    const int jc = FULL ? j : (j < S ? j : S - 1);
    const bool in = FULL || j < S;
    kr[i] = load_raw3<FULL>(K0, K1, K2, kvbase + cc * 8, kvbase + (long)jc * D + cc * 8,
                            in && j < len0, in && j < len1, in && j < len2);
    kg[i][0] = Gb[jc * 3 + 0]; kg[i][1] = Gb[jc * 3 + 1]; kg[i][2] = Gb[jc * 3 + 2];
  }
  Raw3 vr[VPT][4];
  float vg[VPT][4][3];
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int it = tid + i * NT;
    const int sg = (it / CPR) % (BC / 4), cc = it % CPR;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + sg * 4 + u;
      const int jc = FULL ? j : (j < S ? j : S - 1);
      const bool in = FULL || j < S;
      vr[i][u] = load_raw3<FULL>(V0, V1, V2, kvbase + cc * 8, kvbase + (long)jc * D + cc * 8,
                                 in && j < len0, in && j < len1, in && j < len2);
      vg[i][u][0] = Gb[jc * 3 + 0]; vg[i][u][1] = Gb[jc * 3 + 1]; vg[i][u][2] = Gb[jc * 3 + 2];
    }
  }
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const int it = tid + i * NT;
    if (KITEMS % NT == 0 || it < KITEMS) {
      const int row = it / CPR, cc = it % CPR;
      float acc[8];
      fuse8(kr[i], kg[i][0], kg[i][1], kg[i][2], acc);
      *reinterpret_cast<uint4*>(&sK[row * KSTR + cc * 8]) = pack8(acc);
    }
  }
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int it = tid + i * NT;
    if (VITEMS % NT == 0 || it < VITEMS) {
      const int sg = it / CPR, cc = it % CPR;
      float vf[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) fuse8(vr[i][u], vg[i][u][0], vg[i][u][1], vg[i][u][2], vf[u]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint2 w;
        w.x = pack_bf16x2(vf[0][e], vf[1][e]);
        w.y = pack_bf16x2(vf[2][e], vf[3][e]);
        *reinterpret_cast<uint2*>(&sVT[(cc * 8 + e) * VSTR + sg * 4]) = w;
      }
    }
  }
}

template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 8 / NW) void fwd_bf16_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S, int len0, int len1, int len2, int causal, float c,
    float tau, int n_qtiles) {
  constexpr int NT = NW * 64;
  constexpr int BR = NW * 32;
  constexpr int KSTR = D + 8;       // bf16 elements per Kf row in LDS (16-byte pad)
  constexpr int VSTR = BC + 8;      // bf16 elements per Vf^T row in LDS
  constexpr int KK = D / 16;        // MFMA k-steps over d
  constexpr int DB = D / 32;        // 32-row blocks of O^T
  __shared__ __attribute__((aligned(16))) bf16 sK[BC * KSTR];
  __shared__ __attribute__((aligned(16))) bf16 sVT[D * VSTR];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
  // heavy (late) query tiles first so that the causal tail is short
  const int qt = n_qtiles - 1 - (int)(blockIdx.x % n_qtiles);
  const long bh = blockIdx.x / n_qtiles;
  const int off = S - Tq;
  const int tw0 = qt * BR + wave * 32;  // first row of this wave
  const int tq = tw0 + li;              // this lane's row

  const bf16* Qb = Q + bh * (long)Tq * D;
  const long kvbase = bh * (long)S * D;
  const float* Gb = G + bh * (long)S * 3;

  bf16x8 qreg[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 u = make_uint4(0, 0, 0, 0);
    if (tq < Tq) u = *reinterpret_cast<const uint4*>(Qb + (long)tq * D + 16 * kk + 8 * g);
    qreg[kk] = __builtin_bit_cast(bf16x8, u);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  int t_last = qt * BR + BR - 1;
  if (t_last > Tq - 1) t_last = Tq - 1;
  int j_end = S;
  if (causal && t_last + off + 1 < S) j_end = t_last + off + 1;
  const int ntiles = (j_end + BC - 1) / BC;

  for (int jt = 0; jt < ntiles; ++jt) {
    const int j0 = jt * BC;
    __syncthreads();  // all waves are done reading the previous tile
    // ---- fuse K and V of this tile into LDS (interior tiles take the predicate-free path)
    const bool full = (j0 + BC <= len0) && (j0 + BC <= len1) && (j0 + BC <= len2);
    if (full)
      fuse_tile<D, NT, true>(K0, K1, K2, V0, V1, V2, Gb, kvbase, j0, S, len0, len1, len2, sK, sVT);
    else
      fuse_tile<D, NT, false>(K0, K1, K2, V0, V1, V2, Gb, kvbase, j0, S, len0, len1, len2, sK, sVT);
    __syncthreads();

    // ---- S^T = Kf Q^T   (two blocks of 32 slots)
    f32x16 sacc[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[sb][r] = 0.f;
      const bf16* arow = &sK[(32 * sb + swap23(li)) * KSTR + 8 * g];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + 16 * kk);
        sacc[sb] = mfma32(a, qreg[kk], sacc[sb]);
      }
    }
    // register r of block sb holds slot j0 + 32 sb + 16 (r/8) + 8 g + r%8 of row tq
    const bool need_mask = (j0 + BC > S) || (causal && (j0 + BC - 1 > tw0 + off));
    if (need_mask) {
      const int jmax = causal ? (tq + off < S - 1 ? tq + off : S - 1) : S - 1;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + 32 * sb + 16 * (r >> 3) + 8 * g + (r & 7);
          if (j > jmax) sacc[sb][r] = -INFINITY;
        }
    }
    // ---- online softmax (one row per lane; the row's other half lives in lane^32)
    float mx = sacc[0][0];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[sb][r]);
    mx = fmaxf(mx, xor32(mx));
    const float m_new = fmaxf(m, mx);
    // m_new is finite from the first tile on: every row sees slot 0
    const float alpha = (m == -INFINITY) ? 0.f : fast_exp2((m - m_new) * c);
    const float mc = m_new * c;
    float psum = 0.f;
    bf16x8 preg[4];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        // a masked score is -inf: exp2(-inf) = 0 when c > 0; c == 0 is handled by the select
        const float e = fast_exp2(fmaf(sacc[sb][r], c, -mc));
        p[r] = (sacc[sb][r] == -INFINITY) ? 0.f : e;
        psum += p[r];
      }
      preg[2 * sb + 0] = __builtin_bit_cast(bf16x8, pack8(&p[0]));
      preg[2 * sb + 1] = __builtin_bit_cast(bf16x8, pack8(&p[8]));
    }
    lsum = lsum * alpha + psum;
    m = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    // ---- O^T += Vf^T P^T
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const bf16* arow = &sVT[(32 * db + li) * VSTR + 8 * g];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + 16 * ks);
        oacc[db] = mfma32(a, preg[ks], oacc[db]);
      }
    }
  }

  // ---- epilogue: normalise and store this lane's row
  lsum += xor32(lsum);
  if (tq < Tq) {
    const float inv = 1.f / lsum;
    bf16* orow = O + (bh * (long)Tq + tq) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        uint2 w;
        w.x = pack_bf16x2(oacc[db][4 * q4 + 0] * inv, oacc[db][4 * q4 + 1] * inv);
        w.y = pack_bf16x2(oacc[db][4 * q4 + 2] * inv, oacc[db][4 * q4 + 3] * inv);
        *reinterpret_cast<uint2*>(orow + 32 * db + 8 * q4 + 4 * g) = w;
      }
    if (LSE && g == 0) LSE[bh * (long)Tq + tq] = m * tau + __logf(lsum);
  }
}

}  // namespace

hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  constexpr int NW = 8;
  const int n_qtiles = (a.Tq + NW * 32 - 1) / (NW * 32);
  const long nblocks = (long)n_qtiles * a.BH;
  const float c = a.scale * kLog2e;
  // a level without memory is given another level's (same-shaped) buffer and length 0: the
  // kernel then never uses what it reads from it
  const void* Kp[3];
  const void* Vp[3];
  const void* anyK = a.K[0] ? a.K[0] : (a.K[1] ? a.K[1] : a.K[2]);
  const void* anyV = a.V[0] ? a.V[0] : (a.V[1] ? a.V[1] : a.V[2]);
  if (!anyK || !anyV) return hipErrorInvalidValue;
  for (int l = 0; l < 3; ++l) {
    Kp[l] = a.K[l] ? a.K[l] : anyK;
    Vp[l] = a.V[l] ? a.V[l] : anyV;
  }
#define MKA_FWD(D)                                                                              \
  hipLaunchKernelGGL((fwd_bf16_kernel<D, NW>), dim3((unsigned)nblocks), dim3(NW * 64), 0, st,  \
                     (const bf16*)a.Q, (const bf16*)Kp[0], (const bf16*)Kp[1],                  \
                     (const bf16*)Kp[2], (const bf16*)Vp[0], (const bf16*)Vp[1],               \
                     (const bf16*)Vp[2], a.G, (bf16*)a.O, a.LSE, a.Tq, a.S, a.len[0], a.len[1], \
                     a.len[2], a.causal, c, a.scale, n_qtiles)
  if (a.d == 128) MKA_FWD(128); else MKA_FWD(64);
#undef MKA_FWD
  return hipGetLastError();
}

}  // namespace mka
