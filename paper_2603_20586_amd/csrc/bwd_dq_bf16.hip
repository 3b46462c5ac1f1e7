// dQ of the route-fused attention backward, bf16 MFMA path, without atomics.  The paper prints
// no backward; this is the query-side part of the chain rule through Alg. 2 steps 6-9:
//
//   P[t,j]  = exp(tau Q[t].Kf[j] - LSE[t])        dP[t,j] = dO[t].Vf[j]
//   dS[t,j] = P[t,j] (dP[t,j] - D[t])             dQ[t] = tau sum_j dS[t,j] Kf[j] + sum_l dg[t,l] W_r[:,l]
//
// (dg: gradient of the row's router logits, from the main kernel).  A workgroup owns 256
// query rows and walks over the fused K / V stream, which the main backward kernel has written
// to the workspace while it fused its own tiles: dQ of a row is then the sum over ITS OWN
// workgroup's tiles, held in registers and stored once - the alternative, adding one partial
// per (KV tile, row) with f32 atomics from the KV-stationary kernel, is bound by the rate of
// those atomics (about one element per clock and compute unit).  The price is S and dP a second
// time: three MFMA products per pair instead of one.
//
// Skeleton as in the gated-mixture forward: 8 waves x 32 query rows, a lane owns one query row
// (all products are computed transposed: S^T = Kf Q^T, dP^T = Vf dO^T, dQ^T += Kf^T dS^T with
// 32x32x16 MFMAs), 64-slot tiles go from global memory straight into LDS (rings of four K and
// four V tiles, requests two tiles ahead and spread over the sections), one barrier per tile.
// Per unit of 32 slots: section 1 = the two score products (two independent accumulation
// chains), section 2 = P and dS in registers (no running maximum: LSE is known), section 3 = the
// dQ contraction with Kf^T fragments read transposed out of the row-major K tile.  One ring of
// D/16 LDS fragments serves all three operand streams, every slot refilled as soon as its MFMA
// has issued.
#include "attn_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int DQ_BC = 64;   // slots per KV tile
constexpr int DQ_NW = 8;    // waves per workgroup
constexpr int DQ_NT = DQ_NW * 64;
constexpr int DQ_BR = DQ_NW * 32;  // query rows per workgroup

template <int D>
struct DqSmem {
  static constexpr int ROWB = D * 2;         // bytes per tile row (no padding)
  static constexpr int TSZ = DQ_BC * ROWB;   // bytes per tile
  static constexpr int NB = 4;               // ring depth; slot s = K tile at 2 s TSZ, V tile after it
  static constexpr int RING = 2 * NB * TSZ;
  static constexpr int ESTR = D + 4;         // f32 per row of the epilogue's staging tile
  static constexpr int EPI = DQ_BR * ESTR * 4 + D * 3 * 4;  // + the router weights
  static constexpr int TOTAL = RING > EPI ? RING : EPI;  // bytes
};

// One unit of 32 slots (first slot jb, last visible slot jmax) whose K rows start at byte ko of
// the LDS buffer and whose V rows are one tile size further; kn: the same for the next unit.
// fr: ring of D/16 LDS fragments, PF = D/32 slots per operand stream.  On entry slots 0..PF-1
// hold K fragments 0..PF-1 of this unit and slots PF..2PF-1 its V fragments; on exit the same
// for the next unit.  mid1 / mid2 are called in the middle of sections 1 and 3 (the kernel
// issues its tile requests there, one load at a time).
// Register r of the score accumulators <-> slot jb + 8 (r/4) + 4 g + r%4 of the lane's row.
template <int D, bool MASK, typename F1, typename F2>
__device__ __forceinline__ void dq_unit(F1&& mid1, F2&& mid2, bf16x8 (&fr)[D / 16], const char* smem,
                                        unsigned ko, unsigned kn, unsigned a0, unsigned x_lo,
                                        unsigned x_hi, int jb, int jmax,
                                        const bf16x8 (&qreg)[D / 16], const bf16x8 (&doreg)[D / 16],
                                        f32x16 (&acc)[D / 32], float lse2, float dr, float c,
                                        int lane) {
  constexpr int ROWB = D * 2, KK = D / 16, DB = D / 32, PF = KK / 2, TSZ = DqSmem<D>::TSZ;
  const int g = lane >> 5;
  // Lane addresses of this unit.  They are made opaque so that the compiler derives the address
  // of every read from them with one XOR, instead of keeping D/8 loop-invariant variants in
  // registers: the kernel has none to spare.
  unsigned ka = ko + a0, xl = ko + x_lo, xh = ko + x_hi, na = kn + a0;
  asm volatile("" : "+v"(ka), "+v"(xl), "+v"(xh), "+v"(na));
  auto row_frag = [&](unsigned base, int kk, int tensor) __attribute__((always_inline)) {
    return lds_frag(smem + tensor * TSZ + (base ^ (unsigned)(kk << 5)));
  };
  // Kf^T fragment of dQ MFMA i (head dims 32 (i % DB) .., k-step i / DB): the transpose of 8
  // slots x 32 head dims of the row-major K tile
  auto kt_frag = [&](int i) __attribute__((always_inline)) {
    const int db = i % DB, ks = i / DB;
    const uint2 lo = lds_read_tr(reinterpret_cast<const bf16*>(smem + 16 * ks * ROWB + (xl ^ (unsigned)(db << 6))));
    const uint2 hi = lds_read_tr(reinterpret_cast<const bf16*>(smem + 16 * ks * ROWB + (xh ^ (unsigned)(db << 6))));
    return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
  };

  // -- section 1: S^T = Kf Q^T and dP^T = Vf dO^T
  f32x16 s, dp;
#pragma unroll
  for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    s = mfma32(fr[kk % PF], qreg[kk], s);
    dp = mfma32(fr[PF + kk % PF], doreg[kk], dp);
    if (kk + PF < KK) {
      fr[kk % PF] = row_frag(ka, kk + PF, 0);
      fr[PF + kk % PF] = row_frag(ka, kk + PF, 1);
    } else {
      const int i = 2 * (kk + PF - KK);
      fr[kk % PF] = kt_frag(i);
      fr[PF + kk % PF] = kt_frag(i + 1);
    }
    if (kk == KK / 2 - 1) mid1();
    __builtin_amdgcn_sched_barrier(0);
  }

  // -- section 2: P = exp2(c S - LSE log2 e), dS = P (dP - D)
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float p = fast_exp2(fmaf(s[r], c, -lse2));
    if (MASK) {
      const int j = jb + 8 * (r >> 2) + 4 * g + (r & 3);
      p = j > jmax ? 0.f : p;
    }
    s[r] = p * (dp[r] - dr);
  }
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = s[r];
  const bf16x8 b0 = __builtin_bit_cast(bf16x8, pack8(&v[0]));
  const bf16x8 b1 = __builtin_bit_cast(bf16x8, pack8(&v[8]));
  __builtin_amdgcn_sched_barrier(0);

  // -- section 3: dQ^T += Kf^T dS^T; the freed slots take the first fragments of the next unit
#pragma unroll
  for (int i = 0; i < KK; ++i) {
    const int slot = ((i & 1) ? PF : 0) + ((KK - PF + i / 2) % PF);
    acc[i % DB] = mfma32(fr[slot], (i / DB) ? b1 : b0, acc[i % DB]);
    fr[slot] = row_frag(na, i / 2, i & 1);
    if (i == KK / 2 - 1) mid2();
    __builtin_amdgcn_sched_barrier(0);
  }
}

// One tile of BR query rows (index qt) of head bh.  Called by all threads of the workgroup.
template <int D>
__device__ __forceinline__ void bwd_dq_tile(
    const bf16* __restrict__ Q, const bf16* __restrict__ dO, const bf16* __restrict__ Kf,
    const bf16* __restrict__ Vf, const float* __restrict__ LSE2p, const float* __restrict__ Dp,
    const float* __restrict__ dgate, const float* __restrict__ W_r, bf16* __restrict__ dQ,
    float tau, int Tq, int Tqp, int S, int causal, float c, int qt, long bh) {
  using SM = DqSmem<D>;
  constexpr int BR = DQ_BR, BC = DQ_BC, ROWB = SM::ROWB;
  constexpr int KK = D / 16, DB = D / 32, CPR = D / 8, PF = KK / 2;
  extern __shared__ __attribute__((aligned(1024))) unsigned char dq_smem_raw[];
  char* smem = reinterpret_cast<char*>(dq_smem_raw);

  // (opaque: the lane constants derived from it are recomputed per call instead of being kept
  // alive across the two tiles of a workgroup)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63, g = lane >> 5, li = lane & 31;
  const int wave = tid >> 6;
  const int tw0 = qt * BR + wave * 32;  // first row of this wave
  const int tq = tw0 + li;              // this lane's row

  // B operands of the two score products, held for the whole kernel; rows past the end are
  // zeros with LSE = +inf, hence P = 0
  bf16x8 qreg[KK], doreg[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 u = make_uint4(0, 0, 0, 0), w = make_uint4(0, 0, 0, 0);
    if (tq < Tq) {
      u = *reinterpret_cast<const uint4*>(Q + (bh * (long)Tq + tq) * D + 16 * kk + 8 * g);
      w = *reinterpret_cast<const uint4*>(dO + (bh * (long)Tq + tq) * D + 16 * kk + 8 * g);
    }
    qreg[kk] = __builtin_bit_cast(bf16x8, u);
    doreg[kk] = __builtin_bit_cast(bf16x8, w);
  }
  float lse2 = INFINITY, dr = 0.f;
  if (tq < Tq) {
    lse2 = LSE2p[bh * (long)Tqp + tq];
    dr = Dp[bh * (long)Tqp + tq];
  }

  // tiles this workgroup visits, the lane's last visible slot, the wave's first row's
  int t_last = qt * BR + BR - 1;
  if (t_last > Tq - 1) t_last = Tq - 1;
  int j_end = S;
  if (causal && t_last + (S - Tq) + 1 < S) j_end = t_last + (S - Tq) + 1;
  const int NT = (j_end + BC - 1) / BC;  // >= 1: S >= Tq >= 1
  const int jmax = causal ? min(tq + (S - Tq), S - 1) : S - 1;
  const int row_lo = tw0 + (S - Tq);
  const char* kbase = reinterpret_cast<const char*>(Kf + bh * (long)S * D);
  const char* vbase = reinterpret_cast<const char*>(Vf + bh * (long)S * D);

  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  // ---- staging.  One load instruction fills 1 KiB of a tile (RPI rows); a wave issues IPW of
  // them for K and IPW for V per tile.  Lane i of instruction q serves LDS row RPI q + i / CPR,
  // chunk position i % CPR: the slot and the chunk that belong there are fixed per lane.
  constexpr int RPI = 64 / CPR;
  constexpr int IPW = (BC / RPI) / DQ_NW;
  unsigned dslot[IPW], dchunk[IPW];
#pragma unroll
  for (int e = 0; e < IPW; ++e) {
    const int r = RPI * (IPW * wave + e) + lane / CPR;
    dslot[e] = (unsigned)mx_row(r);
    dchunk[e] = 16u * (unsigned)((lane % CPR) ^ mx_swz<D>(r));
  }
  const unsigned lds0 =
      __builtin_amdgcn_readfirstlane((unsigned)(size_t)smem + 1024u * (unsigned)(IPW * wave));
  int rb_w = 0;     // ring position of the next tile to request
  int rq_tile = 0;  // its index (past the end: the last tile again, so that every wave always
                    // has the same number of loads in flight and the counted waits stay exact)
  unsigned rq_off[IPW];
  // rows past the end of the stream repeat its last row: their P is masked to 0
  auto request_begin = [&]() __attribute__((always_inline)) {
    const unsigned j0 = (unsigned)(rq_tile < NT ? rq_tile : NT - 1) * BC;
#pragma unroll
    for (int e = 0; e < IPW; ++e)
      rq_off[e] = min(j0 + dslot[e], (unsigned)(S - 1)) * (unsigned)ROWB + dchunk[e];
    ++rq_tile;
  };
  auto request_part = [&](int q) __attribute__((always_inline)) {
    if (q < IPW) mx_dma16(kbase, rq_off[q], lds0 + (unsigned)(2 * rb_w * SM::TSZ + 1024 * q));
    else mx_dma16(vbase, rq_off[q - IPW], lds0 + (unsigned)((2 * rb_w + 1) * SM::TSZ + 1024 * (q - IPW)));
  };
  auto request_end = [&]() __attribute__((always_inline)) { rb_w = rb_w == SM::NB - 1 ? 0 : rb_w + 1; };
  constexpr int LPT = 2 * IPW;  // loads of a wave per tile

  const unsigned a0 = mx_kfrag0<D>(li, g);
  unsigned x_lo, x_hi;
  mx_trfrag0<D>(lane, x_lo, x_hi);

  // prologue: tiles 0..2 requested, tile 0 landed
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    request_begin();
#pragma unroll
    for (int q = 0; q < LPT; ++q) request_part(q);
    request_end();
  }
  mx_wait_loads<2 * LPT>();
  __syncthreads();

  bf16x8 fr[KK];  // first K and V fragments of unit 0 of tile 0
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    fr[j] = *reinterpret_cast<const bf16x8*>(smem + (a0 ^ (unsigned)(j << 5)));
    fr[PF + j] = *reinterpret_cast<const bf16x8*>(smem + SM::TSZ + (a0 ^ (unsigned)(j << 5)));
  }
  int rb = 0;  // ring position of the tile being consumed
  for (int T = 0; T < NT; ++T) {
    mx_wait_loads<LPT>();  // this wave's part of tile T+1 has landed (T+2 may be in flight)
    loop_barrier();        // tile T+1 complete; the buffers of tile T-1 are free
    request_begin();       // tile T+3, issued in four places of the two units
    const int rb1 = rb == SM::NB - 1 ? 0 : rb + 1;
    const unsigned k0 = (unsigned)(2 * rb * SM::TSZ);   // K rows of unit 0; unit 1 is 32 rows on
    const unsigned k1 = (unsigned)(2 * rb1 * SM::TSZ);  // K rows of unit 0 of tile T+1
    const int j0 = T * BC;
    const bool mask0 = (j0 + 32 > S) || (causal && j0 + 31 > row_lo);
    const bool mask1 = (j0 + 64 > S) || (causal && j0 + 63 > row_lo);
    constexpr int PPS = (2 * IPW + 3) / 4;  // loads of the request per section
    auto part = [&](int sct) __attribute__((always_inline)) {
#pragma unroll
      for (int q = sct * PPS; q < (sct + 1) * PPS && q < 2 * IPW; ++q) request_part(q);
    };
    auto p0 = [&]() __attribute__((always_inline)) { part(0); };
    auto p1 = [&]() __attribute__((always_inline)) { part(1); };
    auto p2 = [&]() __attribute__((always_inline)) { part(2); };
    auto p3 = [&]() __attribute__((always_inline)) { part(3); };
    if (mask0) dq_unit<D, true>(p0, p1, fr, smem, k0, k0 + 32 * ROWB, a0, x_lo, x_hi, j0, jmax, qreg, doreg, acc, lse2, dr, c, lane);
    else dq_unit<D, false>(p0, p1, fr, smem, k0, k0 + 32 * ROWB, a0, x_lo, x_hi, j0, jmax, qreg, doreg, acc, lse2, dr, c, lane);
    if (mask1) dq_unit<D, true>(p2, p3, fr, smem, k0 + 32 * ROWB, k1, a0, x_lo, x_hi, j0 + 32, jmax, qreg, doreg, acc, lse2, dr, c, lane);
    else dq_unit<D, false>(p2, p3, fr, smem, k0 + 32 * ROWB, k1, a0, x_lo, x_hi, j0 + 32, jmax, qreg, doreg, acc, lse2, dr, c, lane);
    request_end();
    rb = rb1;
  }
  mx_wait_loads<0>();  // the surplus requests of the last tiles must land before LDS is reused
  __syncthreads();     // every wave is done with the tile buffers (the epilogue reuses them)

  // ---- epilogue: dQ^T -> rows through LDS; dQ = tau acc + dg W_r^T, rounded once, coalesced
  // stores (the 32 lanes of a half-wave write one row)
  {
    constexpr int ESTR = SM::ESTR;
    float* sE = reinterpret_cast<float*>(smem) + wave * (32 * ESTR);
    float* sW = reinterpret_cast<float*>(smem) + DQ_BR * ESTR;
    const bool route = W_r != nullptr && dgate != nullptr;
    if (route)
      for (int i = tid; i < D * 3; i += DQ_NT) sW[i] = W_r[i];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; r += 4) {
        const int d = 32 * db + 8 * (r >> 2) + 4 * g;
        *reinterpret_cast<float4*>(&sE[li * ESTR + d]) =
            make_float4(acc[db][r], acc[db][r + 1], acc[db][r + 2], acc[db][r + 3]);
      }
    __syncthreads();
    constexpr int FPR = D / 4;  // 4-element groups per row
#pragma unroll
    for (int i = 0; i < 32 * FPR / 64; ++i) {
      const int item = lane + 64 * i;
      const int rr = item / FPR, ch = item % FPR;
      const float4 v4 = *reinterpret_cast<const float4*>(&sE[rr * ESTR + ch * 4]);
      const int t = tw0 + rr;
      if (t < Tq) {
        float o[4] = {v4.x * tau, v4.y * tau, v4.z * tau, v4.w * tau};
        if (route) {
          const float* dgr = dgate + (bh * (long)Tq + t) * 3;
          const float dg0 = dgr[0], dg1 = dgr[1], dg2 = dgr[2];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int k = ch * 4 + e;
            o[e] += dg0 * sW[k * 3 + 0] + dg1 * sW[k * 3 + 1] + dg2 * sW[k * 3 + 2];
          }
        }
        uint2 w;
        w.x = pack_bf16x2(o[0], o[1]);
        w.y = pack_bf16x2(o[2], o[3]);
        *reinterpret_cast<uint2*>(dQ + (bh * (long)Tq + t) * D + ch * 4) = w;
      }
    }
  }
}

template <int D>
__global__ __launch_bounds__(DQ_NT, 1) void bwd_dq_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ dO, const bf16* __restrict__ Kf,
    const bf16* __restrict__ Vf, const float* __restrict__ LSE2p, const float* __restrict__ Dp,
    const float* __restrict__ dgate, const float* __restrict__ W_r, bf16* __restrict__ dQ,
    float tau, int Tq, int Tqp, int S, int causal, float c, int n_qtiles, int BH,
    int interleave, int pair) {
  // all query tiles of one (batch, head) on ONE XCD (block index = 8 * slot + xcd), heaviest
  // tiles first; heads interleaved on small grids (shorter causal tail).
  // pair: a workgroup takes query tile qt and then its mirror tile n_qtiles-1-qt; under a causal
  // mask the two see the same number of K/V tiles in total, so all workgroups weigh the same,
  // and half as many are started.
  const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
  const int n_first = pair ? (n_qtiles + 1) / 2 : n_qtiles;
  int qt0, hl;
  if (interleave) {
    const int hpx = (BH + 7) / 8;
    qt0 = n_qtiles - 1 - slot / hpx;
    hl = slot % hpx;
  } else {
    qt0 = n_qtiles - 1 - slot % n_first;
    hl = slot / n_first;
  }
  const long bh = (long)hl * 8 + xcd;
  if (bh >= BH) return;
  const int qt1 = n_qtiles - 1 - qt0;
  bwd_dq_tile<D>(Q, dO, Kf, Vf, LSE2p, Dp, dgate, W_r, dQ, tau, Tq, Tqp, S, causal, c, qt0, bh);
  if (pair && qt1 != qt0) {
    __syncthreads();  // the first tile's output staging is dead
    bwd_dq_tile<D>(Q, dO, Kf, Vf, LSE2p, Dp, dgate, W_r, dQ, tau, Tq, Tqp, S, causal, c, qt1, bh);
  }
}

template <int D>
hipError_t launch_dq_t(const BwdDqArgs& a, hipStream_t st) {
  const int n_qtiles = (a.Tq + DQ_BR - 1) / DQ_BR;
  // under a causal mask a workgroup takes a heavy and a light query tile (see the kernel)
  const int pair = (a.causal && n_qtiles > 1) ? 1 : 0;
  const int n_first = pair ? (n_qtiles + 1) / 2 : n_qtiles;
  const long nblocks = (long)n_first * ((a.BH + 7) / 8) * 8;
  const int interleave = (!pair && nblocks <= 2 * 256) ? 1 : 0;
  const size_t smem = (size_t)DqSmem<D>::TOTAL;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dq_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((bwd_dq_kernel<D>), dim3((unsigned)nblocks), dim3(DQ_NT), smem, st,
                     (const bf16*)a.Q, (const bf16*)a.dO, (const bf16*)a.Kf, (const bf16*)a.Vf,
                     a.LSE2p, a.Dp, a.dgate, a.W_r, (bf16*)a.dQ, a.scale, a.Tq, a.Tqp, a.S, a.causal, a.scale * kLog2e, n_qtiles, a.BH,
                     interleave, pair);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_dq_bf16(const BwdDqArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  return a.d == 128 ? launch_dq_t<128>(a, st) : launch_dq_t<64>(a, st);
}

}  // namespace mka
