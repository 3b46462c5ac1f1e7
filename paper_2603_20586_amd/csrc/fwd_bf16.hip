// Route-fused attention forward, bf16 MFMA path (paper: Alg. 2 steps 6-7 and 9; attention as
// Eq. (1) with the scale of Eq. (3); online softmax by the max-shift recursion of the section
// "Numerical Stability via Max-Shift", applied over KV blocks with one running max per row).
//
// One workgroup = 8 waves x 32 query rows = 256 rows; KV tiles of 64 slots; one barrier per tile.
//   * fusion (Kf = sum_l G_l K_l, Vf likewise) happens in registers between the global load and
//     the LDS write: raw 16-byte chunks of the three levels are loaded half a tile ahead, mixed
//     in f32, rounded once to bf16; the fused stream exists only in LDS.  Waves 0-3 stage the K
//     half of every tile, waves 4-7 the V half, in half slices issued behind every MFMA of the
//     wave's own work (the kernel is bound by VALU issue: fusion, exponentials and conversions
//     cost more issue cycles than the MFMAs they feed, so none of them may wait for another).
//   * the work of a wave is software-pipelined over units of 32 slots: the S^T MFMAs of the next
//     unit are issued between the exponentials of the current one; the barrier that publishes
//     tile t+1 sits between the two units of tile t (two Kf buffers, three Vf^T buffers).
//   * S^T = Kf Q^T (slots x rows) with 32x32x16 MFMAs: A = Kf rows from LDS, B = Q^T held in
//     registers for the whole kernel.  In the accumulator layout a lane owns ONE query row
//     (column l%32) and 16 of the 32 slots, so row max and row sum are in-lane reductions plus a
//     single exchange with lane^32.
//   * P^T = exp2(c S^T - c m), rounded to bf16 in registers, already is the B operand of
//     O^T += Vf^T P^T (A = Vf^T rows from LDS); all O^T accumulators of a lane belong to its row,
//     so the rescale by exp2(c (m_old - m_new)) is a per-lane scalar.
// Vf is written to LDS transposed ([d][slot]) with the slot order permuted (bits 2 and 3 of the
// slot index swapped) so that the 8 P values a lane packs for one PV k-step pair with ONE
// 16-byte read, and with its ROWS permuted: head-dim index d = 8 cc + e lives in LDS row
// e * (D/8) + cc.  A 16-lane read group then touches 16 consecutive rows (conflict-free with
// the 144-byte row stride) and a 16-lane write group (8 chunks x 2 halves) covers every bank
// once.  The O^T accumulator rows follow the same permutation; the epilogue undoes it while
// transposing O through LDS for coalesced 16-byte stores.
#include "fuse_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

constexpr int FW_BC = 64;   // slots per KV tile
constexpr int FW_NW = 8;    // waves per workgroup
constexpr int FW_NG = 256;  // threads per fusion group (waves 0-3: K, waves 4-7: V)

__device__ __forceinline__ int fw_swap23(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

template <int D>
struct FwdSmem {
  static constexpr int KSTR = D + 8;       // bf16 per Kf row (16-byte pad)
  static constexpr int VSTR = FW_BC + 8;   // bf16 per Vf^T row
  static constexpr int KSZ = FW_BC * KSTR;
  static constexpr int VSZ = D * VSTR;
  static constexpr int VOFF = 2 * KSZ;     // two Kf buffers, then three Vf^T buffers
  static constexpr int TOTAL = 2 * KSZ + 3 * VSZ;  // bf16 elements
};

// ---- staging: raw (unfused) data -> registers -> fused bf16 tile in LDS ----------------------
// Waves 0-3 stage the K half of every tile, waves 4-7 the V half.  A thread's share of a half
// tile is 4 work items ("quarters"), each one 16-byte chunk of the three levels plus the gates of
// its slot.  Quarters are staged in PAIRS, one pair per half step of the MFMA loop: the pair's
// raw data is loaded during one half step and fused during the next, cut into 8 slices that are
// issued one by one behind the PV MFMAs, so that the VALU work runs in the shadow of the wave's
// own matrix instructions and the global loads reach the memory pipeline a few at a time.
struct PairRaw {
  Raw3 r[2];
  float g[2][3];
};
struct StageTmp {
  float acc[2][8];  // running fused values of the two quarters of the pair (f32)
  unsigned w[8];    // V: packed slots 0,1 of the item, kept until slots 2,3 are done
};

// V work item = (4 consecutive slots, one 16-byte chunk).  Thread bits: [2:0] chunk low bits,
// [3] slot-group bit 1 (selects the 8-byte half of a 16-byte column block), [4] slot-group bit 0,
// [6:5] slot-group bits 3:2, [7] chunk bit 3.  A 16-lane LDS write group is then 8 chunks x 2
// halves, which (with the row permutation of the Vf^T tile) covers every bank exactly once.
template <int D>
__device__ __forceinline__ void v_item(int tg, int& sg, int& cc, bool& active) {
  constexpr int CPR = D / 8;
  sg = (((tg >> 3) & 1) << 1) | ((tg >> 4) & 1) | (((tg >> 5) & 3) << 2);
  cc = (tg & 7) | ((tg >> 7) << 3);
  active = CPR == 16 || cc < CPR;  // tg < 256, so cc < 16 always
  if (!active) cc = 0;
}

// K work item i = (slot tg / CPR + RPP i, chunk tg % CPR); d = 64 has only two of them per thread
// (quarters 0 and 2).  tg = thread index inside the fusion group (0..255).
template <int D>
__device__ __forceinline__ bool k_quarter(int q, int& i) {
  constexpr int N = FW_BC * (D / 8) / FW_NG;  // 4 for d = 128, 2 for d = 64
  i = N == 4 ? q : q >> 1;
  return N == 4 || (q & 1) == 0;
}

// raw loads of quarter q of the tile that starts at slot j0 (P0..P2: this group's K or V)
template <int D, bool GV, bool FULL>
__device__ __forceinline__ void stage_load(int q, PairRaw& x, const bf16* __restrict__ P0,
                                           const bf16* __restrict__ P1, const bf16* __restrict__ P2,
                                           const float* __restrict__ Gb, int j0, int S, int len0,
                                           int len1, int len2, int tg) {
  constexpr int CPR = D / 8, RPP = FW_NG / CPR;
  int i, j, cc;
  if (!GV) {
    if (!k_quarter<D>(q, i)) return;
    cc = tg % CPR;
    j = j0 + tg / CPR + RPP * i;
  } else {
    int sg;
    bool active;
    v_item<D>(tg, sg, cc, active);
    j = j0 + sg * 4 + q;
  }
  const int jc = FULL ? j : (j < S ? j : S - 1);
  const bool in = FULL || j < S;
  x.r[q & 1] = load_raw3_b<FULL>(P0, P1, P2, (unsigned)(cc * 16), (unsigned)(jc * D + cc * 8) * 2u,
                                 in && j < len0, in && j < len1, in && j < len2);
  const char* gp = reinterpret_cast<const char*>(Gb) + (unsigned)(jc * 12);
  x.g[q & 1][0] = *reinterpret_cast<const float*>(gp);
  x.g[q & 1][1] = *reinterpret_cast<const float*>(gp + 4);
  x.g[q & 1][2] = *reinterpret_cast<const float*>(gp + 8);
}

// one level (0..2) of the raw data of quarter q of the tile that starts at slot j0; level 2 also
// brings the gates of the slot
template <int D, bool GV, bool FULL>
__device__ __forceinline__ void stage_load_level(int q, int level, PairRaw& x,
                                                 const bf16* __restrict__ P0,
                                                 const bf16* __restrict__ P1,
                                                 const bf16* __restrict__ P2,
                                                 const float* __restrict__ Gb, int j0, int S,
                                                 int len0, int len1, int len2, int tg) {
  constexpr int CPR = D / 8, RPP = FW_NG / CPR;
  int i, j, cc;
  if (!GV) {
    if (!k_quarter<D>(q, i)) return;
    cc = tg % CPR;
    j = j0 + tg / CPR + RPP * i;
  } else {
    int sg;
    bool active;
    v_item<D>(tg, sg, cc, active);
    j = j0 + sg * 4 + q;
  }
  const int jc = FULL ? j : (j < S ? j : S - 1);
  const bool in = FULL || j < S;
  const bf16* P = level == 0 ? P0 : (level == 1 ? P1 : P2);
  const int len = level == 0 ? len0 : (level == 1 ? len1 : len2);
  const bool present = FULL || (in && j < len);
  const unsigned off_b = present ? (unsigned)(jc * D + cc * 8) * 2u : (unsigned)(cc * 16);
  uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(P) + off_b);
  if (!present) v = make_uint4(0, 0, 0, 0);
  if (level == 0) x.r[q & 1].a = v;
  else if (level == 1) x.r[q & 1].b = v;
  else {
    x.r[q & 1].c = v;
    const char* gp = reinterpret_cast<const char*>(Gb) + (unsigned)(jc * 12);
    x.g[q & 1][0] = *reinterpret_cast<const float*>(gp);
    x.g[q & 1][1] = *reinterpret_cast<const float*>(gp + 4);
    x.g[q & 1][2] = *reinterpret_cast<const float*>(gp + 8);
  }
}

// half slice (part 0..3, h = 0/1) of the fusion of quarter q: parts 0..2 add one level each (f32,
// four elements per half), part 3 rounds to bf16 and writes to LDS (dst: Kf tile or Vf^T tile of
// the staged tile)
template <int D, bool GV>
__device__ __forceinline__ void stage_slice(int q, int part, int h, const PairRaw& x, StageTmp& t,
                                            bf16* dst, int tg) {
  constexpr int CPR = D / 8, RPP = FW_NG / CPR, KSTR = D + 8, VSTR = FW_BC + 8;
  int i = q, sg = 0, cc = 0;
  if (!GV) {
    if (!k_quarter<D>(q, i)) return;
  } else {
    bool active;
    v_item<D>(tg, sg, cc, active);
    if (!active) return;
  }
  float* acc = t.acc[q & 1];
  if (part < 3) {
    const uint4& u = part == 0 ? x.r[q & 1].a : (part == 1 ? x.r[q & 1].b : x.r[q & 1].c);
    // gate of the level; with all gates of the slot loaded together, g[.][part]
    const float gl = x.g[q & 1][part];
    const unsigned w0 = h ? u.z : u.x, w1 = h ? u.w : u.y;
    const float f[4] = {bf16lo(w0), bf16hi(w0), bf16lo(w1), bf16hi(w1)};
#pragma unroll
    for (int e = 0; e < 4; ++e)
      acc[4 * h + e] = part == 0 ? gl * f[e] : fmaf(gl, f[e], acc[4 * h + e]);
    // pin the arithmetic to this slice (else it all sinks to where the tile is written)
#pragma unroll
    for (int e = 0; e < 4; ++e) asm volatile("" : "+v"(acc[4 * h + e]));
    return;
  }
  if (!GV) {
    if (h == 1)
      *reinterpret_cast<uint4*>(&dst[(tg / CPR + RPP * i) * KSTR + (tg % CPR) * 8]) = pack8(acc);
  } else if (q == 1) {
#pragma unroll
    for (int e = 4 * h; e < 4 * h + 4; ++e) {
      t.w[e] = pack_bf16x2(t.acc[0][e], t.acc[1][e]);
      asm volatile("" : "+v"(t.w[e]));
    }
  } else if (q == 3) {
    // slots 4 sg .. 4 sg + 3 go to columns col .. col + 3 (bits 2,3 of the slot index swapped)
    const int col = 32 * (sg >> 3) + fw_swap23(4 * (sg & 7));
    const int blk = col >> 3, half = (col >> 2) & 1;
#pragma unroll
    for (int e = 4 * h; e < 4 * h + 4; ++e) {
      const int prow = e * (D / 8) + cc;  // LDS row of head-dim index d = 8 cc + e
      uint2 w;
      w.x = t.w[e];
      w.y = pack_bf16x2(t.acc[0][e], t.acc[1][e]);
      *reinterpret_cast<uint2*>(&dst[prow * VSTR + 8 * blk + 4 * half]) = w;
    }
  }
}

// ---- one half step of a wave: 32 slots (one "unit") of its 32 query rows -----------------------
// Software pipeline: the S^T MFMAs of the NEXT unit are issued between the exponentials of the
// current one, and the staging slices between the PV MFMAs, in exactly the order written here
// (scheduling barriers keep the compiler from regrouping them); LDS fragments are read four
// instructions ahead of their MFMA.
//   s_now : finished S^T of the unit to consume (register r <-> slot jb + 8 (r/4) + 4 g + r%4)
//   s_next: S^T of unit `unit_n` of the Kf tile at sKn, left in flight for the next half step
//   FAST  : interior half step - no masking, staging unconditional and with all levels present
template <int D, bool GV, bool FAST>
__device__ __forceinline__ void half_step(
    f32x16 s_now, f32x16& s_next, const bf16* sKn, int unit_n, int jb, const bf16* sVT, int unit,
    const bf16x8 (&qreg)[D / 16], f32x16 (&oacc)[D / 32], float& m, float& mc, float& lsum, float c,
    int jmax,
    PairRaw& raw, StageTmp& tmp, bf16* dst, int qf, bool do_fuse, int jl, int ql, bool do_load,
    bool full, const bf16* __restrict__ P0, const bf16* __restrict__ P1,
    const bf16* __restrict__ P2, const float* __restrict__ Gb, int S, int len0, int len1, int len2,
    int li, int g, int tg) {
  constexpr int KSTR = D + 8, VSTR = FW_BC + 8, KK = D / 16, DB = D / 32;
  constexpr int PF = 4;          // LDS fragments in flight
  constexpr int EPK = 16 / KK;   // exponentials per S MFMA
  constexpr int NPV = 2 * DB;    // PV MFMAs of the unit
  constexpr int SPM = 16 / (KK + NPV);  // staging half slices per MFMA (1 for d = 128, 2 for 64)
  // half slice hs = 0..15 of the pair: quarter qf + hs / 8, part (hs % 8) / 2, half hs % 2; once
  // both halves of a level are consumed, its registers are reloaded with the same level of
  // quarter ql + hs / 8 of the tile at jl (fused one half step from now)
  auto stage = [&](int hs) __attribute__((always_inline)) {
    const int qo = hs >> 3, part = (hs & 7) >> 1, h = hs & 1;
    if (FAST || do_fuse) stage_slice<D, GV>(qf + qo, part, h, raw, tmp, dst, tg);
    if (h == 1 && part < 3) {
      if (FAST) {
        stage_load_level<D, GV, true>(ql + qo, part, raw, P0, P1, P2, Gb, jl, S, len0, len1, len2, tg);
      } else if (do_load) {
        if (full) stage_load_level<D, GV, true>(ql + qo, part, raw, P0, P1, P2, Gb, jl, S, len0, len1, len2, tg);
        else stage_load_level<D, GV, false>(ql + qo, part, raw, P0, P1, P2, Gb, jl, S, len0, len1, len2, tg);
      }
    }
  };
  bf16x8 fr[PF];
  const bf16* arow = &sKn[(32 * unit_n + li) * KSTR + 8 * g];
#pragma unroll
  for (int kk = 0; kk < PF; ++kk) fr[kk] = *reinterpret_cast<const bf16x8*>(arow + 16 * kk);

  if (!FAST) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = jb + 8 * (r >> 2) + 4 * g + (r & 3);
      if (j > jmax) s_now[r] = -INFINITY;
    }
  }
  // Lazy max-shift: the reference m only moves when the row max has grown by more than 2^8
  // in the exponent; until then P = exp2(c (s - m)) may exceed 1 (at most 256), which bf16 and
  // the f32 sums hold without loss, and the rescale of the accumulators is skipped.  The
  // recursion is unchanged (O and z are always relative to the same m), only m is stale.
  // The common case costs the in-lane maximum and one compare: each half of a row (the lanes li
  // and li + 32) tests its own 16 slots against the row's reference (mc = m c; -inf before the
  // first visible slot, which fails the test); only when some lane of the wave fails it are the
  // halves exchanged, the references moved and the accumulators rescaled.  A unit with masked
  // slots always takes the long way.
  // Every row sees slot 0, so m is finite after the first unit that has a visible slot.
  const float lmax = max16(s_now);
  if (__any(!FAST || !(fmaf(lmax, c, -mc) <= 8.f))) {
    const float mx = fmaxf(lmax, xor32(lmax));
    const bool move = (mx - m) * c > 8.f || m == -INFINITY;
    const float m_new = move ? mx : m;
    const float alpha = move ? ((m == -INFINITY) ? 0.f : fast_exp2((m - m_new) * c)) : 1.f;
    m = m_new;
    mc = m_new * c;
    lsum *= alpha;
    if (__any(move)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
  }

  // -- section A: S^T of the next unit, between the exponentials of this one
  f32x16 sn;
#pragma unroll
  for (int r = 0; r < 16; ++r) sn[r] = 0.f;
  float p[16];
  const bf16* vbase = &sVT[li * VSTR + 8 * (4 * unit + g)];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    sn = mfma32(fr[kk % PF], qreg[kk], sn);
    if (kk + PF < KK) {
      fr[kk % PF] = lds_frag(arow + 16 * (kk + PF));
    } else {  // the K fragments are all on their way: start on the Vf^T fragments
      const int i = kk + PF - KK;  // PV MFMA i uses rows 32 (i % DB), k half i / DB
      if (i < NPV)
        fr[kk % PF] = lds_frag(vbase + 32 * (i % DB) * VSTR + 16 * (i / DB));
    }
#pragma unroll
    for (int r = kk * EPK; r < (kk + 1) * EPK; ++r) {
      float e = fast_exp2(fmaf(s_now[r], c, -mc));
      if (!FAST) e = (s_now[r] == -INFINITY) ? 0.f : e;  // also covers c == 0
      p[r] = e;
    }
#pragma unroll
    for (int hs = kk * SPM; hs < (kk + 1) * SPM; ++hs) stage(hs);
    __builtin_amdgcn_sched_barrier(0);
  }
  s_next = sn;
  const uint4 pk0 = pack8(&p[0]), pk1 = pack8(&p[8]);
  const bf16x8 p0 = __builtin_bit_cast(bf16x8, pk0);
  const bf16x8 p1 = __builtin_bit_cast(bf16x8, pk1);
  // Row sum of P in f32, before the rounding to bf16.  Plain adds on purpose: v_dot2_f32_bf16
  // cannot issue while an MFMA of either wave of the SIMD is in the matrix pipe.
  const float psum = (((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]))) +
                     (((p[8] + p[9]) + (p[10] + p[11])) + ((p[12] + p[13]) + (p[14] + p[15])));
  lsum += psum;
  __builtin_amdgcn_sched_barrier(0);

  // -- section B: O^T += Vf^T P^T (k half 0 = columns 16 ks .. of the unit with P^T regs 0-7),
  // one staging slice (d = 128) or two (d = 64) behind every MFMA
#pragma unroll
  for (int i = 0; i < NPV; ++i) {
    constexpr int KP = KK % PF;  // ring position of PV fragment 0
    oacc[i % DB] = mfma32(fr[(KP + i) % PF], i / DB ? p1 : p0, oacc[i % DB]);
    if (i + PF < NPV) {
      const int n = i + PF;
      fr[(KP + i) % PF] = lds_frag(vbase + 32 * (n % DB) * VSTR + 16 * (n / DB));
    }
#pragma unroll
    for (int hs = (KK + i) * SPM; hs < (KK + i + 1) * SPM; ++hs) stage(hs);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ---- the tile loop of one wave; GV = the wave stages V halves (else K halves) ------------------
// The barrier that publishes tile jt+1 sits in the MIDDLE of tile jt's work: its second unit
// still reads the old Vf^T buffer (hence three of them) while the first S^T of tile jt+1 is
// already being issued.  Staging order: pair B (quarters 2,3) of tile jt+1 is fused in the first
// half step of tile jt, pair A (quarters 0,1) of tile jt+2 in the second.
template <int D, bool GV>
__device__ __forceinline__ void run_tiles(bf16* smem, const bf16* __restrict__ P0,
                                          const bf16* __restrict__ P1, const bf16* __restrict__ P2,
                                          const float* __restrict__ Gb, const bf16x8 (&qreg)[D / 16],
                                          f32x16 (&oacc)[D / 32], float& m, float& mc, float& lsum, float c,
                                          int ntiles, int S, int len0, int len1, int len2,
                                          int causal, int row_lo, int jmax, int li, int g, int tg) {
  using L = FwdSmem<D>;
  constexpr int BC = FW_BC;
  const int lenmin = min(len0, min(len1, len2));
  PairRaw raw = {};  // fully defined on every path, so that it lives in registers
  StageTmp tmp = {};
  // this group's half of tile T lives in K buffer T & 1 or V^T buffer T % 3
  auto dst_of = [&](int kb, int vb) { return smem + (GV ? L::VOFF + vb * L::VSZ : kb * L::KSZ); };
  auto stage_pair_now = [&](int T, int q0, int kb, int vb) __attribute__((always_inline)) {
#pragma unroll
    for (int q = q0; q < q0 + 2; ++q)
      stage_load<D, GV, false>(q, raw, P0, P1, P2, Gb, T * BC, S, len0, len1, len2, tg);
#pragma unroll
    for (int hs = 0; hs < 16; ++hs)
      stage_slice<D, GV>(q0 + (hs >> 3), (hs & 7) >> 1, hs & 1, raw, tmp, dst_of(kb, vb), tg);
  };

  // prologue: tile 0 complete, pair A of tile 1 fused, pair B of tile 1 loaded
  stage_pair_now(0, 0, 0, 0);
  stage_pair_now(0, 2, 0, 0);
  if (ntiles > 1) {
    stage_pair_now(1, 0, 1, 1);
#pragma unroll
    for (int q = 2; q < 4; ++q)
      stage_load<D, GV, false>(q, raw, P0, P1, P2, Gb, BC, S, len0, len1, len2, tg);
  }
  __syncthreads();

  f32x16 s_a, s_b;
  {
    constexpr int KSTR = D + 8;
#pragma unroll
    for (int r = 0; r < 16; ++r) s_a[r] = 0.f;
    const bf16* arow = &smem[li * KSTR + 8 * g];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
      s_a = mfma32(*reinterpret_cast<const bf16x8*>(arow + 16 * kk), qreg[kk], s_a);
  }
  int vb = 0;  // V^T buffer of tile jt
  for (int jt = 0; jt < ntiles; ++jt) {
    const bool has1 = jt + 1 < ntiles, has2 = jt + 2 < ntiles;
    const int j0 = jt * BC;
    const int vb1 = vb == 2 ? 0 : vb + 1, vb2 = vb1 == 2 ? 0 : vb1 + 1;
    const bf16* sK = smem + (jt & 1) * L::KSZ;
    const bf16* sK1 = smem + ((jt + 1) & 1) * L::KSZ;
    const bf16* sVT = smem + L::VOFF + vb * L::VSZ;
    bf16* dst1 = dst_of((jt + 1) & 1, vb1);  // tile jt+1, pair B
    bf16* dst2 = dst_of(jt & 1, vb2);        // tile jt+2, pair A
    // row_lo = first row of the wave + (S - Tq): the wave's rows see slots <= row_lo .. row_lo + 31
    const bool need_mask = (j0 + BC > S) || (causal && (j0 + BC - 1 > row_lo));
    const bool full2 = j0 + 3 * BC <= lenmin;
    const int jl = j0 + 2 * BC;  // both half steps load raw data of tile jt+2
    if (!need_mask && has2 && full2) {
      half_step<D, GV, true>(s_a, s_b, sK, 1, j0, sVT, 0, qreg, oacc, m, mc, lsum, c, jmax, raw, tmp,
                             dst1, 2, true, jl, 0, true, true, P0, P1, P2, Gb, S, len0, len1, len2,
                             li, g, tg);
      loop_barrier();  // tile jt+1 is complete in LDS; K buffer jt&1 may be overwritten
      half_step<D, GV, true>(s_b, s_a, sK1, 0, j0 + 32, sVT, 1, qreg, oacc, m, mc, lsum, c, jmax, raw,
                             tmp, dst2, 0, true, jl, 2, true, true, P0, P1, P2, Gb, S, len0, len1,
                             len2, li, g, tg);
    } else {
      half_step<D, GV, false>(s_a, s_b, sK, 1, j0, sVT, 0, qreg, oacc, m, mc, lsum, c, jmax, raw, tmp,
                              dst1, 2, has1, jl, 0, has2, full2, P0, P1, P2, Gb, S, len0, len1,
                              len2, li, g, tg);
      __syncthreads();
      half_step<D, GV, false>(s_b, s_a, sK1, 0, j0 + 32, sVT, 1, qreg, oacc, m, mc, lsum, c, jmax, raw,
                              tmp, dst2, 0, has2, jl, 2, has2, full2, P0, P1, P2, Gb, S, len0, len1,
                              len2, li, g, tg);
    }
    vb = vb1;
  }
  __syncthreads();  // every wave is done with the tile buffers (the epilogue reuses them)
}

// One tile of BR query rows (index qt) of head bh.  Called by all threads of the workgroup.
template <int D>
__device__ __forceinline__ void fwd_tile(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S, int len0, int len1, int len2, int causal, float c,
    float tau, int qt, long bh) {
  constexpr int BR = FW_NW * 32, BC = FW_BC;
  constexpr int KK = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char fw_smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(fw_smem_raw);

  // (opaque: the lane constants derived from it are recomputed per call instead of being kept
  // alive across the two tiles of a workgroup)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
  const bool grpV = wave >= 4;  // waves 4-7 fuse the V half, waves 0-3 the K half
  const int tg = tid & (FW_NG - 1);
  const int off = S - Tq;
  const int tw0 = qt * BR + wave * 32;  // first row of this wave
  const int tq = tw0 + li;              // this lane's row

  const bf16* Qb = Q + bh * (long)Tq * D;
  const long kvbase = bh * (long)S * D;
  // per-(b,h) bases are wave-uniform; everything below them is a 32-bit offset
  const bf16* K0b = K0 + kvbase;
  const bf16* K1b = K1 + kvbase;
  const bf16* K2b = K2 + kvbase;
  const bf16* V0b = V0 + kvbase;
  const bf16* V1b = V1 + kvbase;
  const bf16* V2b = V2 + kvbase;
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
  float m = -INFINITY, mc = -INFINITY, lsum = 0.f;  // mc = m c, kept beside m

  int t_last = qt * BR + BR - 1;
  if (t_last > Tq - 1) t_last = Tq - 1;
  int j_end = S;
  if (causal && t_last + off + 1 < S) j_end = t_last + off + 1;
  const int ntiles = (j_end + BC - 1) / BC;
  const int jmax = causal ? (tq + off < S - 1 ? tq + off : S - 1) : S - 1;

  // waves 0-3 stage the K half of every tile, waves 4-7 the V half; the two loops have the same
  // trip count and one barrier per trip
  if (!grpV)
    run_tiles<D, false>(smem, K0b, K1b, K2b, Gb, qreg, oacc, m, mc, lsum, c, ntiles, S, len0, len1, len2,
                        causal, tw0 + off, jmax, li, g, tg);
  else
    run_tiles<D, true>(smem, V0b, V1b, V2b, Gb, qreg, oacc, m, mc, lsum, c, ntiles, S, len0, len1, len2,
                       causal, tw0 + off, jmax, li, g, tg);

  // ---- epilogue: normalise, transpose O^T through LDS (tile buffers are free after the last
  // barrier), store rows with coalesced 16-byte writes
  lsum += xor32(lsum);
  {
    constexpr int OSTR = D + 8, CPR = D / 8;
    bf16* sO = smem + wave * (32 * OSTR);
    const float inv = 1.f / lsum;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int prow = 32 * db + 8 * (r >> 2) + 4 * g + (r & 3);  // accumulator row
        const int d = 8 * (prow % CPR) + prow / CPR;               // head-dim index it holds
        sO[li * OSTR + d] = (bf16)(oacc[db][r] * inv);
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32 * CPR / 64; ++i) {
      const int item = lane + 64 * i;
      const int row = item / CPR, ch = item % CPR;
      const uint4 v = *reinterpret_cast<const uint4*>(&sO[row * OSTR + ch * 8]);
      if (tw0 + row < Tq)
        *reinterpret_cast<uint4*>(O + (bh * (long)Tq + tw0 + row) * D + ch * 8) = v;
    }
    if (LSE && g == 0 && tq < Tq) LSE[bh * (long)Tq + tq] = m * tau + __logf(lsum);
  }
}

template <int D>
__global__ __launch_bounds__(FW_NW * 64, 1) void fwd_bf16_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S, int len0, int len1, int len2, int causal, float c,
    float tau, int n_qtiles, int BH, int interleave, int pair) {
  // Workgroups are handed to the 8 XCDs round-robin by block index.  All query tiles of one
  // (batch, head) are given to ONE XCD (block index = 8 * slot + xcd), so that the workgroups
  // that stream the same K/V tiles share that XCD's L2; heavy (late) query tiles go first so
  // that the causal tail is short.
  // pair: a workgroup takes query tile qt and then its mirror tile n_qtiles-1-qt; under a causal
  // mask the two see the same number of K/V tiles in total, so all workgroups weigh the same,
  // and half as many are started.
  const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
  const int n_first = pair ? (n_qtiles + 1) / 2 : n_qtiles;
  int qt0, hl;
  if (interleave) {  // small grids: heaviest tiles of ALL the XCD's heads first (shorter tail)
    const int hpx = (BH + 7) / 8;
    qt0 = n_qtiles - 1 - slot / hpx;
    hl = slot % hpx;
  } else {           // large grids: one head after the other (best L2 reuse of its K/V tiles)
    qt0 = n_qtiles - 1 - slot % n_first;
    hl = slot / n_first;
  }
  const long bh = (long)hl * 8 + xcd;
  if (bh >= BH) return;  // the head count need not be a multiple of 8
  const int qt1 = n_qtiles - 1 - qt0;
  fwd_tile<D>(Q, K0, K1, K2, V0, V1, V2, G, O, LSE, Tq, S, len0, len1, len2, causal, c, tau, qt0,
              bh);
  if (pair && qt1 != qt0) {
    __syncthreads();  // the first tile's output staging is dead
    fwd_tile<D>(Q, K0, K1, K2, V0, V1, V2, G, O, LSE, Tq, S, len0, len1, len2, causal, c, tau, qt1,
                bh);
  }
}

template <int D>
static hipError_t launch_fwd_t(const FwdArgs& a, const void* const Kp[3], const void* const Vp[3],
                               hipStream_t st) {
  constexpr int BR = FW_NW * 32;
  const int n_qtiles = (a.Tq + BR - 1) / BR;
  // under a causal mask a workgroup takes a heavy and a light query tile (see the kernel)
  const int pair = (a.causal && n_qtiles > 1) ? 1 : 0;
  const int n_first = pair ? (n_qtiles + 1) / 2 : n_qtiles;
  const long nblocks = (long)n_first * ((a.BH + 7) / 8) * 8;
  // unpaired and at most 2 workgroups per compute unit (256 CUs): the tail dominates, interleave
  // heads (beyond that the heads' K/V streams evict each other from the L2 and HBM reads triple)
  const int interleave = (!pair && nblocks <= 2 * 256) ? 1 : 0;
  const size_t smem = (size_t)FwdSmem<D>::TOTAL * sizeof(bf16);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_bf16_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_bf16_kernel<D>), dim3((unsigned)nblocks), dim3(FW_NW * 64), smem, st,
                     (const bf16*)a.Q, (const bf16*)Kp[0], (const bf16*)Kp[1], (const bf16*)Kp[2],
                     (const bf16*)Vp[0], (const bf16*)Vp[1], (const bf16*)Vp[2], a.G, (bf16*)a.O,
                     a.LSE, a.Tq, a.S, a.len[0], a.len[1], a.len[2], a.causal,
                     a.scale * kLog2e, a.scale, n_qtiles, a.BH, interleave, pair);
  return hipGetLastError();
}

hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
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
  return a.d == 128 ? launch_fwd_t<128>(a, Kp, Vp, st) : launch_fwd_t<64>(a, Kp, Vp, st);
}

}  // namespace mka
