// Gated mixture of exponentiated scores over up to three K/V memories, bf16 MFMA path (paper:
// section "Theoretical Formulation: Recursive MKA with Online Softmax", first equation, evaluated
// with the max-shift recursion of "Numerical Stability via Max-Shift"):
//
//   O[t] = sum_l lam[t,l] sum_j exp(tau Q[t].K_l[j]) V_l[j] / sum_l lam[t,l] sum_j exp(tau Q[t].K_l[j])
//
// The gate belongs to the QUERY row, so it is a per-row, per-level bias log2 lam[t,l] on the
// scores: the three memories are streamed one after the other as ONE sequence of 64-slot tiles
// through the same online softmax (no tile fusion, no slot alignment; every level has its own
// length and its own bottom-right aligned causal mask).  Without gates (lam == 1) and with one
// memory this is plain softmax attention - the kernel a pre-fused K/V stream would use.
//
// Skeleton as in the route-fused forward: workgroup = 8 waves x 32 query rows, S^T = K Q^T and
// O^T += V^T P^T with 32x32x16 MFMAs (a lane owns one query row), units of 32 slots software-
// pipelined (the S^T MFMAs of the next unit between the exponentials of the current one), one
// barrier per tile.  Differences: the tiles are plain row copies, so they go from
// global memory straight into LDS (global_load_lds_dwordx4: no registers hold data in flight, and
// the prefetch distance is the depth of the buffer rings - three K and four V tiles, a tile is
// requested two tiles before its first use); V stays row-major and its transpose for the second
// product is read with ds_read_b64_tr_b16.  The tile layout that makes this work without padding
// is described where it is defined (slot permutation + chunk swizzle, applied on the global side).
#include "attn_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int MX_BC = 64;   // slots per KV tile
constexpr int MX_BR = 256;  // query rows per workgroup
#ifndef MX_R
#define MX_R 1
#endif
// R: blocks of 32 query rows per wave.  A K or V^T fragment read from LDS feeds R MFMAs, so R = 2
// halves the LDS traffic per flop; the workgroup then has 4 waves (one per SIMD, 512 registers
// each) instead of 8.
template <int R>
struct MixShape {
  static constexpr int NW = MX_BR / (32 * R);  // waves per workgroup
  static constexpr int NT = NW * 64;           // threads
};

template <int D>
struct MixSmem {
  static constexpr int ROWB = D * 2;          // bytes per tile row (no padding)
  static constexpr int TSZ = MX_BC * ROWB;    // bytes per tile
  static constexpr int NKB = 3, NVB = 4;      // ring depths
  static constexpr int VOFF = NKB * TSZ;
  static constexpr int TOTAL = (NKB + NVB) * TSZ;  // bytes (also covers the epilogue's O tiles)
};

struct MixLevels {
  const bf16* K[3];
  const bf16* V[3];
  int S[3];         // slots of the level (0: absent)
  int n[3];         // tiles of the level that this workgroup visits
  int row_lo[3];    // last slot the wave's FIRST row sees
};

// element l of a 3-array without dynamic indexing (which would put the array in scratch memory)
template <typename T>
__device__ __forceinline__ T sel3(int l, const T (&a)[3]) {
  return l == 0 ? a[0] : (l == 1 ? a[1] : a[2]);
}

// first level after l that has tiles (3: none)
__device__ __forceinline__ int mx_next_level(const MixLevels& L, int l) {
  int nl = 3;
  if (l < 2 && L.n[2] > 0) nl = 2;
  if (l < 1 && L.n[1] > 0) nl = 1;
  if (l < 0 && L.n[0] > 0) nl = 0;
  return nl;
}

template <int D>
__device__ __forceinline__ f32x16 mx_s_unit(const char* sK, unsigned a0, const bf16x8 (&qreg)[D / 16]) {
  constexpr int KK = D / 16;
  f32x16 sacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    sacc = mfma32(*reinterpret_cast<const bf16x8*>(sK + (a0 ^ (unsigned)(kk << 5))), qreg[kk], sacc);
  return sacc;
}

// Per row block state of the online softmax and what a half step needs to know about the rows.
struct MixRow {
  float m, lsum;  // running reference exponent (log2 units, gate included) and denominator
  float bl;       // log2 gate of the level being consumed
  float kb;       // bl - m (bl while nothing has been seen): what the exponentials add to c * score
  int jmax;       // last visible slot of that level
};

// Step k (0..7) of the running maximum over the 16 registers of an accumulator: eight steps
// cover it (three-operand maxima; no NaN canonicalisation of the inputs: they come out of an
// MFMA or are -inf).
template <int K>
__device__ __forceinline__ void mx_max_step(float& m, const f32x16& s) {
  // (volatile: the statements keep their place between the MFMAs)
  if (K == 0) asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(s[0]), "v"(s[1]), "v"(s[2]));
  else if (K < 7) asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(m), "v"(s[2 * K + 1]), "v"(s[(2 * K + 2) & 15]));
  else asm volatile("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(m), "v"(s[15]));
}

// One half step of a wave: finish the unit whose S^T is s_now (32 slots from jb of a level:
// softmax, then O^T += V^T P^T with the V rows of unit U of the tile at sV) and compute the S^T
// of the following unit into s_next - for each of the wave's R row blocks, which share every
// LDS fragment.
//
// Every MFMA of the half step is followed by a few vector instructions of another stage of the
// pipeline, so that neither pipe sees a long stretch of the other kind: the S^T MFMAs of the
// next unit run between the exponentials (and the rounding to bf16) of this one, the PV MFMAs of
// this unit between the row sums of its P and the running maximum of the next unit's scores.
//
// Reference exponent.  Lazy max-shift (as in the route-fused forward): the reference only moves
// when an exponent has grown more than 8 beyond it, so P may reach 2^8 and the rescale of the
// accumulators is skipped on almost every unit.  The common case costs the in-lane maximum and
// one compare, both done a half step early (behind the PV MFMAs): each half of a row (the lanes
// li and li + 32) tests its own 16 slots against the row's reference, and `need` says whether
// some lane of the wave failed.  Only then are the halves exchanged, the references moved and
// the accumulators rescaled - at the start of the half step that consumes the unit, when the
// accumulators are at rest.  A masked unit always takes the long way; so does the first unit of
// a level (the caller sets need: the test was made with the previous level's gate).
//
// fr is a ring of D/16 LDS fragments that lives across half steps.  On entry it holds the K
// fragments of the unit whose S^T is computed here; every S MFMA group frees a slot, which is
// refilled with the V^T fragment of the PV MFMAs that will use the same slot; these free it again
// and it is refilled with a K fragment of the unit after the next (at sKnn, unit offset
// included).  Every LDS read is thus issued a whole section before its use.
// a0: mx_kfrag0 of the lane; x_lo / x_hi: byte offsets of the lane's transposed V reads.
// mid_a / mid_b are called in the middle of the two sections (the kernel issues its tile requests
// there, one load instruction at a time, so that the waves' loads do not queue up behind each
// other at the address unit).
// Register r of s_now[.] <-> slot jb + 8 (r/4) + 4 g + r%4 of the lane's row.
template <int D, int R, bool MASK, int U, typename FA, typename FB>
__device__ __forceinline__ void mx_half_step(FA&& mid_a, FB&& mid_b, f32x16 (&s_now)[R], f32x16 (&s_next)[R],
                                             bf16x8 (&fr)[D / 16], const char* sKnn, unsigned a0,
                                             int jb, const char* sV, unsigned x_lo, unsigned x_hi,
                                             const bf16x8 (&qreg)[R][D / 16],
                                             f32x16 (&oacc)[R][D / 32], MixRow (&row)[R], float c,
                                             int lane, bool& need) {
  constexpr int ROWB = D * 2, KK = D / 16, DB = D / 32;
  constexpr int EPK = 16 / KK;   // exponentials per S MFMA
  constexpr int NPV = 2 * DB;    // PV MFMAs of the unit and row block (== KK)
  constexpr int MPS = 8 / NPV;   // steps of the running maximum per PV MFMA
  const int g = lane >> 5;

  if (MASK) {
#pragma unroll
    for (int rb = 0; rb < R; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = jb + 8 * (r >> 2) + 4 * g + (r & 3);
        if (j > row[rb].jmax) s_now[rb][r] = -INFINITY;
      }
  }
  if (MASK || need) {
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
      float mx = max16(s_now[rb]);
      mx = fmaxf(mx, xor32(mx));
      const float m = row[rb].m, bl = row[rb].bl;
      const float cand = (mx == -INFINITY) ? -INFINITY : fmaf(mx, c, bl);
      const bool move = cand - m > 8.f || (m == -INFINITY && cand > -INFINITY);
      const float m_new = move ? cand : m;
      const float alpha = move ? ((m == -INFINITY) ? 0.f : fast_exp2(m - m_new)) : 1.f;
      row[rb].kb = bl - ((m_new == -INFINITY) ? 0.f : m_new);
      row[rb].m = m_new;
      row[rb].lsum *= alpha;
      if (__any(move)) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[rb][db][r] *= alpha;
      }
    }
  }
  float kb[R];
#pragma unroll
  for (int rb = 0; rb < R; ++rb) kb[rb] = row[rb].kb;

  // V^T fragment of PV MFMA i (rows 32 (i % DB) of V^T, k-step i / DB): the transpose of 8 slots
  // x 32 head dims of the row-major V tile.  k positions 0..3 <-> slots 16 ks + 4 g + 0..3,
  // positions 4..7 <-> 8 further: the slots whose P values the lane holds in registers 8 ks ..
  // The head-dim block db only meets the swizzle in an XOR of address bits 6..7.
  auto v_frag = [&](int i) __attribute__((always_inline)) {
    const int db = i % DB, ks = i / DB;
    const char* vrow = sV + (32 * U + 16 * ks) * ROWB;
    const uint2 lo = lds_read_tr(reinterpret_cast<const bf16*>(vrow + (x_lo ^ (unsigned)(db << 6))));
    const uint2 hi = lds_read_tr(reinterpret_cast<const bf16*>(vrow + (x_hi ^ (unsigned)(db << 6))));
#if MKA_DOUBLE & 1
    const uint2 lo2 = lds_read_tr(reinterpret_cast<const bf16*>(vrow + 512 + (x_lo ^ (unsigned)(db << 6))));
    const uint2 hi2 = lds_read_tr(reinterpret_cast<const bf16*>(vrow + 512 + (x_hi ^ (unsigned)(db << 6))));
    asm volatile("" ::"v"(lo2), "v"(hi2));
#endif
    return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
  };

  // -- section A: S^T of the next unit, between the exponentials of this one
  f32x16 sn[R];
#pragma unroll
  for (int rb = 0; rb < R; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) sn[rb][r] = 0.f;
  float p[R][16];
  uint32_t pw[R][8];  // P rounded to bf16, two slots per word
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
    for (int rb = 0; rb < R; ++rb) sn[rb] = mfma32(fr[kk], qreg[rb][kk], sn[rb]);
    fr[kk] = v_frag(kk);
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
#pragma unroll
      for (int r = kk * EPK; r < (kk + 1) * EPK; ++r) {
        float e = fast_exp2(fmaf(s_now[rb][r], c, kb[rb]));
        if (MASK) e = (s_now[rb][r] == -INFINITY) ? 0.f : e;  // also covers c == 0
#if MKA_DOUBLE & 4
        {
          const float again = fast_exp2(fmaf(s_now[rb][r], c, kb[rb] + 1.f));
          asm volatile("" ::"v"(again));
        }
#endif
#if MKA_DOUBLE & 8
        {
          float more = fmaf(s_now[rb][r], c, kb[rb] + 1.f);
          asm volatile("" ::"v"(more));
          more = fmaf(s_now[rb][r], c, kb[rb] + 2.f);
          asm volatile("" ::"v"(more));
        }
#endif
        p[rb][r] = e;
      }
#pragma unroll
      for (int r = kk * EPK; r < (kk + 1) * EPK; r += 2) pw[rb][r / 2] = pack_bf16x2(p[rb][r], p[rb][r + 1]);
    }
    if (kk == KK / 2 - 1) mid_a();
    __builtin_amdgcn_sched_barrier(0);
  }
  bf16x8 pk[R][2];
#pragma unroll
  for (int rb = 0; rb < R; ++rb) {
    s_next[rb] = sn[rb];
    pk[rb][0] = __builtin_bit_cast(bf16x8, make_uint4(pw[rb][0], pw[rb][1], pw[rb][2], pw[rb][3]));
    pk[rb][1] = __builtin_bit_cast(bf16x8, make_uint4(pw[rb][4], pw[rb][5], pw[rb][6], pw[rb][7]));
  }

  // -- section B: O^T += V^T P^T; behind the MFMAs the row sums of P (in f32, before the rounding
  // to bf16: the rounding errors of the numerator have zero mean; plain adds on purpose:
  // v_dot2_f32_bf16 would halve the instruction count but cannot issue while an MFMA of either
  // wave of the SIMD is in the matrix pipe - measured: a wave with dot2 instructions makes no
  // progress next to a wave that streams MFMAs) and the in-lane maximum of the next unit's scores
  float lsum[R], nmax[R];
#pragma unroll
  for (int rb = 0; rb < R; ++rb) lsum[rb] = row[rb].lsum;
#pragma unroll
  for (int i = 0; i < NPV; ++i) {
#pragma unroll
    for (int rb = 0; rb < R; ++rb)
      oacc[rb][i % DB] = mfma32(fr[i], pk[rb][i / DB], oacc[rb][i % DB]);
    fr[i] = lds_frag(sKnn + (a0 ^ (unsigned)(i << 5)));
#if MKA_DOUBLE & 1
    {
      const bf16x8 again = lds_frag(sKnn + 512 + (a0 ^ (unsigned)(i << 5)));
      asm volatile("" ::"v"(again));
    }
#endif
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
#pragma unroll
      for (int r = i * (16 / NPV); r < (i + 1) * (16 / NPV); ++r)
        asm volatile("v_add_f32 %0, %0, %1" : "+v"(lsum[rb]) : "v"(p[rb][r]));  // in place, see above
      // (none behind the first PV MFMA: the last S^T MFMA has only just been issued, and the
      // running maximum is inline assembly, whose distance to the MFMA that writes its operands
      // is the kernel's to keep)
      if (MPS == 1) {
        if (i == 1) { mx_max_step<0>(nmax[rb], s_next[rb]); mx_max_step<1>(nmax[rb], s_next[rb]); }
        if (i == 2) mx_max_step<2>(nmax[rb], s_next[rb]);
        if (i == 3) mx_max_step<3>(nmax[rb], s_next[rb]);
        if (i == 4) mx_max_step<4>(nmax[rb], s_next[rb]);
        if (i == 5) mx_max_step<5>(nmax[rb], s_next[rb]);
        if (i == 6) mx_max_step<6>(nmax[rb], s_next[rb]);
        if (i == 7) mx_max_step<7>(nmax[rb], s_next[rb]);
      } else {
        if (i == 1) { mx_max_step<0>(nmax[rb], s_next[rb]); mx_max_step<1>(nmax[rb], s_next[rb]); mx_max_step<2>(nmax[rb], s_next[rb]); }
        if (i == 2) { mx_max_step<3>(nmax[rb], s_next[rb]); mx_max_step<4>(nmax[rb], s_next[rb]); mx_max_step<5>(nmax[rb], s_next[rb]); }
        if (i == 3) { mx_max_step<6>(nmax[rb], s_next[rb]); mx_max_step<7>(nmax[rb], s_next[rb]); }
      }
    }
    if (i == NPV / 2 - 1) mid_b();
    __builtin_amdgcn_sched_barrier(0);
  }
  bool chk = false;
#pragma unroll
  for (int rb = 0; rb < R; ++rb) {
    row[rb].lsum = lsum[rb];
    // !(.. <= 8): also taken when there is no reference yet (kb = +inf, or NaN with a zero gate)
    chk = chk || !(fmaf(nmax[rb], c, row[rb].kb) <= 8.f);
  }
  need = __any(chk);
}

// One tile of BR query rows (index qt) of head bh against the whole stream of K/V tiles.  Called
// by all threads of the workgroup.
template <int D, int R>
__device__ __forceinline__ void mix_tile(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S0, int S1, int S2, int causal, float c, int qt,
    long bh) {
  using SM = MixSmem<D>;
  constexpr int NW = MixShape<R>::NW;
  constexpr int BR = MX_BR, BC = MX_BC, ROWB = SM::ROWB;
  constexpr int KK = D / 16, DB = D / 32, CPR = D / 8;
  extern __shared__ __attribute__((aligned(1024))) unsigned char mx_smem_raw[];
  char* smem = reinterpret_cast<char*>(mx_smem_raw);

  // (opaque: the lane constants derived from it are recomputed per call instead of being kept
  // alive across the two tiles of a workgroup)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63, g = lane >> 5, li = lane & 31;
  const int wave = tid >> 6;  // left divergent on purpose: uniform mask branches cost registers
  const int tw0 = qt * BR + wave * (32 * R);  // first row of this wave
  // row block rb of the wave: rows tw0 + 32 rb ..; this lane's row there is tw0 + 32 rb + li

  bf16x8 qreg[R][KK];
#pragma unroll
  for (int rb = 0; rb < R; ++rb)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int tq = tw0 + 32 * rb + li;
      uint4 u = make_uint4(0, 0, 0, 0);
      if (tq < Tq) u = *reinterpret_cast<const uint4*>(Q + (bh * (long)Tq + tq) * D + 16 * kk + 8 * g);
      qreg[rb][kk] = __builtin_bit_cast(bf16x8, u);
    }

  MixLevels L;
  // per row block and level: last slot the lane's row sees (may be negative), log2 of its gate
  int jmax0[R], jmax1[R], jmax2[R];
  float bl0[R], bl1[R], bl2[R];
  {
    const bf16* Kp[3] = {K0, K1, K2};
    const bf16* Vp[3] = {V0, V1, V2};
    const int Sp[3] = {S0, S1, S2};
    int t_last = qt * BR + BR - 1;
    if (t_last > Tq - 1) t_last = Tq - 1;
#pragma unroll
    for (int l = 0; l < 3; ++l) {
      const int S = (Kp[l] && Vp[l]) ? Sp[l] : 0;
      L.S[l] = S;
      L.K[l] = Kp[l] + bh * (long)S * D;
      L.V[l] = Vp[l] + bh * (long)S * D;
      int j_end = S;
      if (causal && t_last + (S - Tq) + 1 < S) j_end = t_last + (S - Tq) + 1;
      if (j_end < 0) j_end = 0;
      L.n[l] = (j_end + BC - 1) / BC;
      L.row_lo[l] = tw0 + (S - Tq);
#pragma unroll
      for (int rb = 0; rb < R; ++rb) {
        const int tq = tw0 + 32 * rb + li;
        const int jm = causal ? min(tq + (S - Tq), S - 1) : S - 1;
        float lam = 1.f;
        if (G && tq < Tq) lam = G[(bh * (long)Tq + tq) * 3 + l];
        const float b = __log2f(lam);  // gate 0 -> -inf: the level never contributes to this row
        if (l == 0) { jmax0[rb] = jm; bl0[rb] = b; }
        if (l == 1) { jmax1[rb] = jm; bl1[rb] = b; }
        if (l == 2) { jmax2[rb] = jm; bl2[rb] = b; }
      }
    }
  }
  const int NT = L.n[0] + L.n[1] + L.n[2];

  f32x16 oacc[R][DB];
  MixRow row[R];
#pragma unroll
  for (int rb = 0; rb < R; ++rb) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[rb][db][r] = 0.f;
    row[rb].m = -INFINITY;
    row[rb].lsum = 0.f;
    row[rb].bl = 0.f;
    row[rb].kb = 0.f;
    row[rb].jmax = 0;
  }

  // ---- staging.  One load instruction fills 1 KiB of a tile (RPI rows); a wave issues IPW of
  // them for K and IPW for V per tile.  Lane i of instruction q serves LDS row RPI q + i / CPR,
  // chunk position i % CPR: the slot and the chunk that belong there are fixed per lane.
  constexpr int RPI = 64 / CPR;                     // tile rows per instruction (4 or 8)
  constexpr int IPW = (BC / RPI) / NW;              // instructions per wave, tile and tensor
  static_assert(IPW >= 1, "every wave issues at least one load per tile and tensor");
  unsigned dslot[IPW], dchunk[IPW];
#pragma unroll
  for (int e = 0; e < IPW; ++e) {
    const int r = RPI * (IPW * wave + e) + lane / CPR;
    dslot[e] = (unsigned)mx_row(r);
    dchunk[e] = 16u * (unsigned)((lane % CPR) ^ mx_swz<D>(r));
  }
  const unsigned lds0 =
      __builtin_amdgcn_readfirstlane((unsigned)(size_t)smem + 1024u * (unsigned)(IPW * wave));
  int kb_w = 0, vb_w = 0;  // ring positions of the next tile to request
  // Two cursors walk the tile stream, one for the requests and one for the tile being consumed:
  // level, first slot, tiles left in the level, and the level's data, which is only touched when
  // the level changes (at most twice per workgroup).
  int rq_l = mx_next_level(L, -1), rq_j0 = 0, rq_left = 0;
  unsigned rq_last = 0;
  const bf16* rq_k = nullptr;
  const bf16* rq_v = nullptr;
  auto rq_level = [&](int l) {
    rq_l = l; rq_j0 = 0;
    rq_left = sel3(l, L.n); rq_last = (unsigned)(sel3(l, L.S) - 1);
    rq_k = sel3(l, L.K); rq_v = sel3(l, L.V);
  };
  // Request the next tile of the stream (past its end: the last tile again, so that every wave
  // always has the same number of loads in flight and the counted waits below stay exact).
  // Rows past the end of a level repeat its last row: their scores are masked, and P = 0 times
  // a finite V is 0.  request_begin fixes the addresses, request_part(q) issues load q of the
  // 2 IPW of the tile (K first), request_end moves the cursor on.
  unsigned rq_off[IPW];
  const bf16* rq_kc = nullptr;
  const bf16* rq_vc = nullptr;
  auto request_begin = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < IPW; ++e)
      rq_off[e] = min((unsigned)rq_j0 + dslot[e], rq_last) * (unsigned)ROWB + dchunk[e];
    rq_kc = rq_k;
    rq_vc = rq_v;
    if (rq_left > 1) {
      rq_j0 += BC;
      --rq_left;
    } else {
      const int nl = mx_next_level(L, rq_l);
      if (nl < 3) rq_level(nl);
    }
  };
  auto request_part = [&](int q) __attribute__((always_inline)) {
    if (q < IPW) mx_dma16(rq_kc, rq_off[q], lds0 + (unsigned)(kb_w * SM::TSZ + 1024 * q));
    else mx_dma16(rq_vc, rq_off[q - IPW], lds0 + (unsigned)(SM::VOFF + vb_w * SM::TSZ + 1024 * (q - IPW)));
#if MKA_DOUBLE & 2
    if (q < IPW) mx_dma16(rq_kc, rq_off[q], lds0 + (unsigned)(kb_w * SM::TSZ + 1024 * q));
    else mx_dma16(rq_vc, rq_off[q - IPW], lds0 + (unsigned)(SM::VOFF + vb_w * SM::TSZ + 1024 * (q - IPW)));
#endif
  };
  auto request_end = [&]() __attribute__((always_inline)) {
    kb_w = kb_w == SM::NKB - 1 ? 0 : kb_w + 1;
    vb_w = vb_w == SM::NVB - 1 ? 0 : vb_w + 1;
  };
  auto request_tile = [&]() __attribute__((always_inline)) {
    request_begin();
#pragma unroll
    for (int q = 0; q < 2 * IPW; ++q) request_part(q);
    request_end();
  };
  constexpr int LPT = 2 * IPW * ((MKA_DOUBLE & 2) ? 2 : 1);  // loads of a wave per tile

  if (NT > 0) {
    // lane constants of the LDS reads
    const unsigned a0 = mx_kfrag0<D>(li, g);
    unsigned x_lo, x_hi;
    mx_trfrag0<D>(lane, x_lo, x_hi);

    // prologue: tiles 0..2 requested, tile 0 landed
    rq_level(rq_l);
    request_tile();
    request_tile();
    request_tile();
    mx_wait_loads<2 * LPT>();
    __syncthreads();

    int kb = 0, vb = 0;  // ring positions of the tile being consumed
    f32x16 s_a[R], s_b[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) s_a[rb] = mx_s_unit<D>(smem, a0, qreg[rb]);
    bf16x8 fr[KK];       // K fragments of unit 1 of tile 0
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      fr[kk] = *reinterpret_cast<const bf16x8*>(smem + 32 * ROWB + (a0 ^ (unsigned)(kk << 5)));
    int l = -1, j0 = 0, left = 1, Sl = 0, row_lo = 0;
    bool need = true;    // the unit in s_a has to take the long way through the reference update
    for (int T = 0; T < NT; ++T) {
      mx_wait_loads<LPT>();  // this wave's part of tile T+1 has landed (T+2 may be in flight)
      loop_barrier();        // tile T+1 complete; K buffer of T and V buffer of T-1 are free
      request_begin();       // tile T+3, issued in four places of the two half steps
      if (left > 1) {
        j0 += BC;
        --left;
      } else {  // first tile of a level (T < NT: there is one)
        l = mx_next_level(L, l);
        j0 = 0;
        left = sel3(l, L.n); Sl = sel3(l, L.S); row_lo = sel3(l, L.row_lo);
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
          row[rb].jmax = l == 0 ? jmax0[rb] : (l == 1 ? jmax1[rb] : jmax2[rb]);
          row[rb].bl = l == 0 ? bl0[rb] : (l == 1 ? bl1[rb] : bl2[rb]);
          // no reference yet: +inf (NaN with a zero gate) sends the first unit the long way
          row[rb].kb = row[rb].bl - row[rb].m;
          need = true;
        }
      }
      const int kb1 = kb == SM::NKB - 1 ? 0 : kb + 1;
      const char* sK1 = smem + kb1 * SM::TSZ;
      const char* sV = smem + SM::VOFF + vb * SM::TSZ;
      const bool mask0 = (j0 + 32 > Sl) || (causal && j0 + 31 > row_lo);
      const bool mask1 = (j0 + 64 > Sl) || (causal && j0 + 63 > row_lo);
      // parts of the request per section: 2 IPW loads over 4 sections
      constexpr int PPS = (2 * IPW + 3) / 4;
      auto part = [&](int sct) __attribute__((always_inline)) {
#pragma unroll
        for (int q = sct * PPS; q < (sct + 1) * PPS && q < 2 * IPW; ++q) request_part(q);
      };
      auto p0 = [&]() __attribute__((always_inline)) { part(0); };
      auto p1 = [&]() __attribute__((always_inline)) { part(1); };
      auto p2 = [&]() __attribute__((always_inline)) { part(2); };
      auto p3 = [&]() __attribute__((always_inline)) { part(3); };
      // first half step: unit 0 of tile T; S^T of its unit 1; K fragments of unit 0 of tile T+1
      if (mask0) mx_half_step<D, R, true, 0>(p0, p1, s_a, s_b, fr, sK1, a0, j0, sV, x_lo, x_hi, qreg, oacc, row, c, lane, need);
      else mx_half_step<D, R, false, 0>(p0, p1, s_a, s_b, fr, sK1, a0, j0, sV, x_lo, x_hi, qreg, oacc, row, c, lane, need);
      // second half step: unit 1 of tile T; S^T of unit 0 of tile T+1; K fragments of its unit 1
      if (mask1) mx_half_step<D, R, true, 1>(p2, p3, s_b, s_a, fr, sK1 + 32 * ROWB, a0, j0 + 32, sV, x_lo, x_hi, qreg, oacc, row, c, lane, need);
      else mx_half_step<D, R, false, 1>(p2, p3, s_b, s_a, fr, sK1 + 32 * ROWB, a0, j0 + 32, sV, x_lo, x_hi, qreg, oacc, row, c, lane, need);
      request_end();
      kb = kb1;
      vb = vb == SM::NVB - 1 ? 0 : vb + 1;
    }
    mx_wait_loads<0>();  // the surplus requests of the last tiles must land before LDS is reused
    __syncthreads();     // every wave is done with the tile buffers (the epilogue reuses them)
  }

  // ---- epilogue: normalise, transpose O^T through LDS, store rows with coalesced 16-byte writes
  {
    constexpr int OSTR = D + 8;
    bf16* sO = reinterpret_cast<bf16*>(smem) + wave * (32 * R * OSTR);
    float lsum[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
      lsum[rb] = row[rb].lsum + xor32(row[rb].lsum);
      const float inv = lsum[rb] > 0.f ? 1.f / lsum[rb] : 0.f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int d = 32 * db + 8 * (r >> 2) + 4 * g + (r & 3);
          sO[(32 * rb + li) * OSTR + d] = (bf16)(oacc[rb][db][r] * inv);
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32 * R * CPR / 64; ++i) {
      const int item = lane + 64 * i;
      const int rr = item / CPR, ch = item % CPR;
      const uint4 v = *reinterpret_cast<const uint4*>(&sO[rr * OSTR + ch * 8]);
      if (tw0 + rr < Tq)
        *reinterpret_cast<uint4*>(O + (bh * (long)Tq + tw0 + rr) * D + ch * 8) = v;
    }
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
      const int tq = tw0 + 32 * rb + li;
      if (LSE && g == 0 && tq < Tq)
        LSE[bh * (long)Tq + tq] = lsum[rb] > 0.f ? (row[rb].m + __log2f(lsum[rb])) * kLn2 : -INFINITY;
    }
  }
}

template <int D, int R>
__global__ __launch_bounds__(MixShape<R>::NT, 1) void mix_bf16_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S0, int S1, int S2, int causal, float c, int n_qtiles,
    int BH, int interleave, int pair) {
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
  if (bh >= BH || qt0 < n_qtiles - n_first) return;
  const int qt1 = n_qtiles - 1 - qt0;
  mix_tile<D, R>(Q, K0, K1, K2, V0, V1, V2, G, O, LSE, Tq, S0, S1, S2, causal, c, qt0, bh);
  if (pair && qt1 != qt0) {
    __syncthreads();  // the first tile's output staging is dead
    mix_tile<D, R>(Q, K0, K1, K2, V0, V1, V2, G, O, LSE, Tq, S0, S1, S2, causal, c, qt1, bh);
  }
}

template <int D, int R>
hipError_t launch_mix_t(const MixArgs& a, hipStream_t st) {
  constexpr int BR = MX_BR;
  const int n_qtiles = (a.Tq + BR - 1) / BR;
  // under a causal mask a workgroup takes a heavy and a light query tile (see the kernel;
  // measured at T = 4096, B*H = 128: 10 % off the launch)
  const int pair = (a.causal && n_qtiles > 1) ? 1 : 0;
  const int n_first = pair ? (n_qtiles + 1) / 2 : n_qtiles;
  const long nblocks = (long)n_first * ((a.BH + 7) / 8) * 8;
  const int interleave = (!pair && nblocks <= 2 * 256) ? 1 : 0;
  const size_t smem = (size_t)MixSmem<D>::TOTAL;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mix_bf16_kernel<D, R>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // a level without memory gets a valid pointer and length 0 (never dereferenced beyond row 0,
  // which is not loaded either: it has no tiles)
  const void* anyK = a.K[0] ? a.K[0] : (a.K[1] ? a.K[1] : a.K[2]);
  const void* anyV = a.V[0] ? a.V[0] : (a.V[1] ? a.V[1] : a.V[2]);
  if (!anyK || !anyV) return hipErrorInvalidValue;
  const void* Kp[3];
  const void* Vp[3];
  int Sp[3];
  for (int l = 0; l < 3; ++l) {
    const bool has = a.K[l] && a.V[l] && a.S[l] > 0;
    Kp[l] = has ? a.K[l] : anyK;
    Vp[l] = has ? a.V[l] : anyV;
    Sp[l] = has ? a.S[l] : 0;
  }
  hipLaunchKernelGGL((mix_bf16_kernel<D, R>), dim3((unsigned)nblocks), dim3(MixShape<R>::NT), smem, st,
                     (const bf16*)a.Q, (const bf16*)Kp[0], (const bf16*)Kp[1], (const bf16*)Kp[2],
                     (const bf16*)Vp[0], (const bf16*)Vp[1], (const bf16*)Vp[2], a.G, (bf16*)a.O,
                     a.LSE, a.Tq, Sp[0], Sp[1], Sp[2], a.causal, a.scale * kLog2e, n_qtiles, a.BH,
                     interleave, pair);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_mix_bf16(const MixArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  return a.d == 128 ? launch_mix_t<128, MX_R>(a, st) : launch_mix_t<64, 1>(a, st);
}

}  // namespace mka
