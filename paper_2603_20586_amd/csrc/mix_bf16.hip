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
// pipelined (the S^T MFMAs of the next unit between the exponentials of the current one), the
// barrier that publishes a tile in the middle of the previous one (two K buffers, three V).
// Differences: both tiles are staged as plain row copies (a thread moves one 16-byte chunk of K
// and one of V per half step); V stays row-major and its transpose for the second product is
// read with ds_read_b64_tr_b16; the slots of a tile are permuted over the LDS rows (j = 4a+b ->
// row 4b+a inside every 16) so that both the row reads and the transposed reads are free of
// bank conflicts.
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int MX_BC = 64;  // slots per KV tile
constexpr int MX_NW = 8;   // waves per workgroup
constexpr int MX_NT = MX_NW * 64;

template <int D>
struct MixSmem {
  static constexpr int RSTR = D + 8;         // bf16 per tile row (16-byte pad)
  static constexpr int TSZ = MX_BC * RSTR;   // one tile
  static constexpr int VOFF = 2 * TSZ;       // two K tiles, then three V tiles
  static constexpr int TOTAL = 5 * TSZ;      // bf16 elements
};

// LDS row of slot j (0..63) of a tile
__device__ __forceinline__ int mx_row(int j) {
  return (j & ~15) | ((j & 3) << 2) | ((j >> 2) & 3);
}

struct MixLevels {
  const bf16* K[3];
  const bf16* V[3];
  int S[3];      // slots of the level (0: absent)
  int n[3];      // tiles of the level that this workgroup visits
  int jmax[3];   // last slot the lane's row sees (may be negative)
  int row_lo[3]; // last slot the wave's FIRST row sees
  float bl[3];   // log2 of the lane's gate
};

// element l of a 3-array without dynamic indexing (which would put the array in scratch memory)
template <typename T>
__device__ __forceinline__ T sel3(int l, const T (&a)[3]) {
  return l == 0 ? a[0] : (l == 1 ? a[1] : a[2]);
}

// stream tile T -> level and first slot
__device__ __forceinline__ void mx_tile_of(const MixLevels& L, int T, int& l, int& j0) {
  l = (T >= L.n[0]) + (T >= L.n[0] + L.n[1]);
  const int start = l == 0 ? 0 : (l == 1 ? L.n[0] : L.n[0] + L.n[1]);
  j0 = (T - start) * MX_BC;
}

template <int D>
__device__ __forceinline__ f32x16 mx_s_unit(const bf16* sK, int unit, const bf16x8 (&qreg)[D / 16],
                                            int li, int g) {
  constexpr int RSTR = D + 8, KK = D / 16;
  f32x16 sacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
  const bf16* arow = &sK[mx_row(32 * unit + li) * RSTR + 8 * g];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    sacc = mfma32(*reinterpret_cast<const bf16x8*>(arow + 16 * kk), qreg[kk], sacc);
  return sacc;
}

// One half step of a wave: finish the unit whose S^T is s_now (32 slots from jb of a level with
// log2-gate bl and visibility limit jmax), issue the S^T of unit `unit_n` of the K tile at sKn.
// m is the running reference exponent in log2 units (gate included); register r of s_now <->
// slot jb + 8 (r/4) + 4 g + r%4 of the lane's row.
template <int D, bool MASK>
__device__ __forceinline__ void mx_half_step(f32x16 s_now, f32x16& s_next, const bf16* sKn,
                                             int unit_n, int jb, int jmax, float bl,
                                             const bf16* sV, int unit,
                                             const bf16x8 (&qreg)[D / 16], f32x16 (&oacc)[D / 32],
                                             float& m, float& lsum, float c, int lane) {
  constexpr int RSTR = D + 8, KK = D / 16, DB = D / 32;
  constexpr int PF = 4;          // LDS fragments in flight
  constexpr int EPK = 16 / KK;   // exponentials per S MFMA
  constexpr int NPV = 2 * DB;    // PV MFMAs of the unit
  const int g = lane >> 5, li = lane & 31;
  bf16x8 fr[PF];
  const bf16* arow = &sKn[mx_row(32 * unit_n + li) * RSTR + 8 * g];
#pragma unroll
  for (int kk = 0; kk < PF; ++kk) fr[kk] = *reinterpret_cast<const bf16x8*>(arow + 16 * kk);

  if (MASK) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = jb + 8 * (r >> 2) + 4 * g + (r & 3);
      if (j > jmax) s_now[r] = -INFINITY;
    }
  }
  float mx = fmaxf(s_now[0], s_now[1]);
#pragma unroll
  for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s_now[r]);
  mx = fmaxf(mx, xor32(mx));
  // Lazy max-shift (as in the route-fused forward): the reference exponent only moves when the
  // row's largest exponent has grown by more than 8, so P may reach 2^8 and the rescale of the
  // accumulators is skipped on almost every unit.
  const float cand = (mx == -INFINITY) ? -INFINITY : fmaf(mx, c, bl);
  const bool move = cand - m > 8.f || (m == -INFINITY && cand > -INFINITY);
  const float m_new = move ? cand : m;
  const float alpha = move ? ((m == -INFINITY) ? 0.f : fast_exp2(m - m_new)) : 1.f;
  const float kb = bl - ((m_new == -INFINITY) ? 0.f : m_new);
  m = m_new;
  if (__any(move)) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
  }

  // V^T fragment of PV MFMA i (rows 32 (i % DB) of V^T, k-step i / DB): the transpose of 8 slots
  // x 32 head dims of the row-major V tile.  k positions 0..3 <-> slots 16 ks + 4 g + 0..3,
  // positions 4..7 <-> 8 further: the slots whose P values the lane holds in registers 8 ks ..
  const int ti = lane & 15, gsel = (lane >> 4) & 1;
  const bf16* vcol = sV + 16 * gsel + 4 * (ti & 3);
  auto v_frag = [&](int i) __attribute__((always_inline)) {
    const int db = i % DB, ks = i / DB;
    const int j0 = 32 * unit + 16 * ks + 4 * g + (ti >> 2);
    const uint2 lo = lds_read_tr(vcol + mx_row(j0) * RSTR + 32 * db);
    const uint2 hi = lds_read_tr(vcol + mx_row(j0 + 8) * RSTR + 32 * db);
    return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
  };

  // -- section A: S^T of the next unit, between the exponentials of this one
  f32x16 sn;
#pragma unroll
  for (int r = 0; r < 16; ++r) sn[r] = 0.f;
  float p[16];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    sn = mfma32(fr[kk % PF], qreg[kk], sn);
    if (kk + PF < KK) {
      fr[kk % PF] = *reinterpret_cast<const bf16x8*>(arow + 16 * (kk + PF));
    } else {  // the K fragments are all on their way: start on the V^T fragments
      const int i = kk + PF - KK;
      if (i < NPV) fr[kk % PF] = v_frag(i);
    }
#pragma unroll
    for (int r = kk * EPK; r < (kk + 1) * EPK; ++r) {
      float e = fast_exp2(fmaf(s_now[r], c, kb));
      if (MASK) e = (s_now[r] == -INFINITY) ? 0.f : e;  // also covers c == 0
      p[r] = e;
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  s_next = sn;
  const uint4 pk0 = pack8(&p[0]), pk1 = pack8(&p[8]);
  const bf16x8 p0 = __builtin_bit_cast(bf16x8, pk0);
  const bf16x8 p1 = __builtin_bit_cast(bf16x8, pk1);
  // row sum of the bf16-rounded P (what the PV product uses), two values per instruction
  const bf16x2 ones = {(bf16)1.f, (bf16)1.f};
  float psum = 0.f;
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk0.x), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk0.y), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk0.z), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk0.w), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk1.x), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk1.y), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk1.z), ones, psum, false);
  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk1.w), ones, psum, false);
  lsum = lsum * alpha + psum;
  __builtin_amdgcn_sched_barrier(0);

  // -- section B: O^T += V^T P^T
#pragma unroll
  for (int i = 0; i < NPV; ++i) {
    constexpr int KP = KK % PF;  // ring position of PV fragment 0
    oacc[i % DB] = mfma32(fr[(KP + i) % PF], i / DB ? p1 : p0, oacc[i % DB]);
    if (i + PF < NPV) fr[(KP + i) % PF] = v_frag(i + PF);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int D>
__global__ __launch_bounds__(MX_NT, 1) void mix_bf16_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S0, int S1, int S2, int causal, float c, int n_qtiles,
    int BH, int interleave) {
  using SM = MixSmem<D>;
  constexpr int BR = MX_NW * 32, BC = MX_BC, RSTR = SM::RSTR;
  constexpr int KK = D / 16, DB = D / 32, CPR = D / 8;
  constexpr int RP = MX_NT / CPR;  // tile rows the workgroup copies per half step (32 or 64)
  extern __shared__ __attribute__((aligned(16))) unsigned char mx_smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(mx_smem_raw);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
  // all query tiles of one (batch, head) on ONE XCD (block index = 8 * slot + xcd), heaviest
  // tiles first; heads interleaved on small grids (shorter causal tail)
  const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
  int qt, hl;
  if (interleave) {
    const int hpx = (BH + 7) / 8;
    qt = n_qtiles - 1 - slot / hpx;
    hl = slot % hpx;
  } else {
    qt = n_qtiles - 1 - slot % n_qtiles;
    hl = slot / n_qtiles;
  }
  const long bh = (long)hl * 8 + xcd;
  if (bh >= BH) return;
  const int tw0 = qt * BR + wave * 32;  // first row of this wave
  const int tq = tw0 + li;              // this lane's row

  bf16x8 qreg[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 u = make_uint4(0, 0, 0, 0);
    if (tq < Tq) u = *reinterpret_cast<const uint4*>(Q + (bh * (long)Tq + tq) * D + 16 * kk + 8 * g);
    qreg[kk] = __builtin_bit_cast(bf16x8, u);
  }

  MixLevels L;
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
      L.jmax[l] = causal ? min(tq + (S - Tq), S - 1) : S - 1;
      L.row_lo[l] = tw0 + (S - Tq);
      float lam = 1.f;
      if (G && tq < Tq) lam = G[(bh * (long)Tq + tq) * 3 + l];
      L.bl[l] = __log2f(lam);  // gate 0 -> -inf: the level never contributes to this row
    }
  }
  const int NT = L.n[0] + L.n[1] + L.n[2];

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  // ---- staging: pair p = (tile p / 2, half p % 2) of the tile stream; a thread owns one 16-byte
  // chunk of K and one of V of the pair (d = 64: the first pair of a tile is the whole tile)
  // Everything per thread is precomputed: byte offset of its chunk inside a row block, LDS
  // offsets of the two halves; per pair only the (uniform) level base and first slot change.
  const int crow = tid / CPR, ccol = (tid % CPR) * 8;
  const unsigned lds_o[2] = {(unsigned)(mx_row(crow) * RSTR + ccol),
                             (unsigned)(mx_row((RP + crow) & (BC - 1)) * RSTR + ccol)};
  const unsigned g_o = (unsigned)(crow * D + ccol) * 2u;  // bytes from the pair's first row
  uint4 rk = make_uint4(0, 0, 0, 0), rv = make_uint4(0, 0, 0, 0);
  auto pair_active = [&](int p) { return (p >> 1) < NT && (RP * (p & 1) < BC); };
  auto load_pair = [&](int p) __attribute__((always_inline)) {
    if (!pair_active(p)) return;
    int l, j0;
    mx_tile_of(L, p >> 1, l, j0);
    const int jp = j0 + RP * (p & 1);  // first slot of the pair (uniform)
    const int Sl = sel3(l, L.S);
    const char* kp = reinterpret_cast<const char*>(sel3(l, L.K)) + (unsigned)jp * (unsigned)(D * 2);
    const char* vp = reinterpret_cast<const char*>(sel3(l, L.V)) + (unsigned)jp * (unsigned)(D * 2);
    if (jp + RP <= Sl) {  // all rows of the pair exist (uniform)
      rk = *reinterpret_cast<const uint4*>(kp + g_o);
      rv = *reinterpret_cast<const uint4*>(vp + g_o);
    } else {  // tail of the level: rows past its end are zeros (P is 0 there, 0 * garbage is not)
      const bool valid = jp + crow < Sl;
      const unsigned o = valid ? g_o : (unsigned)(ccol * 2) - (unsigned)jp * (unsigned)(D * 2);
      rk = *reinterpret_cast<const uint4*>(kp + (int)o);
      rv = *reinterpret_cast<const uint4*>(vp + (int)o);
      if (!valid) {
        rk = make_uint4(0, 0, 0, 0);
        rv = make_uint4(0, 0, 0, 0);
      }
    }
  };
  int kbuf_w = 0, vbuf_w = 0;  // buffers of the tile that the next write_pair targets
  auto write_pair = [&](int p) __attribute__((always_inline)) {
    if (pair_active(p)) {
      const unsigned o = lds_o[p & 1];
      *reinterpret_cast<uint4*>(&smem[kbuf_w * SM::TSZ + o]) = rk;
      *reinterpret_cast<uint4*>(&smem[SM::VOFF + vbuf_w * SM::TSZ + o]) = rv;
    }
    if (p & 1) {  // tile finished: move on to the next one's buffers
      kbuf_w ^= 1;
      vbuf_w = vbuf_w == 2 ? 0 : vbuf_w + 1;
    }
  };

  if (NT > 0) {
    // prologue: tile 0 and the first half of tile 1 in LDS, the second half in flight
#pragma unroll
    for (int p = 0; p < 3; ++p) {
      load_pair(p);
      write_pair(p);
    }
    load_pair(3);
    __syncthreads();

    f32x16 s_a = mx_s_unit<D>(smem, 0, qreg, li, g), s_b;
    int vb = 0;  // V buffer of the tile being consumed
    int l_cur, j0_cur;
    mx_tile_of(L, 0, l_cur, j0_cur);
    for (int T = 0; T < NT; ++T) {
      const bf16* sK = smem + (T & 1) * SM::TSZ;
      const bf16* sK1 = smem + ((T + 1) & 1) * SM::TSZ;
      const bf16* sV = smem + SM::VOFF + vb * SM::TSZ;
      const int l = l_cur, j0 = j0_cur;
      const int Sl = sel3(l, L.S), jmax = sel3(l, L.jmax), row_lo = sel3(l, L.row_lo);
      const float bl = sel3(l, L.bl);
      const bool mask0 = (j0 + 32 > Sl) || (causal && j0 + 31 > row_lo);
      const bool mask1 = (j0 + 64 > Sl) || (causal && j0 + 63 > row_lo);
      // first half step: unit 0 of tile T; staging pair 2T+3 written, 2T+4 loaded
      if (mask0) mx_half_step<D, true>(s_a, s_b, sK, 1, j0, jmax, bl, sV, 0, qreg, oacc, m, lsum, c, lane);
      else mx_half_step<D, false>(s_a, s_b, sK, 1, j0, jmax, bl, sV, 0, qreg, oacc, m, lsum, c, lane);
      write_pair(2 * T + 3);
      load_pair(2 * T + 4);
      __syncthreads();  // tile T+1 is complete in LDS; K buffer T&1 may be overwritten
      // second half step: unit 1 of tile T (S^T of unit 0 of tile T+1 goes in flight)
      if (mask1) mx_half_step<D, true>(s_b, s_a, sK1, 0, j0 + 32, jmax, bl, sV, 1, qreg, oacc, m, lsum, c, lane);
      else mx_half_step<D, false>(s_b, s_a, sK1, 0, j0 + 32, jmax, bl, sV, 1, qreg, oacc, m, lsum, c, lane);
      write_pair(2 * T + 4);
      load_pair(2 * T + 5);
      vb = vb == 2 ? 0 : vb + 1;
      if (T + 1 < NT) mx_tile_of(L, T + 1, l_cur, j0_cur);
    }
    __syncthreads();  // every wave is done with the tile buffers (the epilogue reuses them)
  }

  // ---- epilogue: normalise, transpose O^T through LDS, store rows with coalesced 16-byte writes
  lsum += xor32(lsum);
  {
    constexpr int OSTR = D + 8;
    bf16* sO = smem + wave * (32 * OSTR);
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int d = 32 * db + 8 * (r >> 2) + 4 * g + (r & 3);
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
    if (LSE && g == 0 && tq < Tq)
      LSE[bh * (long)Tq + tq] = lsum > 0.f ? (m + __log2f(lsum)) * kLn2 : -INFINITY;
  }
}

template <int D>
hipError_t launch_mix_t(const MixArgs& a, hipStream_t st) {
  constexpr int BR = MX_NW * 32;
  const int n_qtiles = (a.Tq + BR - 1) / BR;
  const long nblocks = (long)n_qtiles * ((a.BH + 7) / 8) * 8;
  const int interleave = nblocks <= 2 * 256 ? 1 : 0;
  const size_t smem = (size_t)MixSmem<D>::TOTAL * sizeof(bf16);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mix_bf16_kernel<D>),
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
  hipLaunchKernelGGL((mix_bf16_kernel<D>), dim3((unsigned)nblocks), dim3(MX_NT), smem, st,
                     (const bf16*)a.Q, (const bf16*)Kp[0], (const bf16*)Kp[1], (const bf16*)Kp[2],
                     (const bf16*)Vp[0], (const bf16*)Vp[1], (const bf16*)Vp[2], a.G, (bf16*)a.O,
                     a.LSE, a.Tq, Sp[0], Sp[1], Sp[2], a.causal, a.scale * kLog2e, n_qtiles, a.BH,
                     interleave);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_mix_bf16(const MixArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  return a.d == 128 ? launch_mix_t<128>(a, st) : launch_mix_t<64>(a, st);
}

}  // namespace mka
