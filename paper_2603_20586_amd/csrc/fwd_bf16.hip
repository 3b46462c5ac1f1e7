// Route-fused attention forward, bf16 MFMA path (paper: Alg. 2 steps 6-7 and 9; attention as
// Eq. (1) with the scale of Eq. (3); online softmax by the max-shift recursion of the section
// "Numerical Stability via Max-Shift", applied over KV blocks with one running max per row).
//
// One workgroup = 8 waves x 32 query rows = 256 rows.  KV tiles of 64 slots, double-buffered in
// LDS, one barrier per tile:
//   * fusion (Kf = sum_l G_l K_l, Vf likewise) happens in registers between the global load and
//     the LDS write: raw 16-byte chunks of the three levels are prefetched one tile ahead, mixed
//     in f32, rounded once to bf16; the fused stream exists only in LDS.  Waves 0-3 fuse the K
//     half of a tile AFTER their MFMA work, waves 4-7 fuse the V half BEFORE theirs, so that on
//     each SIMD one wave's VALU work runs beside the other wave's MFMAs.
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
  static constexpr int BUF = KSZ + VSZ;    // one buffer: Kf then Vf^T
  static constexpr int TOTAL = 2 * BUF;    // bf16 elements
};

// ---- raw (unfused) data of half a tile, prefetched into registers -------------------------
// One register set serves both halves (a wave only ever holds one of them): up to 4 chunks of
// three levels plus the gates of their slots.
struct HalfRaw {
  Raw3 r[4];
  float g[4][3];
};
template <int D>
struct KRaw {
  static constexpr int N = FW_BC * (D / 8) / FW_NG;  // chunks per thread (4 for d=128, 2 for d=64)
};

// tg = thread index inside the fusion group (0..255)
template <int D, bool FULL>
__device__ __forceinline__ void load_k(HalfRaw& x, const bf16* __restrict__ K0,
                                       const bf16* __restrict__ K1, const bf16* __restrict__ K2,
                                       const float* __restrict__ Gb, int j0, int S,
                                       int len0, int len1, int len2, int tg) {
  constexpr int CPR = D / 8, RPP = FW_NG / CPR;  // rows per pass
  const int cc = tg % CPR;
#pragma unroll
  for (int i = 0; i < KRaw<D>::N; ++i) {
    const int j = j0 + tg / CPR + RPP * i;
    const int jc = FULL ? j : (j < S ? j : S - 1);
    const bool in = FULL || j < S;
    x.r[i] = load_raw3_b<FULL>(K0, K1, K2, (unsigned)(cc * 16), (unsigned)(jc * D + cc * 8) * 2u, in && j < len0,
                                  in && j < len1, in && j < len2);
    const char* gp = reinterpret_cast<const char*>(Gb) + (unsigned)(jc * 12);
    x.g[i][0] = *reinterpret_cast<const float*>(gp);
    x.g[i][1] = *reinterpret_cast<const float*>(gp + 4);
    x.g[i][2] = *reinterpret_cast<const float*>(gp + 8);
  }
}

template <int D>
__device__ __forceinline__ void fuse_store_k(const HalfRaw& x, bf16* sK, int tg) {
  constexpr int CPR = D / 8, RPP = FW_NG / CPR, KSTR = D + 8;
  const int cc = tg % CPR;
#pragma unroll
  for (int i = 0; i < KRaw<D>::N; ++i) {
    const int row = tg / CPR + RPP * i;
    float acc[8];
    fuse8(x.r[i], x.g[i][0], x.g[i][1], x.g[i][2], acc);
    *reinterpret_cast<uint4*>(&sK[row * KSTR + cc * 8]) = pack8(acc);
  }
}

// V work item = (4 consecutive slots, one 16-byte chunk).  Thread bits: [2:0] chunk low bits,
// [3] slot-group bit 1 (selects the 8-byte half of a 16-byte column block), [4] slot-group bit 0,
// [6:5] slot-group bits 3:2, [7] chunk bit 3.  A 16-lane LDS write group is then 8 chunks x 2
// halves, which (with the row permutation of the Vf^T tile) covers every bank exactly once.
template <int D>
__device__ __forceinline__ void v_item(int tg, int& sg, int& cc, bool& active) {
  constexpr int CPR = D / 8;
  sg = (((tg >> 3) & 1) << 1) | ((tg >> 4) & 1) | (((tg >> 5) & 3) << 2);
  cc = (tg & 7) | ((tg >> 7) << 3);
  active = cc < CPR;
  if (!active) cc = 0;
}

template <int D, bool FULL>
__device__ __forceinline__ void load_v(HalfRaw& x, const bf16* __restrict__ V0,
                                       const bf16* __restrict__ V1, const bf16* __restrict__ V2,
                                       const float* __restrict__ Gb, int j0, int S,
                                       int len0, int len1, int len2, int tg) {
  int sg, cc;
  bool active;
  v_item<D>(tg, sg, cc, active);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int j = j0 + sg * 4 + u;
    const int jc = FULL ? j : (j < S ? j : S - 1);
    const bool in = FULL || j < S;
    x.r[u] = load_raw3_b<FULL>(V0, V1, V2, (unsigned)(cc * 16), (unsigned)(jc * D + cc * 8) * 2u, in && j < len0,
                                  in && j < len1, in && j < len2);
    const char* gp = reinterpret_cast<const char*>(Gb) + (unsigned)(jc * 12);
    x.g[u][0] = *reinterpret_cast<const float*>(gp);
    x.g[u][1] = *reinterpret_cast<const float*>(gp + 4);
    x.g[u][2] = *reinterpret_cast<const float*>(gp + 8);
  }
}

template <int D>
__device__ __forceinline__ void fuse_store_v(const HalfRaw& x, bf16* sVT, int tg) {
  constexpr int VSTR = FW_BC + 8;
  int sg, cc;
  bool active;
  v_item<D>(tg, sg, cc, active);
  if (!active) return;
  float vf[4][8];
#pragma unroll
  for (int u = 0; u < 4; ++u) fuse8(x.r[u], x.g[u][0], x.g[u][1], x.g[u][2], vf[u]);
  // slots 4 sg .. 4 sg + 3 go to columns col .. col + 3 (bits 2,3 of the slot index swapped)
  const int col = 32 * (sg >> 3) + fw_swap23(4 * (sg & 7));
  const int blk = col >> 3, half = (col >> 2) & 1;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int prow = e * (D / 8) + cc;  // LDS row of head-dim index d = 8 cc + e
    uint2 w;
    w.x = pack_bf16x2(vf[0][e], vf[1][e]);
    w.y = pack_bf16x2(vf[2][e], vf[3][e]);
    *reinterpret_cast<uint2*>(&sVT[prow * VSTR + 8 * blk + 4 * half]) = w;
  }
}

// ---- MFMA work of one tile: two sub-steps of 32 slots ----------------------------------------
template <int D, bool MASK>
__device__ __forceinline__ void compute_tile(const bf16* sK, const bf16* sVT,
                                             const bf16x8 (&qreg)[D / 16], f32x16 (&oacc)[D / 32],
                                             float& m, float& lsum, float c, int j0, int jmax,
                                             int li, int g) {
  constexpr int KSTR = D + 8, VSTR = FW_BC + 8, KK = D / 16, DB = D / 32;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
    const bf16* arow = &sK[(32 * sb + li) * KSTR + 8 * g];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + 16 * kk);
      sacc = mfma32(a, qreg[kk], sacc);
    }
    // register r <-> slot j0 + 32 sb + 8 (r/4) + 4 g + r%4 of this lane's row
    if (MASK) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = j0 + 32 * sb + 8 * (r >> 2) + 4 * g + (r & 3);
        if (j > jmax) sacc[r] = -INFINITY;
      }
    }
    float mx = fmaxf(sacc[0], sacc[1]);
#pragma unroll
    for (int r = 2; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
    mx = fmaxf(mx, xor32(mx));
    // Lazy max-shift: the reference m only moves when the row max has grown by more than 2^8
    // in the exponent; until then P = exp2(c (s - m)) may exceed 1 (at most 256), which bf16 and
    // the f32 sums hold without loss, and the rescale of the accumulators is skipped.  The
    // recursion is unchanged (O and z are always relative to the same m), only m is stale.
    // Every row sees slot 0, so m is finite after the first sub-step that has a visible slot.
    const bool move = (mx - m) * c > 8.f || m == -INFINITY;
    const float m_new = move ? mx : m;
    const float alpha = move ? ((m == -INFINITY) ? 0.f : fast_exp2((m - m_new) * c)) : 1.f;
    const float mc = (m_new == -INFINITY) ? 0.f : m_new * c;
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float e = fast_exp2(fmaf(sacc[r], c, -mc));
      if (MASK) e = (sacc[r] == -INFINITY) ? 0.f : e;  // also covers c == 0
      p[r] = e;
    }
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
    m = m_new;
    if (__any(move)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    // O^T += Vf^T P^T: k-step ks covers columns 16 ks .. 16 ks + 15 of the Vf^T tile
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const bf16* vrow = &sVT[(32 * db + li) * VSTR];  // LDS rows: see the row permutation
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(vrow + 8 * (4 * sb + 0 + g));
      const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(vrow + 8 * (4 * sb + 2 + g));
      oacc[db] = mfma32(a0, p0, oacc[db]);
      oacc[db] = mfma32(a1, p1, oacc[db]);
    }
  }
}

template <int D>
__global__ __launch_bounds__(FW_NW * 64, 1) void fwd_bf16_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K0, const bf16* __restrict__ K1,
    const bf16* __restrict__ K2, const bf16* __restrict__ V0, const bf16* __restrict__ V1,
    const bf16* __restrict__ V2, const float* __restrict__ G, bf16* __restrict__ O,
    float* __restrict__ LSE, int Tq, int S, int len0, int len1, int len2, int causal, float c,
    float tau, int n_qtiles, int BH, int interleave) {
  using L = FwdSmem<D>;
  constexpr int BR = FW_NW * 32, BC = FW_BC;
  constexpr int KK = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char fw_smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(fw_smem_raw);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
  const bool grpV = wave >= 4;  // waves 4-7 fuse the V half, waves 0-3 the K half
  const int tg = tid & (FW_NG - 1);
  // Workgroups are handed to the 8 XCDs round-robin by block index.  All query tiles of one
  // (batch, head) are given to ONE XCD (block index = 8 * slot + xcd), so that the workgroups
  // that stream the same K/V tiles share that XCD's L2; heavy (late) query tiles go first so
  // that the causal tail is short.
  const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
  int qt, hl;
  if (interleave) {  // small grids: heaviest tiles of ALL the XCD's heads first (shorter tail)
    const int hpx = (BH + 7) / 8;
    qt = n_qtiles - 1 - slot / hpx;
    hl = slot % hpx;
  } else {           // large grids: one head after the other (best L2 reuse of its K/V tiles)
    qt = n_qtiles - 1 - slot % n_qtiles;
    hl = slot / n_qtiles;
  }
  const long bh = (long)hl * 8 + xcd;
  if (bh >= BH) return;  // the head count need not be a multiple of 8
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
  float m = -INFINITY, lsum = 0.f;

  int t_last = qt * BR + BR - 1;
  if (t_last > Tq - 1) t_last = Tq - 1;
  int j_end = S;
  if (causal && t_last + off + 1 < S) j_end = t_last + off + 1;
  const int ntiles = (j_end + BC - 1) / BC;
  const int lenmin = min(len0, min(len1, len2));
  const int jmax = causal ? (tq + off < S - 1 ? tq + off : S - 1) : S - 1;

  HalfRaw raw = {};  // fully defined on every path, so that it lives in registers
  // waves 0-3 own the K half of every tile, waves 4-7 the V half
  auto load_half = [&](int jt) {
    const int j0 = jt * BC;
    const bool full = j0 + BC <= lenmin;
    if (!grpV) {
      if (full) load_k<D, true>(raw, K0b, K1b, K2b, Gb, j0, S, len0, len1, len2, tg);
      else load_k<D, false>(raw, K0b, K1b, K2b, Gb, j0, S, len0, len1, len2, tg);
    } else {
      if (full) load_v<D, true>(raw, V0b, V1b, V2b, Gb, j0, S, len0, len1, len2, tg);
      else load_v<D, false>(raw, V0b, V1b, V2b, Gb, j0, S, len0, len1, len2, tg);
    }
  };
  auto store_half = [&](int buf) {
    bf16* sK = smem + buf * L::BUF;
    if (!grpV) fuse_store_k<D>(raw, sK, tg);
    else fuse_store_v<D>(raw, sK + L::KSZ, tg);
  };

  // prologue: tile 0 into buffer 0, raw data of tile 1 into registers
  load_half(0);
  store_half(0);
  if (ntiles > 1) load_half(1);
  __syncthreads();

  for (int jt = 0; jt < ntiles; ++jt) {
    const bool has1 = jt + 1 < ntiles, has2 = jt + 2 < ntiles;
    // the V group fuses tile jt+1 before its MFMA work, the K group after: on every SIMD one
    // wave's VALU-heavy fusion then runs beside the other wave's MFMAs
    if (grpV && has1) {
      store_half((jt + 1) & 1);
      if (has2) load_half(jt + 2);
    }
    {
      const bf16* sK = smem + (jt & 1) * L::BUF;
      const bf16* sVT = sK + L::KSZ;
      const int j0 = jt * BC;
      const bool need_mask = (j0 + BC > S) || (causal && (j0 + BC - 1 > tw0 + off));
      if (need_mask) compute_tile<D, true>(sK, sVT, qreg, oacc, m, lsum, c, j0, jmax, li, g);
      else compute_tile<D, false>(sK, sVT, qreg, oacc, m, lsum, c, j0, jmax, li, g);
    }
    if (!grpV && has1) {
      store_half((jt + 1) & 1);
      if (has2) load_half(jt + 2);
    }
    __syncthreads();  // tile jt+1 is complete in LDS; buffer jt&1 may be overwritten next
  }

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
static hipError_t launch_fwd_t(const FwdArgs& a, const void* const Kp[3], const void* const Vp[3],
                               hipStream_t st) {
  constexpr int BR = FW_NW * 32;
  const int n_qtiles = (a.Tq + BR - 1) / BR;
  const long nblocks = (long)n_qtiles * ((a.BH + 7) / 8) * 8;
  // at most 4 workgroups per compute unit (256 CUs): the causal tail dominates, interleave heads
  const int interleave = nblocks <= 4 * 256 ? 1 : 0;
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
                     a.scale * kLog2e, a.scale, n_qtiles, a.BH, interleave);
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
