// Backward of route-fused attention, bf16 MFMA path.  The paper prints no backward; this is
// the chain rule through Alg. 2 steps 5-9 (router -> route-fusion -> causal softmax attention):
//   D[t]     = dO[t].O[t]
//   P[t,j]   = exp(tau Q[t].Kf[j] - LSE[t])            (recomputed, never stored)
//   dVf[j]   = sum_t P[t,j] dO[t]          dP[t,j] = dO[t].Vf[j]
//   dS[t,j]  = P[t,j] (dP[t,j] - D[t])
//   dKf[j]   = tau sum_t dS[t,j] Q[t]      dQ[t]   = tau sum_j dS[t,j] Kf[j]
//   dK_l[j]  = G[j,l] dKf[j]               dV_l[j] = G[j,l] dVf[j]          (un-fusion)
//   dlam[j,l]= dKf[j].K_l[j] + dVf[j].V_l[j]
//   dg[j,l]  = G[j,l] (dlam[j,l] - sum_m G[j,m] dlam[j,m])                   (softmax Jacobian)
//   dQ[t]   += sum_l dg[j(t),l] W_r[:,l]   dW_r = sum Q[t]^T dg   db_r = sum dg   (new slots only)
//
// Launch sequence:
//   prep    D = rowsum(dO*O)
//   main    one workgroup owns 128 KV slots (four blocks of 32): fuses its Kf/Vf ONCE (and
//           writes them to the workspace for the dQ kernel), keeps them as MFMA B operands in
//           registers, then walks over the 32-row query tiles that can see it, three tiles in
//           flight and one barrier per tile.  Two waves per slot block: the "V" wave computes
//           S = Q Kf^T -> P -> dVf^T += dO^T P for tile i and hands P^T over through LDS; the
//           "K" wave, one tile behind, computes dP = dO Vf^T, dS = P (dP - D),
//           dKf^T += Q^T dS.  Q / dO tiles are kept row-major only: the operands that contract
//           over query rows (dO^T, Q^T) are read with transposing LDS loads.
//           Epilogue: un-fusion, dlam, dg through LDS, coalesced accesses.
//   dq      (its own file) query-stationary: S, dP a second time, sum_j dS Kf in registers,
//           dQ = tau*acc + dg W_r^T -> bf16.  Adding dQ from the main kernel instead needs one f32 atomic per (KV
//           tile, row, head dim); they retire at about one element per clock and compute unit
//           and took four fifths of that kernel's time.
//   wpart   per-workgroup partial sums of Q^T dg and dg       (only with a router)
//   reduce  fixed-order sum of the partials -> dW_r, db_r     (deterministic)
#include "attn_tile.h"
#include "fuse_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int BCB = 128;  // slots per workgroup of the main kernel
constexpr int FIN_ROWS = 256;  // rows per workgroup of the finish kernel

__device__ __forceinline__ int swap23(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

// ------------------------------------------------------------------ prep
// Per query row: D = dO.O and LSE in log2 units, in arrays padded to whole 32-row tiles per
// (batch, head) (padding: D = 0, LSE = +inf, hence P = 0), so that the other kernels can fetch a
// tile's rows without tests.
constexpr int PREP_U = 4;  // items per thread
template <int D>
__global__ __launch_bounds__(256) void bwd_prep_kernel(const bf16* __restrict__ dO,
                                                       const bf16* __restrict__ O,
                                                       const float* __restrict__ LSE,
                                                       float* __restrict__ Dp,
                                                       float* __restrict__ LSE2p, int Tq, int Tqp,
                                                       long prows) {
  constexpr int CPR = D / 8;
  // PREP_U items (row, 16-byte chunk) per thread, 256 items apart, all loads issued first
  uint4 ra[PREP_U], rb[PREP_U];
  long prow_[PREP_U], row_[PREP_U];
  bool real_[PREP_U];
#pragma unroll
  for (int u = 0; u < PREP_U; ++u) {
    const long item = ((long)blockIdx.x * PREP_U + u) * 256 + threadIdx.x;
    const long prow = item / CPR;  // padded row index
    const int cc = (int)(item % CPR);
    const long bh = prow / Tqp;
    const int t = (int)(prow % Tqp);
    real_[u] = prow < prows && t < Tq;
    prow_[u] = prow;
    row_[u] = bh * Tq + t;
    ra[u] = rb[u] = make_uint4(0, 0, 0, 0);
    if (real_[u]) {
      ra[u] = load16_stream(dO + row_[u] * D + cc * 8);
      rb[u] = load16_stream(O + row_[u] * D + cc * 8);
    }
  }
#pragma unroll
  for (int u = 0; u < PREP_U; ++u) {
    float a[8], b[8];
    unpack8(ra[u], a);
    unpack8(rb[u], b);
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) part = fmaf(a[e], b[e], part);
    part = group_sum<CPR>(part);  // CPR consecutive lanes hold one row
    if (prow_[u] < prows && threadIdx.x % CPR == 0) {
      Dp[prow_[u]] = real_[u] ? part : 0.f;
      LSE2p[prow_[u]] = real_[u] ? LSE[row_[u]] * kLog2e : INFINITY;
    }
  }
}

// ------------------------------------------------------------------ main
template <int D>
struct BwdSmem {
  static constexpr int BR = 32;          // query rows per tile
  static constexpr int RSTR = D + 8;     // set-up only: padded row-major Kf / Vf rows
  // One slot of the query-tile ring: Q tile, dO tile (32 rows of D bf16 each, no padding, chunks
  // swizzled as in the K / V tiles of the attention kernels) and the rows' LSE and D values.
  // A tile is requested three iterations before its first use and read in two: five slots.
  static constexpr int NSLOT = 5;
  static constexpr int QB = BR * D * 2;          // bytes of one Q or dO tile
  static constexpr int SLOTB = 2 * QB + 256;     // Q, dO, 32 LSE, 32 D
  static constexpr int SBUF = BCB * BR;          // P^T tile: [slot][row], 64-byte rows, chunks rotated (bf16)
  static constexpr int OFF_P = NSLOT * SLOTB;    // bytes; two P^T tiles
  static constexpr int LOOP_END = OFF_P + 2 * SBUF * 2;
  // set-up only: row-major Kf and Vf of the workgroup's 128 slots, behind the first three ring
  // slots (whose tiles are requested before the set-up and land while it runs)
  static constexpr int OFF_KROW = 3 * SLOTB / 2;  // bf16 elements
  static constexpr int OFF_VROW = OFF_KROW + BCB * RSTR;
  static constexpr int SETUP_END = 3 * SLOTB + 2 * BCB * RSTR * 2;  // bytes
  static constexpr int TOTAL = LOOP_END > SETUP_END ? LOOP_END : SETUP_END;  // bytes
};

// LDS row of query row t (0..31) of a Q / dO tile (the slot permutation of the K / V tiles of the
// attention kernels).  The tiles are read two ways: as MFMA A operands by rows (16 lanes read 16
// rows x 16 bytes) and, for the products that contract over query rows, TRANSPOSED with
// ds_read_b64_tr_b16 (32 lanes read 4 consecutive query rows x 64 bytes); t = 4a + b -> row
// 4b + a (inside each group of 16) together with the chunk swizzle keeps both conflict-free.
__device__ __forceinline__ int tile_row(int t) {
  return (t & 16) | ((t & 3) << 2) | ((t >> 2) & 3);
}

// One key tile (128 slots, index jt) of head bh: set-up, loop over the query tiles that see it,
// epilogue.  Called by all 512 threads of the workgroup.
template <int D>
__device__ __forceinline__ void bwd_main_tile(
    const bf16* __restrict__ dO, const bf16* __restrict__ Q, const bf16* __restrict__ K0,
    const bf16* __restrict__ K1, const bf16* __restrict__ K2, const bf16* __restrict__ V0,
    const bf16* __restrict__ V1, const bf16* __restrict__ V2, const float* __restrict__ G,
    const float* __restrict__ LSE2p, const float* __restrict__ Dp, int Tqp, bf16* __restrict__ dK0,
    bf16* __restrict__ dK1, bf16* __restrict__ dK2, bf16* __restrict__ dV0, bf16* __restrict__ dV1,
    bf16* __restrict__ dV2, bf16* __restrict__ Kf_out, bf16* __restrict__ Vf_out,
    unsigned char* __restrict__ dS_out, int n_kvt, float* __restrict__ dgate, int Tq, int S,
    int len0, int len1, int len2, int causal, float c, float tau, int jt, long bh) {
  using L = BwdSmem<D>;
  constexpr int BR = L::BR, RSTR = L::RSTR;
  constexpr int CPR = D / 8, KK = D / 16, DB = D / 32, NT = 512;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);
  char* lds = reinterpret_cast<char*>(smem_raw);

  // 8 waves = 2 per SIMD.  Waves 0-3 (role V) and 4-7 (role K) each own the same four blocks
  // of 32 slots: role V computes S -> P -> dVf^T, role K (one tile behind, P^T through LDS)
  // dP -> dS -> dKf^T.  A wave so holds one
  // accumulator set and one B operand instead of two, which is what lets two waves share a SIMD
  // and hide each other's LDS / MFMA latency.
  // (opaque: the lane constants derived from it are recomputed per call instead of being kept
  // alive across the two tiles of a workgroup)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
  const bool roleK = wave >= 4;
  const int sw = wave & 3;  // slot block of this wave
  const int J0 = jt * BCB;
  const int off = S - Tq;
  const long kvbase = bh * (long)S * D;
  const long qbase = bh * (long)Tq * D;
  const float* Gb = G + bh * (long)S * 3;
  const int jmine = J0 + 32 * sw + li;  // the slot this lane owns in S / dP / dVf^T / dKf^T

  // first query tile that can see slot J0 (rows t with t + off >= J0)
  int t_first = 0;
  if (causal && J0 - off > 0) t_first = J0 - off;
  const int n_qt = (Tq + BR - 1) / BR;
  const int qt0 = t_first / BR;

  // ---- staging: query tiles go from global memory straight into LDS (no registers hold data in
  // flight), requested three iterations before their first use; every requesting wave issues an
  // equal share of a tile's load instructions (1 KiB each: lane i fills LDS row RPI q + i / CPR, chunk
  // position i % CPR of instruction q, and picks the query row and chunk that belong there),
  // wave 0 one more for the rows' LSE and D values.
  constexpr int ROWB = D * 2, RPI = 64 / CPR;
  constexpr int IPT = L::QB / 1024;  // load instructions per tensor and tile
  // The role-V waves (the first four) issue all of them: the role-K waves then have no loads
  // of their own to wait for, and when they store dS their stores are all that counts on their
  // vmcnt (measured against requests spread over all eight waves: main kernel -1 %).
  constexpr int RQW = 4;             // waves that issue the tile requests
  constexpr int LPW = 2 * IPT / RQW; // per requesting wave
  const int n_tiles = n_qt - qt0;
  const int uw = __builtin_amdgcn_readfirstlane(wave);
  const char* Qb = reinterpret_cast<const char*>(Q + qbase);
  const char* dOb = reinterpret_cast<const char*>(dO + qbase);
  unsigned st_row[LPW], st_chunk[LPW];
#pragma unroll
  for (int e = 0; e < LPW; ++e) {
    const int q = (RQW * e + (uw % RQW)) % IPT;
    const int r = RPI * q + lane / CPR;
    st_row[e] = (unsigned)tile_row(r);
    st_chunk[e] = 16u * (unsigned)((lane % CPR) ^ mx_swz<D>(r));
  }
  const float* ld_src = (lane < 32 ? LSE2p : Dp) + bh * (long)Tqp + (lane & 31);
  const unsigned lds_base = (unsigned)(size_t)lds;
  // tile k of this workgroup (past the last one: the last again, so that the counted waits stay
  // exact) into ring slot `slot`; rows past the end repeat the last row (their LSE is +inf)
  auto request = [&](int k, int slot) __attribute__((always_inline)) {
    const int t0 = (qt0 + (k < n_tiles ? k : n_tiles - 1)) * BR;
    const unsigned sb = lds_base + (unsigned)(slot * L::SLOTB);
    if (uw < RQW)
#pragma unroll
    for (int e = 0; e < LPW; ++e) {
      const int idx = RQW * e + uw, tensor = idx / IPT, q = idx % IPT;
      const unsigned o = min((unsigned)t0 + st_row[e], (unsigned)(Tq - 1)) * (unsigned)ROWB + st_chunk[e];
      mx_dma16(tensor ? dOb : Qb, o, sb + (unsigned)(tensor * L::QB + 1024 * q));
    }
    if (uw == 0) mx_dma4(ld_src + t0, sb + 2 * L::QB);
  };
  // before a barrier that publishes a tile: all but the two youngest tiles of this wave landed
  // (the counts are exact because a requesting wave issues nothing else that counts on vmcnt
  // inside the loop)
  auto wait_tile = [&]() __attribute__((always_inline)) {
    if (uw == 0) mx_wait_loads<2 * (LPW + 1)>();
    else if (uw < RQW) mx_wait_loads<2 * LPW>();
  };

  // the first three query tiles fly while the set-up runs
  request(0, 0);
  request(1, 1);
  request(2, 2);

  // ---- set-up: fuse the 128 slots once.  Item = (4 consecutive slots, 16-byte chunk).
  // [B*H,S,d] of the workspace has the layout of the K / V tensors: element offsets are shared.
  {
    bf16* sKrow = smem + L::OFF_KROW;
    bf16* sVrow = smem + L::OFF_VROW;
    const bf16* Ksrc[3] = {K0, K1, K2};
    const bf16* Vsrc[3] = {V0, V1, V2};
    const int lens[3] = {len0, len1, len2};
    for (int it = tid; it < (BCB / 4) * CPR; it += NT) {
      const int sg = it / CPR, cc = it % CPR;
      // all 24 raw chunks and the gates of the item first (one round trip to memory instead of
      // four): unconditional loads, an absent entry reads row 0 of the (b,h) block and is
      // replaced by zeros afterwards
      uint4 rk[4][3], rv[4][3];
      float gg[4][3];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = J0 + sg * 4 + u;
        const int jc = j < S ? j : S - 1;
#pragma unroll
        for (int l = 0; l < 3; ++l) {
          const bool present = j < S && j < lens[l];
          const long o = kvbase + (present ? (long)j * D : 0) + cc * 8;
          rk[u][l] = *reinterpret_cast<const uint4*>(Ksrc[l] + o);
          rv[u][l] = *reinterpret_cast<const uint4*>(Vsrc[l] + o);
          gg[u][l] = Gb[jc * 3 + l];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = J0 + sg * 4 + u;
        const bool in = j < S;
        const uint4 z = make_uint4(0, 0, 0, 0);
        Raw3 k3, v3;
        k3.a = (in && j < len0) ? rk[u][0] : z;  v3.a = (in && j < len0) ? rv[u][0] : z;
        k3.b = (in && j < len1) ? rk[u][1] : z;  v3.b = (in && j < len1) ? rv[u][1] : z;
        k3.c = (in && j < len2) ? rk[u][2] : z;  v3.c = (in && j < len2) ? rv[u][2] : z;
        float kf[8], vf[8];
        fuse8(k3, gg[u][0], gg[u][1], gg[u][2], kf);
        fuse8(v3, gg[u][0], gg[u][1], gg[u][2], vf);
        const uint4 pk = pack8(kf), pv = pack8(vf);
        *reinterpret_cast<uint4*>(&sKrow[(sg * 4 + u) * RSTR + cc * 8]) = pk;
        *reinterpret_cast<uint4*>(&sVrow[(sg * 4 + u) * RSTR + cc * 8]) = pv;
        if (in) {  // the fused stream, for the dQ kernel (Vf only if it recomputes dP)
          const long eoff = kvbase + (long)j * D + cc * 8;
          *reinterpret_cast<uint4*>(Kf_out + eoff) = pk;
          if (Vf_out) *reinterpret_cast<uint4*>(Vf_out + eoff) = pv;
        }
      }
    }
  }
  __syncthreads();
  // B operand held in registers for the whole kernel: Kf rows (role V, for S) or Vf rows (role
  // K, for dP) of the wave's 32 slots
  bf16x8 breg[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    breg[kk] = *reinterpret_cast<const bf16x8*>(smem + (roleK ? L::OFF_VROW : L::OFF_KROW) + (32 * sw + li) * RSTR + 16 * kk + 8 * g);
  // one accumulator set per wave: dVf^T (role V) or dKf^T (role K)
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  // lane constants of the LDS reads: A operand rows (slot li of a 32-row tile, head dims 8 g ..)
  // and transposed reads (k-step of 16 query rows, 32 head dims)
  const unsigned aq0 = mx_kfrag0<D>(swap23(li), g);
  unsigned xq_lo, xq_hi;
  {
    const int i = lane & 15, gsel = (lane >> 4) & 1, khalf = lane >> 5;
    const int cl = 2 * gsel + ((i & 3) >> 1), sub = 8 * (i & 1);
    const int r_lo = tile_row(8 * khalf + (i >> 2)), r_hi = tile_row(8 * khalf + (i >> 2) + 4);
    xq_lo = (unsigned)(r_lo * ROWB + 16 * (cl ^ mx_swz<D>(r_lo)) + sub);
    xq_hi = (unsigned)(r_hi * ROWB + 16 * (cl ^ mx_swz<D>(r_hi)) + sub);
  }
  // A operand (32 head dims x 16 query rows) = transpose of query rows 16 half .. of a tile at
  // byte offset tb, head dims 32 db ..: db only meets the swizzle in an XOR of address bits 6..7
  auto tr_frag = [&](unsigned tb, int db, int half) __attribute__((always_inline)) {
    const char* base = lds + tb + 16 * half * ROWB;
    const uint2 lo = lds_read_tr(reinterpret_cast<const bf16*>(base + (xq_lo ^ (unsigned)(db << 6))));
    const uint2 hi = lds_read_tr(reinterpret_cast<const bf16*>(base + (xq_hi ^ (unsigned)(db << 6))));
    return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
  };

  // ---- main loop, ONE barrier per iteration.  In iteration `it`
  //   all:    request tile it+3
  //   role K: for tile it-1: dP = dO Vf^T, dS = P (dP - D) with P^T read back from LDS,
  //           dKf^T += Q^T dS
  //   role V: for tile it: S = Q Kf^T, P = exp2(c S - LSE), publishes P^T, dVf^T += dO^T P
  // so S is computed once, and every hand-over (P^T, requested tiles) crosses one barrier.
  wait_tile();
  __syncthreads();  // tile 0 is complete; the set-up buffers are dead (the B operands are in registers)

  // chunk-rotated address of the lane's 16 bytes (8 query rows 16 h + 8 g ..) in a P^T tile
  const int Rl = 32 * sw + li;
  auto pt_off = [&](int h) { return Rl * BR + 8 * ((2 * h + g + (Rl >> 1)) & 3); };
  bf16* sPbase = reinterpret_cast<bf16*>(lds + L::OFF_P);

  // role K leaves dS of every (key tile, query tile) pair in the workspace for the dQ kernel: its
  // two packed registers, 1 KiB per store instruction (block layout: see bwd_dqg_bf16.hip)
  // ordered [head][group of 8 query tiles][key tile][slot half][tile in group][4 KiB]: the dQ
  // kernel's workgroup (8 query tiles) then streams one contiguous 32 KiB run per 64 slots
  unsigned char* ds_lane = nullptr;
  const int n_qg = (n_qt + 7) / 8;
  if (dS_out) ds_lane = dS_out + (sw >> 1) * 32768 + (sw & 1) * 2048 + li * 32 + g * 16;

  int b5 = 0;  // it % NSLOT
  for (int it = 0; it < n_tiles + 1; ++it) {
    request(it + 3, b5 + 3 >= L::NSLOT ? b5 + 3 - L::NSLOT : b5 + 3);
    if (roleK) {
      if (it >= 1) {
        const int k = it - 1;
        const unsigned tb = (unsigned)((b5 == 0 ? L::NSLOT - 1 : b5 - 1) * L::SLOTB);  // slot of tile it-1
        const bf16* sP = sPbase + (k & 1) * L::SBUF;
        f32x16 pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) pacc[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 ao = lds_frag(lds + tb + L::QB + (aq0 ^ (unsigned)(kk << 5)));
          pacc = mfma32(ao, breg[kk], pacc);
        }
        // register r <-> row 16 (r/8) + 8 g + r%8 of the tile, column = the lane's slot
        const float* sDv = reinterpret_cast<const float*>(lds + tb + 2 * L::QB + 128);
        float v[16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int tl = 16 * h + 8 * g;
          const float4 d0 = *reinterpret_cast<const float4*>(&sDv[tl]);
          const float4 d1 = *reinterpret_cast<const float4*>(&sDv[tl + 4]);
          const float dv[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
          float pf[8];
          unpack8(*reinterpret_cast<const uint4*>(&sP[pt_off(h)]), pf);
#pragma unroll
          for (int u = 0; u < 8; ++u) v[8 * h + u] = pf[u] * (pacc[8 * h + u] - dv[u]);  // dS
        }
        const uint4 s0 = pack8(&v[0]), s1 = pack8(&v[8]);
        const bf16x8 sB0 = __builtin_bit_cast(bf16x8, s0), sB1 = __builtin_bit_cast(bf16x8, s1);
        // dKf^T += Q^T dS (k-step = 16 query rows; A read transposed out of the row-major tile;
        // accumulator row m of block db = head dim 32 db + m)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a0 = tr_frag(tb, db, 0);
          const bf16x8 a1 = tr_frag(tb, db, 1);
          acc[db] = mfma32(a0, sB0, acc[db]);
          acc[db] = mfma32(a1, sB1, acc[db]);
        }
        if (ds_lane) {  // behind the MFMAs: the stores then do not delay their issue
          __builtin_amdgcn_sched_barrier(0);
          const int qtile = qt0 + k;
          const size_t blk = (((size_t)bh * n_qg + (qtile >> 3)) * n_kvt + jt) * 65536 + (size_t)(qtile & 7) * 4096;
          // streamed past the caches: 2 B per pair is far more than the L2 holds, and the query
          // tiles that the other key tiles of the head re-read should stay there
          store16_stream(ds_lane + blk, s0);
          store16_stream(ds_lane + blk + 1024, s1);
        }
      }
    } else {
      if (it < n_tiles) {
        const int t0 = (qt0 + it) * BR;
        const unsigned tb = (unsigned)(b5 * L::SLOTB);
        bf16* sP = sPbase + (it & 1) * L::SBUF;
        const bool need_mask = (J0 + BCB > S) || (causal && (J0 + BCB - 1 > t0 + off));
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 aq = lds_frag(lds + tb + (aq0 ^ (unsigned)(kk << 5)));
          sacc = mfma32(aq, breg[kk], sacc);
        }
        const float* sL = reinterpret_cast<const float*>(lds + tb + 2 * L::QB);
        float v[16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int tl = 16 * h + 8 * g;
          const float4 l0 = *reinterpret_cast<const float4*>(&sL[tl]);
          const float4 l1 = *reinterpret_cast<const float4*>(&sL[tl + 4]);
          const float lv[8] = {l0.x, l0.y, l0.z, l0.w, l1.x, l1.y, l1.z, l1.w};
#pragma unroll
          for (int u = 0; u < 8; ++u) v[8 * h + u] = fast_exp2(fmaf(sacc[8 * h + u], c, -lv[u]));
        }
        if (need_mask) {  // diagonal and tail tiles only (uniform branch, outside the hot path)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int t = t0 + 16 * (r >> 3) + 8 * g + (r & 7);
            const bool vis = (jmine < S) && (!causal || jmine <= t + off);
            v[r] = vis ? v[r] : 0.f;
          }
        }
        const uint4 p0 = pack8(&v[0]), p1 = pack8(&v[8]);
        *reinterpret_cast<uint4*>(&sP[pt_off(0)]) = p0;
        *reinterpret_cast<uint4*>(&sP[pt_off(1)]) = p1;
        const bf16x8 pB0 = __builtin_bit_cast(bf16x8, p0), pB1 = __builtin_bit_cast(bf16x8, p1);
        // dVf^T += dO^T P
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a0 = tr_frag(tb + L::QB, db, 0);
          const bf16x8 a1 = tr_frag(tb + L::QB, db, 1);
          acc[db] = mfma32(a0, pB0, acc[db]);
          acc[db] = mfma32(a1, pB1, acc[db]);
        }
      }
    }
    wait_tile();  // this wave's part of tile it+1 has landed (role K: nothing to wait for; its
                  // dS stores count on vmcnt too, and must not be waited for here)
    loop_barrier();
    b5 = b5 == L::NSLOT - 1 ? 0 : b5 + 1;
  }
  mx_wait_loads<0>();  // the surplus requests must land before the epilogue reuses the buffers
  __syncthreads();

  // ---- epilogue.  dKf^T (held by role K) then dVf^T (role V) go through LDS as f32 [slot][d] so
  // that the un-fusion (dK_l = G_l tau dKf, dV_l = G_l dVf) is written with coalesced 16-byte
  // stores and the gate gradients dlam_l = dKf.K_l + dVf.V_l are formed from coalesced 16-byte
  // loads.  Item = (slot, 16-byte chunk): CPR consecutive lanes hold one slot's row.
  constexpr int ESTR = D + 4;                 // f32 per staged row
  constexpr int NITEM = BCB * CPR / NT;       // items per thread
  static_assert((size_t)BCB * ESTR * 4 <= (size_t)L::TOTAL, "staging tile must fit");
  float* sE = reinterpret_cast<float*>(smem_raw);
  const int ecc = tid % CPR, erow0 = tid / CPR;
  constexpr int ERS = NT / CPR;               // slots covered per pass
  float dlam[NITEM][3];
#pragma unroll
  for (int i = 0; i < NITEM; ++i) dlam[i][0] = dlam[i][1] = dlam[i][2] = 0.f;
  const bf16* Kp[3] = {K0, K1, K2};
  const bf16* Vp[3] = {V0, V1, V2};
  bf16* dKp[3] = {dK0, dK1, dK2};
  bf16* dVp[3] = {dV0, dV1, dV2};
  const int len[3] = {len0, len1, len2};
  // all raw K_l / V_l chunks and gates of the thread's items, for both passes, are requested now
  // (unconditional loads: an absent entry reads row 0 of the (b,h) block and is not used): one
  // round trip to memory for the whole epilogue, overlapped with the staging of the accumulators
  uint4 rawK[NITEM][3], rawV[NITEM][3];
  float gl[NITEM][3];
#pragma unroll
  for (int i = 0; i < NITEM; ++i) {
    const int j = J0 + erow0 + ERS * i;
    const int jc = j < S ? j : S - 1;
#pragma unroll
    for (int l = 0; l < 3; ++l) {
      const bool present = j < S && j < len[l];
      const long o = kvbase + (present ? (long)j * D : 0) + ecc * 8;
      rawK[i][l] = *reinterpret_cast<const uint4*>(Kp[l] + o);
      rawV[i][l] = *reinterpret_cast<const uint4*>(Vp[l] + o);
      gl[i][l] = Gb[jc * 3 + l];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    __syncthreads();  // LDS free (main loop done / previous pass consumed)
    if (roleK == (pass == 0)) {
      const float f = pass == 0 ? tau : 1.f;  // dKf carries the factor tau
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int d = 32 * db + 8 * (r >> 2) + 4 * g + (r & 3);
          sE[(32 * sw + li) * ESTR + d] = acc[db][r] * f;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NITEM; ++i) {
      const int sl = erow0 + ERS * i;
      const int j = J0 + sl;
      if (j < S) {
        const float4 a0 = *reinterpret_cast<const float4*>(&sE[sl * ESTR + ecc * 8]);
        const float4 a1 = *reinterpret_cast<const float4*>(&sE[sl * ESTR + ecc * 8 + 4]);
        const float v[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        const long o = kvbase + (long)j * D + ecc * 8;
#pragma unroll
        for (int l = 0; l < 3; ++l) {
          const bool present = j < len[l];
          const float g_l = present ? gl[i][l] : 0.f;
          bf16* dst = pass == 0 ? dKp[l] : dVp[l];
          if (dst) {
            float o8[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o8[e] = g_l * v[e];
            *reinterpret_cast<uint4*>(dst + o) = pack8(o8);
          }
          if (present) {
            float x[8];
            unpack8(pass == 0 ? rawK[i][l] : rawV[i][l], x);
            float a = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) a = fmaf(v[e], x[e], a);
            dlam[i][l] += a;
          }
        }
      }
    }
  }
  if (dgate) {
#pragma unroll
    for (int i = 0; i < NITEM; ++i) {
      const float d0 = group_sum<CPR>(dlam[i][0]);
      const float d1 = group_sum<CPR>(dlam[i][1]);
      const float d2 = group_sum<CPR>(dlam[i][2]);
      const int j = J0 + erow0 + ERS * i;
      const int t = j - off;
      if (j < S && t >= 0 && ecc == 0) {
        const float g0 = Gb[j * 3 + 0], g1 = Gb[j * 3 + 1], g2 = Gb[j * 3 + 2];
        const float mean = g0 * d0 + g1 * d1 + g2 * d2;
        float* out = dgate + (bh * (long)Tq + t) * 3;
        out[0] = g0 * (d0 - mean);
        out[1] = g1 * (d1 - mean);
        out[2] = g2 * (d2 - mean);
      }
    }
  }
}

template <int D>
__global__ __launch_bounds__(512, 1) void bwd_main_kernel(
    const bf16* __restrict__ dO, const bf16* __restrict__ Q, const bf16* __restrict__ K0,
    const bf16* __restrict__ K1, const bf16* __restrict__ K2, const bf16* __restrict__ V0,
    const bf16* __restrict__ V1, const bf16* __restrict__ V2, const float* __restrict__ G,
    const float* __restrict__ LSE2p, const float* __restrict__ Dp, int Tqp, bf16* __restrict__ dK0,
    bf16* __restrict__ dK1, bf16* __restrict__ dK2, bf16* __restrict__ dV0, bf16* __restrict__ dV1,
    bf16* __restrict__ dV2, bf16* __restrict__ Kf_out, bf16* __restrict__ Vf_out,
    unsigned char* __restrict__ dS_out, float* __restrict__ dgate, int Tq, int S,
    int len0, int len1, int len2, int causal, float c, float tau, int n_kvtiles, int BH,
    int pair) {
  // All KV tiles of one (batch, head) run on ONE XCD (block index = 8 * slot + xcd): they share
  // the head's Q / dO tiles in that XCD's L2.  Tile 0 sees every query row, so ascending tile
  // order is heaviest first.
  // pair: a workgroup takes tile jt and then its mirror tile n_kvtiles-1-jt.  Under a causal mask
  // the two see the same number of query tiles in total, so all workgroups weigh the same and
  // the compute units finish together; and there are half as many workgroups to start.
  const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
  const int n_first = pair ? (n_kvtiles + 1) / 2 : n_kvtiles;
  const int jt0 = slot % n_first, jt1 = n_kvtiles - 1 - jt0;
  const long bh = (long)(slot / n_first) * 8 + xcd;
  if (bh >= BH) return;
  bwd_main_tile<D>(dO, Q, K0, K1, K2, V0, V1, V2, G, LSE2p, Dp, Tqp, dK0, dK1, dK2, dV0, dV1, dV2,
                   Kf_out, Vf_out, dS_out, n_kvtiles, dgate, Tq, S, len0, len1, len2, causal, c, tau,
                   jt0, bh);
  if (pair && jt1 != jt0) {
    __syncthreads();  // the first tile's epilogue staging is dead
    bwd_main_tile<D>(dO, Q, K0, K1, K2, V0, V1, V2, G, LSE2p, Dp, Tqp, dK0, dK1, dK2, dV0, dV1, dV2,
                     Kf_out, Vf_out, dS_out, n_kvtiles, dgate, Tq, S, len0, len1, len2, causal, c,
                     tau, jt1, bh);
  }
}

// ------------------------------------------------------------------ router-gradient partials
// Per-workgroup partial sums of Q^T dg and dg in a fixed order.
template <int D>
__global__ __launch_bounds__(256) void bwd_wpart_kernel(const float* __restrict__ dgate,
                                                        const bf16* __restrict__ Q,
                                                        float* __restrict__ dWpart, long rows) {
  constexpr int CPR = D / 8, RL = 256 / CPR;  // row lanes per workgroup
  __shared__ float sPart[RL][D * 3 + 3];
  const int tid = threadIdx.x, cc = tid % CPR, rl = tid / CPR;
  float wacc[8][3];
  float bacc[3] = {0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < 8; ++e) wacc[e][0] = wacc[e][1] = wacc[e][2] = 0.f;
  const long row0 = (long)blockIdx.x * FIN_ROWS;
  // (rows past the end read the last row with zero weights: no early exit, so that the loads
  // of four iterations are in flight at once)
#pragma unroll 4
  for (int i = rl; i < FIN_ROWS; i += RL) {
    const bool in = row0 + i < rows;
    const long row = in ? row0 + i : rows - 1;
    const float dg0 = in ? dgate[row * 3 + 0] : 0.f, dg1 = in ? dgate[row * 3 + 1] : 0.f,
                dg2 = in ? dgate[row * 3 + 2] : 0.f;
    float q[8];
    unpack8(load16_stream(Q + row * D + cc * 8), q);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      wacc[e][0] = fmaf(q[e], dg0, wacc[e][0]);
      wacc[e][1] = fmaf(q[e], dg1, wacc[e][1]);
      wacc[e][2] = fmaf(q[e], dg2, wacc[e][2]);
    }
    if (cc == 0) { bacc[0] += dg0; bacc[1] += dg1; bacc[2] += dg2; }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int l = 0; l < 3; ++l) sPart[rl][(cc * 8 + e) * 3 + l] = wacc[e][l];
  if (cc == 0)
#pragma unroll
    for (int l = 0; l < 3; ++l) sPart[rl][D * 3 + l] = bacc[l];
  __syncthreads();
  for (int i = tid; i < D * 3 + 3; i += 256) {
    float s = 0.f;
    for (int r = 0; r < RL; ++r) s += sPart[r][i];  // fixed order
    dWpart[(long)blockIdx.x * (D * 3 + 3) + i] = s;
  }
}

// Fixed-order sum of the per-workgroup partials (two levels so that the chain stays short).
__global__ __launch_bounds__(256) void bwd_reduce_kernel(const float* __restrict__ dWpart,
                                                         int nparts, int width,
                                                         float* __restrict__ dW_r,
                                                         float* __restrict__ db_r) {
  __shared__ float sred[256];
  const int i = blockIdx.x;  // one output element per workgroup
  float s = 0.f;
  for (int p = threadIdx.x; p < nparts; p += 256) s += dWpart[(long)p * width + i];
  sred[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int k = 0; k < 256; ++k) t += sred[k];
    if (i < width - 3) {
      if (dW_r) dW_r[i] = t;
    } else if (db_r) {
      db_r[i - (width - 3)] = t;
    }
  }
}

size_t a256(size_t n) { return (n + 255) & ~(size_t)255; }

// Stored score gradients (the dQ kernel then needs one product per pair instead of three): one
// 8 KiB block per (128-slot key tile, 32-row query tile) of every head, the full rectangle (under
// a causal mask about half of it is written and read).  Provided when it stays below this many
// bytes in total and below 4 GiB per head (32-bit block offsets); C5 needs 4 GiB.
constexpr size_t kDsCapBytes = (size_t)32 << 30;
size_t ds_bytes(int BH, int Tq, int S) {
  // query tiles padded to whole groups of 8 (one workgroup of the dQ kernel)
  const size_t per_head = (size_t)((S + BCB - 1) / BCB) * (size_t)((Tq + 255) / 256) * 8 * 8192;
  if (per_head >= ((size_t)1 << 32)) return 0;
  const size_t all = per_head * (size_t)BH;
  return all <= kDsCapBytes ? all : 0;
}

struct BwdWs {
  size_t off_d, off_lse, off_dg, off_part, off_kf, off_vf, off_ds, total;
  int nparts, Tqp;
};
// with_ds: Kf, then the dS blocks (no Vf: the dQ kernel does not recompute dP); else Kf and Vf
BwdWs carve(int BH, int Tq, int S, int d, bool with_ds) {
  BwdWs w;
  const size_t rows = (size_t)BH * Tq;
  w.nparts = (int)((rows + FIN_ROWS - 1) / FIN_ROWS);
  w.Tqp = (Tq + 31) / 32 * 32;  // D and LSE rows are padded to whole 32-row tiles per (b,h)
  const size_t prows = (size_t)BH * w.Tqp;
  w.off_d = 0;
  w.off_lse = w.off_d + a256(prows * sizeof(float));
  w.off_dg = w.off_lse + a256(prows * sizeof(float));
  w.off_part = w.off_dg + a256(rows * 3 * sizeof(float));
  w.off_kf = w.off_part + a256((size_t)w.nparts * (d * 3 + 3) * sizeof(float));
  w.off_vf = w.off_kf + a256((size_t)BH * S * d * sizeof(bf16));
  w.off_ds = w.off_vf;
  const size_t vf_end = w.off_vf + a256((size_t)BH * S * d * sizeof(bf16));
  const size_t ds_end = w.off_ds + a256(ds_bytes(BH, Tq, S));
  // the size for the stored gradients is always above the other route's, so that the size of
  // the caller's workspace tells which route is wanted
  w.total = with_ds ? (ds_end > vf_end + 256 ? ds_end : vf_end + 256) : vf_end;
  return w;
}

template <int D>
hipError_t launch_bwd_t(const BwdArgs& a, hipStream_t st) {
  using L = BwdSmem<D>;
  // the route with stored score gradients when the caller's workspace has the size asked for it
  const bool with_ds = ds_bytes(a.BH, a.Tq, a.S) > 0 &&
                       a.workspace_bytes >= carve(a.BH, a.Tq, a.S, D, true).total;
  const BwdWs w = carve(a.BH, a.Tq, a.S, D, with_ds);
  unsigned char* ws = static_cast<unsigned char*>(a.workspace);
  float* Dp = reinterpret_cast<float*>(ws + w.off_d);
  float* LSE2p = reinterpret_cast<float*>(ws + w.off_lse);
  float* dgate = a.W_r ? reinterpret_cast<float*>(ws + w.off_dg) : nullptr;
  float* dWpart = reinterpret_cast<float*>(ws + w.off_part);
  bf16* Kf = reinterpret_cast<bf16*>(ws + w.off_kf);
  bf16* Vf = with_ds ? nullptr : reinterpret_cast<bf16*>(ws + w.off_vf);
  unsigned char* dSb = with_ds ? ws + w.off_ds : nullptr;
  const long rows = (long)a.BH * a.Tq;
  constexpr int CPR = D / 8;

  const long prows = (long)a.BH * w.Tqp;
  hipLaunchKernelGGL((bwd_prep_kernel<D>), dim3((unsigned)((prows * CPR + 256 * PREP_U - 1) / (256 * PREP_U))), dim3(256),
                     0, st, (const bf16*)a.dO, (const bf16*)a.O, a.LSE, Dp, LSE2p, a.Tq, w.Tqp,
                     prows);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  // a level without memory borrows another level's buffer and has length 0 (never used)
  const void* Kp[3];
  const void* Vp[3];
  const void* anyK = a.K[0] ? a.K[0] : (a.K[1] ? a.K[1] : a.K[2]);
  const void* anyV = a.V[0] ? a.V[0] : (a.V[1] ? a.V[1] : a.V[2]);
  if (!anyK || !anyV) return hipErrorInvalidValue;
  for (int l = 0; l < 3; ++l) {
    Kp[l] = a.K[l] ? a.K[l] : anyK;
    Vp[l] = a.V[l] ? a.V[l] : anyV;
  }
  const int n_kvtiles = (a.S + BCB - 1) / BCB;
  const size_t smem = (size_t)L::TOTAL;
  static bool attr_set = false;
  if (!attr_set) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_main_kernel<D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // Work distribution (see the kernel): under a causal mask a workgroup takes a heavy key tile
  // and its light mirror tile (measured at B*H = 64, T = 2048: 6 % off the backward pass against
  // one tile per workgroup; persistent workgroups with a static share each were 10 % slower).
  const int hpx = (a.BH + 7) / 8;
  const int pair = (a.causal && n_kvtiles > 1) ? 1 : 0;
  const int n_first = pair ? (n_kvtiles + 1) / 2 : n_kvtiles;
  const unsigned nwg = (unsigned)((long)n_first * hpx * 8);
  hipLaunchKernelGGL((bwd_main_kernel<D>), dim3(nwg),
                     dim3(512), smem, st, (const bf16*)a.dO, (const bf16*)a.Q,
                     (const bf16*)Kp[0], (const bf16*)Kp[1], (const bf16*)Kp[2],
                     (const bf16*)Vp[0], (const bf16*)Vp[1], (const bf16*)Vp[2], a.G, LSE2p, Dp, w.Tqp,
                     (bf16*)a.dK[0], (bf16*)a.dK[1], (bf16*)a.dK[2], (bf16*)a.dV[0],
                     (bf16*)a.dV[1], (bf16*)a.dV[2], Kf, Vf, dSb, dgate, a.Tq, a.S, a.len[0], a.len[1],
                     a.len[2], a.causal, a.scale * kLog2e, a.scale, n_kvtiles, a.BH, pair);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  if (with_ds) {
    BwdDqgArgs q;
    q.Kf = Kf; q.dS = dSb; q.dgate = dgate; q.W_r = a.W_r; q.dQ = a.dQ;
    q.BH = a.BH; q.Tq = a.Tq; q.S = a.S; q.d = D; q.causal = a.causal; q.scale = a.scale;
    q.n_qt32 = (a.Tq + 31) / 32; q.n_kvt = n_kvtiles;
    e = launch_bwd_dqg_bf16(q, st);
  } else {
    BwdDqArgs q;
    q.Q = a.Q; q.dO = a.dO; q.Kf = Kf; q.Vf = Vf; q.LSE2p = LSE2p; q.Dp = Dp; q.Tqp = w.Tqp; q.dgate = dgate; q.W_r = a.W_r; q.dQ = a.dQ;
    q.BH = a.BH; q.Tq = a.Tq; q.S = a.S; q.d = D; q.causal = a.causal; q.scale = a.scale;
    e = launch_bwd_dq_bf16(q, st);
  }
  if (e != hipSuccess) return e;

  if (a.W_r && (a.dW_r || a.db_r)) {
    hipLaunchKernelGGL((bwd_wpart_kernel<D>), dim3(w.nparts), dim3(256), 0, st, dgate,
                       (const bf16*)a.Q, dWpart, rows);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_reduce_kernel, dim3(D * 3 + 3), dim3(256), 0, st, dWpart, w.nparts,
                       D * 3 + 3, a.dW_r, a.db_r);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace

size_t bwd_workspace_bytes(int BH, int Tq, int S, int d, bool with_ds) {
  if (with_ds && ds_bytes(BH, Tq, S) == 0) return 0;
  return carve(BH, Tq, S, d, with_ds).total;
}

hipError_t launch_bwd_bf16(const BwdArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  return a.d == 128 ? launch_bwd_t<128>(a, st) : launch_bwd_t<64>(a, st);
}

}  // namespace mka
