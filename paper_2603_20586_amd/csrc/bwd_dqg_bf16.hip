// dQ of the route-fused attention backward from STORED score gradients, bf16 MFMA path - the
// route taken when the workspace has room for them; the kernel that recomputes them
// (bwd_dq_bf16.hip) serves the minimal workspace.  The paper prints
// no backward; this is the query-side contraction of the chain rule through Alg. 2 step 9:
//
//   dQ[t] = tau sum_j dS[t,j] Kf[j] + sum_l dg[t,l] W_r[:,l]
//
// with dS[t,j] = P[t,j] (dP[t,j] - D[t]) taken from the workspace, where the main backward kernel
// has left it in bf16, instead of being formed a second time: one MFMA product per pair here
// against three there, paid for with 2 bytes per pair written and read back (2.2 GB each way at
// T = 4096, B H = 128).
//
// A workgroup owns 256 query rows (8 waves x 32 rows, a wave = one 32-row query tile of the main
// kernel) and walks over the key stream in stages of 64 slots.  The stage's Kf rows (shared,
// row-major, the tile layout of attn_tile.h; mostly L2 hits) go from global memory straight into
// LDS, four stages ahead, one barrier per stage.  Every wave's own dS piece (4 KiB per stage) is
// loaded into registers four stages ahead - as assembly with counted waits, because the compiler's
// own wait counts do not see the LDS-direct loads and would drain the queue - and written to a
// private LDS buffer.  dQ^T += Kf^T dS^T with 32x32x16 MFMAs: both operands are read TRANSPOSED
// out of LDS (ds_read_b64_tr_b16) - Kf^T from the row-major key tile, dS^T from the layout below -
// and dQ^T stays in registers until the epilogue adds the router term and stores bf16 rows once.
// Every sum has a fixed order.
// Measured (T = 4096, B H = 128): 0.53 ms against 0.80 ms for the recomputing kernel; the dS stream
// arrives at 4.8 TB/s whatever the prefetch depth (4 or 6 stages) or the block order, the kernel
// takes the same time without its MFMAs and LDS reads (0.54 ms), 0.35 ms without the dS loads and
// 0.47 ms without the Kf loads.  The main kernel pays 0.12 ms for the stores (non-temporal, and
// counted in its role-K waves' vmcnt waits; with cached stores and uncounted waits it paid 0.18
// ms and this kernel 0.55), so that in a loop of back-to-back calls the backward as a whole
// takes 2.22 ms against 2.37 ms.
//
// dS layout: per (head, group of 8 query tiles, 128-slot key tile) 64 KiB = [slot half: 2][query
// tile in group: 8][4 KiB]; inside the 4 KiB (64 slots x 32 rows) [slot block: 2][row half h: 2]
// [slot li: 32][g: 2][8 rows], i.e. what the main kernel's role-K waves hold in their two packed
// registers, 1 KiB per store instruction.  A workgroup here reads one contiguous 32 KiB run per
// stage.
#include "attn_tile.h"
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

constexpr int DG_BC = 64;            // slots per stage
constexpr int DG_NW = 8;             // waves per workgroup
constexpr int DG_NT = DG_NW * 64;
constexpr int DG_BR = DG_NW * 32;    // query rows per workgroup
constexpr int DG_PIECE = 1024 + 128; // LDS stride of the 1 KiB pieces of a wave's dS: the two row
                                     // halves that one transposed read touches land 128 B apart
                                     // (mod 256), so the 32 lanes it serves at a time hit 32 banks
constexpr int DG_WST = 4 * DG_PIECE; // LDS bytes per wave and stage

constexpr int DG_PD = 4;             // stages of dS in flight per wave (16 registers each)

// 16 bytes per lane from global memory (uniform base + per-lane byte offset) into registers,
// issued as assembly so that the wait is the caller's: the compiler's own wait counts see neither
// this load nor the LDS-direct ones and would either miss it or drain the whole queue.  The
// destination must not be touched before a counted s_waitcnt vmcnt has covered the load.
__device__ __forceinline__ void dg_load16(u32x4& dst, const void* base, unsigned off) {
  asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(off), "s"(base) : "memory");
}

template <int D>
struct DgSmem {
  static constexpr int ROWB = D * 2;
  static constexpr int KT = DG_BC * ROWB;              // the stage's Kf rows
  static constexpr int NST = DG_PD + 1;                // depth of the ring of Kf tiles
  static constexpr int OFF_DS = NST * KT;              // per wave: one buffer of DG_WST bytes
  static constexpr int RING = OFF_DS + DG_NW * DG_WST;
  static constexpr int ESTR = D + 4;                   // f32 per row of the epilogue's staging tile
  static constexpr int EPI = DG_BR * ESTR * 4 + D * 3 * 4;
  static constexpr int TOTAL = RING > EPI ? RING : EPI;  // bytes
};

// One tile of 256 query rows (index qt) of head bh.  Called by all threads of the workgroup.
template <int D>
__device__ __forceinline__ void bwd_dqg_tile(const bf16* __restrict__ Kf,
                                             const unsigned char* __restrict__ dS,
                                             const float* __restrict__ dgate,
                                             const float* __restrict__ W_r, bf16* __restrict__ dQ,
                                             float tau, int Tq, int S, int causal, int n_qt32,
                                             int n_kvt, int qt, long bh) {
  using SM = DgSmem<D>;
  constexpr int ROWB = SM::ROWB, DB = D / 32, CPR = D / 8;
  extern __shared__ __attribute__((aligned(1024))) unsigned char dg_smem_raw[];
  char* smem = reinterpret_cast<char*>(dg_smem_raw);

  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63, g = lane >> 5, li = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qt32 = qt * DG_NW + wave;   // this wave's 32-row query tile
  const int tw0 = qt32 * 32;            // its first row
  const int off = S - Tq;
  const bool has_rows = qt32 < n_qt32;

  // stages this workgroup visits
  int t_last = qt * DG_BR + DG_BR - 1;
  if (t_last > Tq - 1) t_last = Tq - 1;
  int j_end = S;
  if (causal && t_last + off + 1 < S) j_end = t_last + off + 1;
  const int NS = (j_end + DG_BC - 1) / DG_BC;  // >= 1: S >= Tq >= 1

  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  // ---- staging.  Kf rows: one load instruction fills 1 KiB of the stage's key tile (RPI rows);
  // lane i of instruction q serves LDS row RPI q + i / CPR, chunk position i % CPR, and picks the
  // slot and the chunk that belong there.  dS: four 1 KiB pieces per wave, copied as they are.
  constexpr int RPI = 64 / CPR;
  constexpr int IPW = (DG_BC / RPI) / DG_NW;
  static_assert(IPW >= 1, "every wave issues at least one key-tile load per stage");
  unsigned kslot[IPW], kchunk[IPW];
#pragma unroll
  for (int e = 0; e < IPW; ++e) {
    const int r = RPI * (IPW * wave + e) + lane / CPR;
    kslot[e] = (unsigned)mx_row(r);
    kchunk[e] = 16u * (unsigned)((lane % CPR) ^ mx_swz<D>(r));
  }
  const char* kbase = reinterpret_cast<const char*>(Kf + bh * (long)S * D);
  // this head's dS blocks, ordered [group of 8 query tiles = this workgroup][key tile][wave]: the
  // workgroup streams 64 KiB per key tile.  Query tiles are padded to whole groups, so a wave
  // without rows reads blocks that nobody wrote and ignores them.
  const int n_qg = (n_qt32 + 7) / 8;
  const unsigned char* dsbase = dS + (size_t)bh * n_qg * n_kvt * 65536;
  const unsigned lds0 = (unsigned)(size_t)smem;
  // past the end of the stream every request repeats the last stage, so that the counted waits
  // stay exact
  auto request_k = [&](int s, int slot) __attribute__((always_inline)) {
    const int sc = s < NS ? s : NS - 1;
#pragma unroll
    for (int e = 0; e < IPW; ++e) {
      const unsigned o = min((unsigned)(sc * DG_BC) + kslot[e], (unsigned)(S - 1)) * (unsigned)ROWB + kchunk[e];
      mx_dma16(kbase, o, lds0 + (unsigned)(slot * SM::KT) + 1024u * (unsigned)(IPW * wave + e));
    }
  };
  u32x4 dsr[DG_PD][4];  // the wave's dS pieces of the next DG_PD stages
  auto request_ds = [&](int s, u32x4 (&r)[4]) __attribute__((always_inline)) {
    const int sc = s < NS ? s : NS - 1;
    const unsigned blk = ((unsigned)qt * (unsigned)n_kvt + (unsigned)(sc >> 1)) * 65536u +
                         (unsigned)(sc & 1) * 32768u + (unsigned)wave * 4096u;
#pragma unroll
    for (int p = 0; p < 4; ++p) dg_load16(r[p], dsbase, blk + 1024u * p + 16u * lane);
  };

  // lane constants of the transposed reads: Kf^T fragments as in the attention kernels; dS^T
  // fragments: source lane (k' = (lane % 16) / 4, r = lane % 4) of a 16-lane group addresses
  // slot 4 (lane / 32) + k' (+ 8 for the second read) of the k-step, rows 16 h + 4 r .. with
  // h = (lane / 16) % 2
  unsigned x_lo, x_hi;
  mx_trfrag0<D>(lane, x_lo, x_hi);
  const unsigned bx = (unsigned)(((lane & 15) >> 2) * 32 + ((lane & 3) >> 1) * 16 + (lane & 1) * 8 +
                                 ((lane >> 4) & 1) * DG_PIECE + (lane >> 5) * 128);
  // this wave's dS buffer: written and read by this wave only, and a wave's LDS operations
  // execute in order, so the write of stage s simply follows the reads of stage s-1
  char* sD = smem + SM::OFF_DS + wave * DG_WST;

  // Issue order: Kf(u), dS(u) for the first PD stages; then in iteration i: Kf(i+PD), dS(i+PD).
  // Loads return in order, so at the top of iteration s stage s has landed once at most the
  // PD-1 younger stages are outstanding.
  constexpr int LPS = IPW + 4;  // loads of a wave per stage
#pragma unroll
  for (int u = 0; u < DG_PD; ++u) {
    request_k(u, u);
    request_ds(u, dsr[u]);
  }
  int rb = 0;
  // The loop runs whole groups of PD stages (stages past the end move the last stage's data once
  // more and compute nothing): a body without stage-count branches keeps every wave's load
  // stream, and the compiler's own wait counts for the register loads, the same in every trip.
  for (int s0 = 0; s0 < NS; s0 += DG_PD) {
#pragma unroll
    for (int u = 0; u < DG_PD; ++u) {
      const int s = s0 + u;
      mx_wait_loads<(DG_PD - 1) * LPS>();  // Kf(s) and dS(s) of this wave have landed
#pragma unroll
      for (int p = 0; p < 4; ++p)
        *reinterpret_cast<u32x4*>(sD + p * DG_PIECE + 16 * lane) = dsr[u][p];
      __syncthreads();  // Kf tile s complete; the buffer of Kf tile s-1 is free
      request_k(s + DG_PD, rb >= 1 ? rb - 1 : SM::NST - 1);
      request_ds(s + DG_PD, dsr[u]);
      // a wave skips the stages none of its rows can see (their blocks may not even be written)
      const bool vis = has_rows && s < NS && (!causal || s * DG_BC - off <= tw0 + 31);
      if (vis) {
        const char* sK = smem + rb * SM::KT;
        // fragments of k-step ks (16 slots): dS^T as the B operand, Kf^T (DB blocks of 32 head
        // dims) as A operands.  They are read one k-step ahead of their MFMAs: left to itself the
        // compiler reads each fragment right before its MFMA, and every MFMA then waits a full
        // LDS round trip.
        auto frags = [&](int ks, bf16x8& b, bf16x8 (&a)[DB]) __attribute__((always_inline)) {
          const char* dp = sD + (ks >> 1) * (2 * DG_PIECE) + (ks & 1) * 512 + bx;
          const uint2 blo = lds_read_tr(reinterpret_cast<const bf16*>(dp));
          const uint2 bhi = lds_read_tr(reinterpret_cast<const bf16*>(dp + 256));
          b = __builtin_bit_cast(bf16x8, make_uint4(blo.x, blo.y, bhi.x, bhi.y));
          const char* kr = sK + 16 * ks * ROWB;
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const uint2 lo = lds_read_tr(reinterpret_cast<const bf16*>(kr + (x_lo ^ (unsigned)(db << 6))));
            const uint2 hi = lds_read_tr(reinterpret_cast<const bf16*>(kr + (x_hi ^ (unsigned)(db << 6))));
            a[db] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
          }
        };
        bf16x8 b0, b1, a0[DB], a1[DB];
        frags(0, b0, a0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 4; ks += 2) {
          frags(ks + 1, b1, a1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int db = 0; db < DB; ++db) acc[db] = mfma32(a0[db], b0, acc[db]);
          __builtin_amdgcn_sched_barrier(0);
          if (ks + 2 < 4) frags(ks + 2, b0, a0);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int db = 0; db < DB; ++db) acc[db] = mfma32(a1[db], b1, acc[db]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      rb = rb == SM::NST - 1 ? 0 : rb + 1;
    }
  }
  mx_wait_loads<0>();  // the surplus requests must land before LDS is reused
  __syncthreads();

  // ---- epilogue: dQ^T -> rows through LDS; dQ = tau acc + dg W_r^T, rounded once, coalesced
  // stores (the 32 lanes of a half-wave write one row)
  {
    constexpr int ESTR = SM::ESTR;
    float* sE = reinterpret_cast<float*>(smem) + wave * (32 * ESTR);
    float* sW = reinterpret_cast<float*>(smem) + DG_BR * ESTR;
    const bool route = W_r != nullptr && dgate != nullptr;
    if (route)
      for (int i = tid; i < D * 3; i += DG_NT) sW[i] = W_r[i];
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
__global__ __launch_bounds__(DG_NT, 1) void bwd_dqg_kernel(
    const bf16* __restrict__ Kf, const unsigned char* __restrict__ dS,
    const float* __restrict__ dgate, const float* __restrict__ W_r, bf16* __restrict__ dQ,
    float tau, int Tq, int S, int causal, int n_qt32, int n_kvt, int n_qtiles, int BH,
    int interleave, int pair) {
  // all query tiles of one (batch, head) on ONE XCD (block index = 8 * slot + xcd), heaviest
  // tiles first; under a causal mask a workgroup takes query tile qt and then its mirror tile
  // n_qtiles-1-qt (equal weights, half as many workgroups)
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
  bwd_dqg_tile<D>(Kf, dS, dgate, W_r, dQ, tau, Tq, S, causal, n_qt32, n_kvt, qt0, bh);
  if (pair && qt1 != qt0) {
    __syncthreads();  // the first tile's output staging is dead
    bwd_dqg_tile<D>(Kf, dS, dgate, W_r, dQ, tau, Tq, S, causal, n_qt32, n_kvt, qt1, bh);
  }
}

template <int D>
hipError_t launch_dqg_t(const BwdDqgArgs& a, hipStream_t st) {
  const int n_qtiles = (a.Tq + DG_BR - 1) / DG_BR;
  const int pair = (a.causal && n_qtiles > 1) ? 1 : 0;
  const int n_first = pair ? (n_qtiles + 1) / 2 : n_qtiles;
  const long nblocks = (long)n_first * ((a.BH + 7) / 8) * 8;
  const int interleave = (!pair && nblocks <= 2 * 256) ? 1 : 0;
  const size_t smem = (size_t)DgSmem<D>::TOTAL;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dqg_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((bwd_dqg_kernel<D>), dim3((unsigned)nblocks), dim3(DG_NT), smem, st,
                     (const bf16*)a.Kf, (const unsigned char*)a.dS, a.dgate, a.W_r, (bf16*)a.dQ,
                     a.scale, a.Tq, a.S, a.causal, a.n_qt32, a.n_kvt, n_qtiles, a.BH, interleave,
                     pair);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_dqg_bf16(const BwdDqgArgs& a, hipStream_t st) {
  if (a.BH == 0 || a.Tq == 0) return hipSuccess;
  return a.d == 128 ? launch_dqg_t<128>(a, st) : launch_dqg_t<64>(a, st);
}

}  // namespace mka
