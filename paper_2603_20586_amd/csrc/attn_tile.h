// Row-major 64-slot K / V tiles in LDS, filled straight from global memory and read as MFMA
// operands: layout (slot permutation + chunk swizzle), the LDS-direct load and the lane constants
// of the fragment reads.  Shared by the attention kernels that stream plain (already fused, or
// single-memory) K / V rows: the gated-mixture forward and the dQ kernel of the backward.
//
// An LDS-direct load (global_load_lds_dwordx4) writes the 64 lanes' 16 bytes to consecutive LDS
// addresses, so tile rows carry no padding; instead the 16-byte chunks of a row are XOR-swizzled
// by the row number and the slots of a tile are permuted over the rows (j = 4a+b -> row 4b+a
// inside every 16): row reads (ds_read_b128, 16 lanes = 16 rows, one chunk) and transposed reads
// (ds_read_b64_tr_b16, 4 rows x 4 chunks per 16 lanes) are then free of bank conflicts for
// d = 128 (the transposed reads of d = 64 are two-way conflicted).  The swizzle is applied on the
// global side: every lane picks the chunk that belongs at its LDS position.
#pragma once
#include "mka_dev.h"

namespace mka {

// LDS row of slot j (0..63) of a tile (an involution)
__device__ __forceinline__ int mx_row(int j) {
  return (j & ~15) | ((j & 3) << 2) | ((j >> 2) & 3);
}
// chunk c of row r sits at chunk position c ^ mx_swz(r) of the row
template <int D>
__device__ __forceinline__ int mx_swz(int r) {
  return D == 128 ? (r & 15) : ((r >> 1) & 7);
}

// 16 bytes per lane from global memory (uniform base + per-lane byte offset) to LDS address
// lds + 16 * lane.  Counted by vmcnt like any other load; the LDS write is done when the count
// drops.  m0 carries the LDS address (one wait state between its write and the load).
__device__ __forceinline__ void mx_dma16(const void* base, unsigned off, unsigned lds) {
#if MKA_ELIM & 8
  return;
#endif
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(base), "s"(lds)
               : "memory");
}
// 4 bytes per lane, each lane with its own address, to LDS address lds + 4 * lane.
__device__ __forceinline__ void mx_dma4(const void* src, unsigned lds) {
#if MKA_ELIM & 8
  return;
#endif
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :
               : "v"(src), "s"(lds)
               : "memory");
}
template <int N>
__device__ __forceinline__ void mx_wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// Byte offset, inside a tile, of the lane's first K fragment of unit 0 (slot li of the unit, head
// dims 8 g ..): fragment kk of unit u is at (a0 ^ (kk << 5)) + 32 u ROWB, because the chunk index
// 2 kk + g only meets the swizzle in an XOR and unit and tile offsets are multiples of 2 KiB.
template <int D>
__device__ __forceinline__ unsigned mx_kfrag0(int li, int g) {
  const int r = mx_row(li);
  return (unsigned)(r * (D * 2) + 16 * (g ^ mx_swz<D>(r)));
}

// Byte offsets, inside a 32-slot unit, of the lane's two transposed reads of MFMA k-step 0, head
// dims 0..31 (k positions 0..3 <-> slots 4 g + 0..3, positions 4..7 <-> slots 8 + 4 g + 0..3):
// the read of k-step ks, head-dim block db is at (x ^ (db << 6)) + 16 ks ROWB, because db only
// meets the swizzle in an XOR of address bits 6..7.
template <int D>
__device__ __forceinline__ void mx_trfrag0(int lane, unsigned& x_lo, unsigned& x_hi) {
  constexpr int ROWB = D * 2;
  const int g = lane >> 5, ti = lane & 15, gsel = (lane >> 4) & 1;
  const int cl = 2 * gsel + ((ti >> 1) & 1), sub = 8 * (ti & 1);
  const int r_lo = 4 * (ti >> 2) + g, r_hi = r_lo + 2;  // rows of slots 4 g + ti / 4 (+ 8)
  x_lo = (unsigned)(r_lo * ROWB + 16 * (cl ^ (mx_swz<D>(r_lo) & 3)) + sub) ^
         (unsigned)(16 * (mx_swz<D>(r_lo) & ~3));
  x_hi = (unsigned)(r_hi * ROWB + 16 * (cl ^ (mx_swz<D>(r_hi) & 3)) + sub) ^
         (unsigned)(16 * (mx_swz<D>(r_hi) & ~3));
}

}  // namespace mka
