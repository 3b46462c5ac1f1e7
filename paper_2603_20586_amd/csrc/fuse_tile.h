// Route-fusion of one 16-byte chunk (8 bf16) of a slot's three memory rows (paper: Alg. 2
// step 6, Xf = sum_l lam_l * L_l, applied to projected K/V rows): f32 math, caller rounds once.
//
// Loads are issued unconditionally so that a caller can batch many of them before the first
// use.  FULL = every level is present at the slot (interior tiles): no predicates at all.
// Otherwise the address of an absent entry is redirected to row 0 of the same (b,h) block,
// which always exists, and the loaded bits are replaced by zero — never multiplied by a zero
// gate, so stale NaN/Inf bits in unused cache rows cannot leak into the result.
#pragma once
#include "mka_dev.h"

namespace mka {

struct Raw3 {
  uint4 a, b, c;
};

// base_chunk: element offset of the same chunk in row 0 of this (b,h) block; eoff: element
// offset of the wanted chunk.  OFF is int when the pointers already address the (b,h) block
// (lets the compiler use scalar-base + 32-bit-offset addressing), long otherwise.
template <bool FULL, typename OFF>
__device__ __forceinline__ Raw3 load_raw3(const bf16* __restrict__ P0, const bf16* __restrict__ P1,
                                          const bf16* __restrict__ P2, OFF base_chunk, OFF eoff,
                                          bool p0, bool p1, bool p2) {
  Raw3 r;
  if constexpr (FULL) {
    r.a = *reinterpret_cast<const uint4*>(P0 + eoff);
    r.b = *reinterpret_cast<const uint4*>(P1 + eoff);
    r.c = *reinterpret_cast<const uint4*>(P2 + eoff);
  } else {
    r.a = *reinterpret_cast<const uint4*>(P0 + (p0 ? eoff : base_chunk));
    r.b = *reinterpret_cast<const uint4*>(P1 + (p1 ? eoff : base_chunk));
    r.c = *reinterpret_cast<const uint4*>(P2 + (p2 ? eoff : base_chunk));
    const uint4 z = make_uint4(0, 0, 0, 0);
    if (!p0) r.a = z;
    if (!p1) r.b = z;
    if (!p2) r.c = z;
  }
  return r;
}

// Same, addressed by 32-bit BYTE offsets from per-(b,h) base pointers that are uniform over the
// wave: the compiler can then keep the bases in scalar registers and needs no 64-bit vector
// address arithmetic per load.
template <bool FULL>
__device__ __forceinline__ Raw3 load_raw3_b(const bf16* __restrict__ P0, const bf16* __restrict__ P1,
                                            const bf16* __restrict__ P2, unsigned base_b,
                                            unsigned off_b, bool p0, bool p1, bool p2) {
  const char* c0 = reinterpret_cast<const char*>(P0);
  const char* c1 = reinterpret_cast<const char*>(P1);
  const char* c2 = reinterpret_cast<const char*>(P2);
  Raw3 r;
  if constexpr (FULL) {
    r.a = *reinterpret_cast<const uint4*>(c0 + off_b);
    r.b = *reinterpret_cast<const uint4*>(c1 + off_b);
    r.c = *reinterpret_cast<const uint4*>(c2 + off_b);
  } else {
    r.a = *reinterpret_cast<const uint4*>(c0 + (p0 ? off_b : base_b));
    r.b = *reinterpret_cast<const uint4*>(c1 + (p1 ? off_b : base_b));
    r.c = *reinterpret_cast<const uint4*>(c2 + (p2 ? off_b : base_b));
    const uint4 z = make_uint4(0, 0, 0, 0);
    if (!p0) r.a = z;
    if (!p1) r.b = z;
    if (!p2) r.c = z;
  }
  return r;
}

__device__ __forceinline__ void fuse8(const Raw3& r, float g0, float g1, float g2, float* out) {
  float f[8];
  unpack8(r.a, f);
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e] = g0 * f[e];
  unpack8(r.b, f);
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e] = fmaf(g1, f[e], out[e]);
  unpack8(r.c, f);
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e] = fmaf(g2, f[e], out[e]);
}

}  // namespace mka
