// Device-side helpers shared by the gfx950 kernels: vector types for the MFMA
// builtins, bf16 <-> f32 conversion on packed dwords, DPP reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mka {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Elimination builds (measurement only, never shipped: the build script passes the flag on request,
// MKA_EXTRA_HIPCC_FLAGS=-DMKA_ELIM=<bits>).  Each bit removes one kind of work from the MFMA
// kernels' loops while every memory access and every loop count stays what it was; the results
// are wrong, the launch times say what the removed work costs on the critical path.
//   1 MFMAs   2 LDS fragment reads   4 exponentials   8 LDS-direct tile loads   16 loop barriers
// Under the board's power limit an elimination build also changes what the MFMAs draw (tiles that
// are never loaded are constant data), so the attention core has the opposite hooks as well,
// MKA_DOUBLE=<bits>: one kind of work done twice on the same data, results unchanged.
//   1 LDS fragment reads   2 LDS-direct tile loads   4 exponentials   8 two more FMAs per score
#ifndef MKA_ELIM
#define MKA_ELIM 0
#endif
#ifndef MKA_DOUBLE
#define MKA_DOUBLE 0
#endif

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// A dword holding two bf16 (low half = element 0).  Widening to f32 is exact.
__device__ __forceinline__ float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// Two f32 -> one dword of two bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  bf16x2 p = {(bf16)lo, (bf16)hi};
  return __builtin_bit_cast(uint32_t, p);
}

__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = bf16lo(u.x); f[1] = bf16hi(u.x);
  f[2] = bf16lo(u.y); f[3] = bf16hi(u.y);
  f[4] = bf16lo(u.z); f[5] = bf16hi(u.z);
  f[6] = bf16lo(u.w); f[7] = bf16hi(u.w);
}

__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 u;
  u.x = pack_bf16x2(f[0], f[1]);
  u.y = pack_bf16x2(f[2], f[3]);
  u.z = pack_bf16x2(f[4], f[5]);
  u.w = pack_bf16x2(f[6], f[7]);
  return u;
}

// Gates and routing index from the three fp64 router logits (Alg. 2 step 5: softmax over the
// levels; index = smallest level that attains the maximum).  The differences to the maximum are
// formed in fp64, the exponentials and the normalisation in f32: gates are stored as f32 and
// hold to about 2e-7 of the fp64 value.  Shared by the router and the decode append kernel so
// that a token's gate is the same bits whichever of them produced it.
__device__ __forceinline__ int gates_from_logits(double g0, double g1, double g2, float* lam) {
  int best = 0;
  double gm = g0;
  if (g1 > gm) { gm = g1; best = 1; }
  if (g2 > gm) { gm = g2; best = 2; }
  const float e0 = expf((float)(g0 - gm)), e1 = expf((float)(g1 - gm)), e2 = expf((float)(g2 - gm));
  const float inv = 1.0f / (e0 + e1 + e2);
  lam[0] = e0 * inv;
  lam[1] = e1 * inv;
  lam[2] = e2 * inv;
  return best;
}

// Gates of the routing variants (paper: section "Routing Mechanism Ablation"): mode 0 soft (the
// function above), 1 fixed 1/3, 2 hard top-2 (the smallest logit is dropped, the other two soft
// gates renormalised), 3 hard top-1 (indicator of the largest logit).  Ties go to the lower level.
// The decisions are taken on the fp64 logits.  Returns the argmax.
__device__ __forceinline__ int gates_variant(double g0, double g1, double g2, int mode, float* lam) {
  if (mode == 0) return gates_from_logits(g0, g1, g2, lam);
  int best = 0, drop = 0;
  double gm = g0, gn = g0;
  if (g1 > gm) { gm = g1; best = 1; }
  if (g2 > gm) { gm = g2; best = 2; }
  if (g1 <= gn) { gn = g1; drop = 1; }
  if (g2 <= gn) { gn = g2; drop = 2; }
  if (mode == 1) {
    lam[0] = lam[1] = lam[2] = 1.0f / 3.0f;
  } else if (mode == 3) {
    lam[0] = best == 0 ? 1.f : 0.f;
    lam[1] = best == 1 ? 1.f : 0.f;
    lam[2] = best == 2 ? 1.f : 0.f;
  } else {
    const float e0 = drop == 0 ? 0.f : expf((float)(g0 - gm));
    const float e1 = drop == 1 ? 0.f : expf((float)(g1 - gm));
    const float e2 = drop == 2 ? 0.f : expf((float)(g2 - gm));
    const float inv = 1.0f / (e0 + e1 + e2);
    lam[0] = e0 * inv;
    lam[1] = e1 * inv;
    lam[2] = e2 * inv;
  }
  return best;
}

// 16-byte streaming load (data that is read exactly once).
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte streaming store (data that no kernel of the same call reads back soon): past the
// caches, so that it does not push out what other workgroups are re-reading.
__device__ __forceinline__ void store16_stream(void* p, const uint4& v) {
  __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(p));
}

__device__ __forceinline__ float fast_exp2(float x) {
#if MKA_ELIM & 4
  return x;
#else
  return __builtin_amdgcn_exp2f(x);
#endif
}

// 32x32x16 bf16 MFMA, f32 accumulate.  Operand layout (wave of 64 lanes, lane l):
//   A (32 x 16): row l%32, k = 8*(l/32) .. +7        (8 bf16 per lane)
//   B (16 x 32): column l%32, k = 8*(l/32) .. +7
//   C/D (32 x 32): column l%32, register r holds row 8*(r/4) + 4*(l/32) + r%4
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
#if MKA_ELIM & 1
  asm volatile("; mfma removed" : "+v"(c) : "v"(a), "v"(b));  // keeps the operands' producers alive
  return c;
#else
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
}

// 16-byte MFMA operand fragment out of LDS (ds_read_b128)
__device__ __forceinline__ bf16x8 lds_frag(const void* p) {
#if MKA_ELIM & 2
  bf16x8 r;
  asm volatile("; lds read removed" : "=v"(r) : "v"((unsigned)(size_t)p));  // no instruction, address kept alive
  return r;
#else
  return *reinterpret_cast<const bf16x8*>(p);
#endif
}

// workgroup barrier inside the tile loops
__device__ __forceinline__ void loop_barrier() {
#if !(MKA_ELIM & 16)
  __syncthreads();
#endif
}

// Transposed 16-bit LDS read (gfx950): inside every 16-lane group, lane i receives, for
// k = 0..3, element (i & 3) of the 8 bytes addressed by lane 4k + (i >> 2).  With lane s
// addressing row (s >> 2), columns 4 (s & 3) .. +3 of a row-major block, lane i gets column i of
// rows 0..3: the block's transpose, which is the MFMA A-operand layout (row = lane, 4 k-values).
typedef short lds_v4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 lds_read_tr(const bf16* p) {
#if MKA_ELIM & 2
  uint2 r;
  asm volatile("; lds read removed" : "=v"(r) : "v"((unsigned)(size_t)p));
  return r;
#else
  typedef __attribute__((address_space(3))) lds_v4s* lptr;
  const lds_v4s v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
  return __builtin_bit_cast(uint2, v);
#endif
}
// Largest of 16 accumulator registers with eight three-operand maxima (no NaN canonicalisation
// of the inputs: they come out of an MFMA or are -inf).
__device__ __forceinline__ float max16(const f32x16& s) {
  float m;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(s[0]), "v"(s[1]), "v"(s[2]));
#pragma unroll
  for (int r = 3; r < 15; r += 2) asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(m), "v"(s[r]), "v"(s[r + 1]));
  asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(m), "v"(s[15]));
  return m;
}

// Exchange with the lane 32 away (the other half of the wave).
// One v_permlane32_swap (a VALU instruction of gfx950, no LDS round trip): with both operands
// equal to v, the first result holds the lower half's values in both halves of the wave, the
// second the upper half's; each lane then picks the one that is not its own.
__device__ __forceinline__ float xor32(float v) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const unsigned u = __float_as_uint(v);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float((threadIdx.x & 32) ? r.x : r.y);
}

// Sum / max over aligned groups of 2^k lanes via xor butterflies.
template <int WIDTH>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = 1; o < WIDTH; o <<= 1) v += __shfl_xor(v, o, 64);
  return v;
}
template <int WIDTH>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = 1; o < WIDTH; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace mka
