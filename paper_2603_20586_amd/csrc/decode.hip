// One decode step of route-fused attention (paper: Alg. 2 step 8 — append to the cache — then
// steps 5-7 and 9 for the single new query row of every (batch, head)).
//
// Three launches:
//   append   writes the new token's K/V entries into slot j_new of the supplied levels and the
//            new slot's gate (router on q, fp64 fma chain in ascending k, as in the router
//            kernel) into the gate cache; without router weights the gate row is left as the
//            caller wrote it;
//   split    grid (n_splits, B*H): a workgroup streams its slice of the six raw caches and the
//            gate cache exactly once with 16-byte loads (LPR lanes cover one slot's row, so a
//            wave instruction covers 64/LPR slots), mixes the three levels with the slot's
//            gates on the fly (the fused stream is never stored), and keeps a max-shift online
//            softmax state (m, z, acc[d]) per lane group; states are merged across the wave,
//            then across the workgroup's waves, and written as one partial per split;
//   combine  merges the partials of each (b,h) and writes O (and LSE).
// The split kernel is bound by HBM bandwidth: per slot it reads 6 rows of d elements plus
// 12 bytes of gates and does about 6 d fused multiply-adds.
#include <type_traits>

#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return v + __int_as_float(moved);
}

// Sum over aligned groups of LPR lanes; every lane of the group gets the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "lanes per row");
  v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);  // row_half_mirror: the other quad of the 8-lane half
  if constexpr (LPR >= 16) v = dpp_add<0x140>(v);  // row_mirror: the other half of the 16-lane row
  if constexpr (LPR >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

template <typename T>
struct Chunk;  // 16 bytes of a row, widened to f32
template <>
struct Chunk<bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) { unpack8(v, f); }
};
template <>
struct Chunk<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
};

template <typename T, int D>
__global__ __launch_bounds__(64) void decode_append_kernel(
    const T* __restrict__ q, const T* __restrict__ kn0, const T* __restrict__ kn1,
    const T* __restrict__ kn2, const T* __restrict__ vn0, const T* __restrict__ vn1,
    const T* __restrict__ vn2, T* __restrict__ Kc0, T* __restrict__ Kc1, T* __restrict__ Kc2,
    T* __restrict__ Vc0, T* __restrict__ Vc1, T* __restrict__ Vc2, float* __restrict__ Gc,
    const float* __restrict__ W_r, const float* __restrict__ b_r, int32_t* __restrict__ idx,
    int cap0, int cap1, int cap2, int capG, int j_new, int routing) {
  const long bh = blockIdx.x;
  const int lane = threadIdx.x;
  __shared__ double sg[3];
  const T* kn[3] = {kn0, kn1, kn2};
  const T* vn[3] = {vn0, vn1, vn2};
  T* Kc[3] = {Kc0, Kc1, Kc2};
  T* Vc[3] = {Vc0, Vc1, Vc2};
  const int cap[3] = {cap0, cap1, cap2};
#pragma unroll
  for (int l = 0; l < 3; ++l) {
    if (kn[l] && vn[l]) {
      for (int e = lane; e < D; e += 64) {
        Kc[l][(bh * cap[l] + j_new) * D + e] = kn[l][bh * D + e];
        Vc[l][(bh * cap[l] + j_new) * D + e] = vn[l][bh * D + e];
      }
    }
  }
  if (!W_r) return;  // the new slot's gate row is the caller's (uniform branch)
  if (lane < 3) {
    double acc = b_r ? (double)b_r[lane] : 0.0;
    for (int k = 0; k < D; ++k)
      acc = fma((double)(float)q[bh * D + k], (double)W_r[k * 3 + lane], acc);
    sg[lane] = acc;
  }
  __syncthreads();
  if (lane == 0) {
    float lam[3];
    const int best = gates_variant(sg[0], sg[1], sg[2], routing, lam);
    float* out = Gc + (bh * capG + j_new) * 3;
    out[0] = lam[0];
    out[1] = lam[1];
    out[2] = lam[2];
    if (idx) idx[bh] = best;
  }
}

// partial layout per (bh, split): acc[0..D-1], m (log2 units), z
// SKIP (hard routing, section "Routing Mechanism Ablation"): a level whose cached gate is exactly
// zero cannot contribute to the slot, so its K / V rows are not loaded (the load is predicated
// per lane group: with top-1 gates a third of the bytes is read).  The gates of a trip are then
// needed before its row loads are issued: they are fetched one trip ahead.
template <typename T, int D, int U, bool SKIP>
__global__ __launch_bounds__(256) void decode_split_kernel(
    const T* __restrict__ q, const T* __restrict__ K0, const T* __restrict__ K1,
    const T* __restrict__ K2, const T* __restrict__ V0, const T* __restrict__ V1,
    const T* __restrict__ V2, const float* __restrict__ Gc, float* __restrict__ partial, int S,
    int len0, int len1, int len2, int cap0, int cap1, int cap2, int capG, int chunk, float c) {
  constexpr int EPL = Chunk<T>::N;      // elements per lane
  constexpr int LPR = D / EPL;          // lanes per row
  constexpr int SPI = 64 / LPR;         // slots per wave instruction
  constexpr int NWV = 4;
  __shared__ float sred[NWV][D + 2];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int sub = lane / LPR, cl = lane % LPR;
  const int split = blockIdx.x, n_splits = gridDim.x;
  const long bh = blockIdx.y;
  const int j_lo = split * chunk;
  const int j_hi = (j_lo + chunk < S) ? j_lo + chunk : S;

  float qf[EPL];
  {
    float t[EPL];
    // q is tiny and shared by all lanes of a column; a plain load is fine
    const T* qp = q + bh * D + cl * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) t[e] = (float)qp[e];
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] = t[e] * c;
  }
  // K0..V2 are never null here (a level without memory arrives as another level's buffer with
  // length 0, see the launcher); everything below the per-(b,h) base is a 32-bit byte offset
  const char* k0 = reinterpret_cast<const char*>(K0 + bh * (long)cap0 * D + cl * EPL);
  const char* k1 = reinterpret_cast<const char*>(K1 + bh * (long)cap1 * D + cl * EPL);
  const char* k2 = reinterpret_cast<const char*>(K2 + bh * (long)cap2 * D + cl * EPL);
  const char* v0 = reinterpret_cast<const char*>(V0 + bh * (long)cap0 * D + cl * EPL);
  const char* v1 = reinterpret_cast<const char*>(V1 + bh * (long)cap1 * D + cl * EPL);
  const char* v2 = reinterpret_cast<const char*>(V2 + bh * (long)cap2 * D + cl * EPL);
  const char* gp = reinterpret_cast<const char*>(Gc + bh * (long)capG * 3);

  float m = -INFINITY, z = 0.f;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  constexpr int STEP = NWV * SPI;  // slots covered by the workgroup per sub-step
  const int lenmin = min(len0, min(len1, len2));
  // One trip = U sub-steps.  All 6 U raw 16-byte loads of the trip (and the gates) are issued
  // before the first use, unconditionally: an absent entry reads slot 0 of the same (b,h)
  // instead and its bits are replaced by zero (never multiplied by a zero gate, so stale NaN /
  // Inf bits in unused cache rows cannot leak).  FULL = every slot of the trip exists at every
  // level: no predicates at all.
  // gates of the trip that starts at `base` (a slot past the end of the slice reads row 0)
  float gpre[U][3];
  auto load_gates = [&](int base) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = base + u * STEP + wave * SPI + sub;
      const char* gj = gp + (j < j_hi ? (unsigned)j * 12u : 0u);
      gpre[u][0] = *reinterpret_cast<const float*>(gj);
      gpre[u][1] = *reinterpret_cast<const float*>(gj + 4);
      gpre[u][2] = *reinterpret_cast<const float*>(gj + 8);
    }
  };
  if (SKIP) load_gates(j_lo);
  auto trip = [&](int base, auto full_c) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_c)::value;
    uint4 rk[U][3], rv[U][3];
    float g[U][3];
    bool ok[U];
    if (SKIP) {
      const uint4 zero = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * STEP + wave * SPI + sub;
        ok[u] = FULL || j < j_hi;
        const unsigned rowb = (unsigned)j * (unsigned)(D * sizeof(T));
        const int lens[3] = {len0, len1, len2};
        const char* kb[3] = {k0, k1, k2};
        const char* vb[3] = {v0, v1, v2};
#pragma unroll
        for (int l = 0; l < 3; ++l) {
          const bool present = FULL || (ok[u] && j < lens[l]);
          g[u][l] = present ? gpre[u][l] : 0.f;
          rk[u][l] = zero;
          rv[u][l] = zero;
          if (g[u][l] != 0.f) {  // only these lanes issue the loads
            rk[u][l] = load16_stream(kb[l] + rowb);
            rv[u][l] = load16_stream(vb[l] + rowb);
          }
        }
      }
      load_gates(base + STEP * U);  // for the next trip
    } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = base + u * STEP + wave * SPI + sub;
      ok[u] = FULL || j < j_hi;
      const bool p0 = FULL || (ok[u] && j < len0), p1 = FULL || (ok[u] && j < len1),
                 p2 = FULL || (ok[u] && j < len2);
      const unsigned rowb = (unsigned)j * (unsigned)(D * sizeof(T));
      rk[u][0] = load16_stream(k0 + (p0 ? rowb : 0u));
      rk[u][1] = load16_stream(k1 + (p1 ? rowb : 0u));
      rk[u][2] = load16_stream(k2 + (p2 ? rowb : 0u));
      rv[u][0] = load16_stream(v0 + (p0 ? rowb : 0u));
      rv[u][1] = load16_stream(v1 + (p1 ? rowb : 0u));
      rv[u][2] = load16_stream(v2 + (p2 ? rowb : 0u));
      const char* gj = gp + (ok[u] ? (unsigned)j * 12u : 0u);
      g[u][0] = *reinterpret_cast<const float*>(gj);
      g[u][1] = *reinterpret_cast<const float*>(gj + 4);
      g[u][2] = *reinterpret_cast<const float*>(gj + 8);
      if (!FULL) {
        const uint4 zero = make_uint4(0, 0, 0, 0);
        if (!p0) { rk[u][0] = zero; rv[u][0] = zero; g[u][0] = 0.f; }
        if (!p1) { rk[u][1] = zero; rv[u][1] = zero; g[u][1] = 0.f; }
        if (!p2) { rk[u][2] = zero; rv[u][2] = zero; g[u][2] = 0.f; }
      }
    }
    }
    float s[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float d[3];
#pragma unroll
      for (int l = 0; l < 3; ++l) {
        float kk[EPL];
        Chunk<T>::unpack(rk[u][l], kk);
        d[l] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d[l] = fmaf(qf[e], kk[e], d[l]);
      }
      const float part = fmaf(g[u][0], d[0], fmaf(g[u][1], d[1], g[u][2] * d[2]));
      const float tot = row_sum<LPR>(part);
      s[u] = ok[u] ? tot : -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u]);
    const float m_new = fmaxf(m, mx);
    const float mref = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m - mref);
    z *= alpha;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float p = fast_exp2(s[u] - mref);
      z += p;
#pragma unroll
      for (int l = 0; l < 3; ++l) {
        const float w = p * g[u][l];
        float vv[EPL];
        Chunk<T>::unpack(rv[u][l], vv);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(w, vv[e], acc[e]);
      }
    }
    m = m_new;
  };
  for (int base = j_lo; base < j_hi; base += STEP * U) {
    if (base + STEP * U <= j_hi && base + STEP * U <= lenmin) trip(base, std::true_type{});
    else trip(base, std::false_type{});
  }

  // merge the SPI lane groups of the wave (same column chunk, different slots)
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
    const float m2 = __shfl_xor(m, o, 64);
    const float z2 = __shfl_xor(z, o, 64);
    const float mn = fmaxf(m, m2);
    const float mref = (mn == -INFINITY) ? 0.f : mn;
    const float a1 = fast_exp2(m - mref), a2 = fast_exp2(m2 - mref);
    z = z * a1 + z2 * a2;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float o2 = __shfl_xor(acc[e], o, 64);
      acc[e] = acc[e] * a1 + o2 * a2;
    }
    m = mn;
  }
  if (sub == 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) sred[wave][cl * EPL + e] = acc[e];
    if (cl == 0) {
      sred[wave][D] = m;
      sred[wave][D + 1] = z;
    }
  }
  __syncthreads();
  float* out = partial + (bh * n_splits + split) * (long)(D + 2);
  float mn = sred[0][D];
#pragma unroll
  for (int w = 1; w < NWV; ++w) mn = fmaxf(mn, sred[w][D]);
  const float mref = (mn == -INFINITY) ? 0.f : mn;
  for (int e = tid; e < D; e += 256) {
    float a = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) a += sred[w][e] * fast_exp2(sred[w][D] - mref);
    out[e] = a;
  }
  if (tid == 0) {
    float zz = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) zz += sred[w][D + 1] * fast_exp2(sred[w][D] - mref);
    out[D] = mn;
    out[D + 1] = zz;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(const float* __restrict__ partial,
                                                           T* __restrict__ O,
                                                           float* __restrict__ LSE, int n_splits) {
  const long bh = blockIdx.x;
  const int e = threadIdx.x;
  const float* p = partial + bh * n_splits * (long)(D + 2);
  float mn = -INFINITY;
  for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, p[s * (D + 2) + D]);
  float a = 0.f, z = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float w = fast_exp2(p[s * (D + 2) + D] - mn);  // mn is finite: slot 0 always exists
    a = fmaf(p[s * (D + 2) + e], w, a);
    z = fmaf(p[s * (D + 2) + D + 1], w, z);
  }
  O[bh * D + e] = (T)(a / z);
  if (LSE && e == 0) LSE[bh] = (mn + log2f(z)) * kLn2;
}

template <typename T, int D>
hipError_t launch_decode_t(const DecodeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((decode_append_kernel<T, D>), dim3(a.BH), dim3(64), 0, st, (const T*)a.q,
                     (const T*)a.k_new[0], (const T*)a.k_new[1], (const T*)a.k_new[2],
                     (const T*)a.v_new[0], (const T*)a.v_new[1], (const T*)a.v_new[2],
                     (T*)a.Kc[0], (T*)a.Kc[1], (T*)a.Kc[2], (T*)a.Vc[0], (T*)a.Vc[1],
                     (T*)a.Vc[2], a.Gc, a.W_r, a.b_r, a.idx, a.cap[0], a.cap[1], a.cap[2], a.capG,
                     a.j_new, a.routing);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // a level without memory borrows another level's buffer (and capacity) and has length 0: the
  // kernel then never uses what it reads from it
  const void* Kp[3];
  const void* Vp[3];
  int capp[3];
  int any = a.Kc[0] ? 0 : (a.Kc[1] ? 1 : 2);
  if (!a.Kc[any] || !a.Vc[any]) return hipErrorInvalidValue;
  for (int l = 0; l < 3; ++l) {
    const bool has = a.Kc[l] && a.Vc[l];
    Kp[l] = has ? a.Kc[l] : a.Kc[any];
    Vp[l] = has ? a.Vc[l] : a.Vc[any];
    capp[l] = has ? a.cap[l] : a.cap[any];
  }
  constexpr int EPL = Chunk<T>::N, LPR = D / EPL, SPI = 64 / LPR, U = 4;
  constexpr int GRAN = 4 * SPI * U;  // slots the workgroup covers per loop trip
  int chunk = (a.S + a.n_splits - 1) / a.n_splits;
  chunk = (chunk + GRAN - 1) / GRAN * GRAN;
  const float c = a.scale * kLog2e;
  const int l0 = a.Kc[0] && a.Vc[0] ? a.len[0] : 0, l1 = a.Kc[1] && a.Vc[1] ? a.len[1] : 0,
            l2 = a.Kc[2] && a.Vc[2] ? a.len[2] : 0;
  if (a.routing == 2 || a.routing == 3)  // hard routing: gate-aware loads
    hipLaunchKernelGGL((decode_split_kernel<T, D, U, true>), dim3(a.n_splits, a.BH), dim3(256), 0,
                       st, (const T*)a.q, (const T*)Kp[0], (const T*)Kp[1], (const T*)Kp[2],
                       (const T*)Vp[0], (const T*)Vp[1], (const T*)Vp[2], a.Gc, a.partial, a.S, l0,
                       l1, l2, capp[0], capp[1], capp[2], a.capG, chunk, c);
  else
    hipLaunchKernelGGL((decode_split_kernel<T, D, U, false>), dim3(a.n_splits, a.BH), dim3(256), 0,
                       st, (const T*)a.q, (const T*)Kp[0], (const T*)Kp[1], (const T*)Kp[2],
                       (const T*)Vp[0], (const T*)Vp[1], (const T*)Vp[2], a.Gc, a.partial, a.S, l0,
                       l1, l2, capp[0], capp[1], capp[2], a.capG, chunk, c);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(a.BH), dim3(D), 0, st, a.partial,
                     (T*)a.O, a.LSE, a.n_splits);
  return hipGetLastError();
}

}  // namespace

int decode_auto_splits(int BH, int S) {
  // aim at ~8 workgroups per compute unit (256 CUs) without making slices shorter than 512 slots
  int n = (2048 + BH - 1) / BH;
  const int by_len = (S + 511) / 512;
  if (n > by_len) n = by_len;
  if (n < 1) n = 1;
  if (n > kMaxSplits) n = kMaxSplits;
  return n;
}

hipError_t launch_decode(const DecodeArgs& a, hipStream_t st) {
  if (a.BH == 0) return hipSuccess;
  if (a.bf16) return a.d == 128 ? launch_decode_t<bf16, 128>(a, st) : launch_decode_t<bf16, 64>(a, st);
  return a.d == 128 ? launch_decode_t<float, 128>(a, st) : launch_decode_t<float, 64>(a, st);
}

}  // namespace mka
