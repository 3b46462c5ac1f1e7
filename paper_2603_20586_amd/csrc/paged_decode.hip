// Decode over the fused (routed) KV cache in a paged layout.  The paper caches the fused keys /
// values of Alg. 2 step 7 instead of raw token KV (section "Route-Fused MKA (FastMKA)") and
// switches from a contiguous to a paged KV layout for long contexts (section "Experimental
// Setup"); this is that configuration: one K and one V stream per head - a third of the bytes of
// the three raw caches - whose slots live in fixed-size pages of a pool, found through a page
// table per sequence.
//
//   O[b,h] = softmax(tau q[b,h] . Kf[b,h,0..len_b-1]^T) Vf[b,h,0..len_b-1]
//
// Pool layout [n_pages, H, P, d] (P slots per page, a power of two >= 16), table [B, max_pages]
// int32 (logical page -> physical page), per-sequence lengths on the device.  Split-K as in the
// contiguous decode: grid (n_splits, B*H), 16 lanes cover one slot's row with 16-byte
// non-temporal loads, a wave instruction four slots, a wave's 16 slots of a trip lie in one page
// (one table lookup per wave and trip), all eight loads of a trip are issued before the first
// use, max-shift online softmax per lane group, states merged wave -> workgroup -> split.
// Bound by reading the cache once.
#include "mka_dev.h"
#include "mka_internal.h"

namespace mka {

namespace {

template <int D>
__global__ __launch_bounds__(256) void paged_split_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ Kpool, const bf16* __restrict__ Vpool,
    const int32_t* __restrict__ table, const int32_t* __restrict__ seq_len,
    float* __restrict__ partial, int H, int logP, int max_pages, int n_pages, float c) {
  constexpr int EPL = 8, LPR = D / EPL, SPI = 64 / LPR, U = 16 / SPI, NWV = 4;
  __shared__ float sred[NWV][D + 2];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int sub = lane / LPR, cl = lane % LPR;
  const int split = blockIdx.x, n_splits = gridDim.x;
  const long bh = blockIdx.y;
  const int b = (int)(bh / H), h = (int)(bh % H);
  const int P = 1 << logP;
  // a length beyond what the table can address, or a page id outside the pool, is clamped: the
  // kernel never leaves the pool whatever the caller's table holds
  int S = seq_len[b];
  S = S < 0 ? 0 : (S > max_pages * P ? max_pages * P : S);
  // slices of whole 64-slot trips
  int chunk = (S + n_splits - 1) / n_splits;
  chunk = (chunk + 63) / 64 * 64;
  const int j_lo = split * chunk;
  const int j_hi = (j_lo + chunk < S) ? j_lo + chunk : S;

  float qf[EPL];
  {
    float t[EPL];
    unpack8(*reinterpret_cast<const uint4*>(q + bh * D + cl * EPL), t);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] = t[e] * c;
  }
  const int32_t* tab = table + (long)b * max_pages;
  const long page_stride = (long)H * P * D;        // elements per physical page
  const long head_off = (long)h * P * D + cl * EPL;

  float m = -INFINITY, z = 0.f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  for (int base = j_lo; base < j_hi; base += 64) {
    const int j0 = base + 16 * wave;  // the wave's 16 slots: inside one page (P >= 16)
    // a wave past the end of the sequence reads page 0 of the table (exists: S >= 1) and masks
    const int lp = j0 < S ? (j0 >> logP) : 0;
    int pg = tab[lp];
    pg = pg < 0 ? 0 : (pg >= n_pages ? n_pages - 1 : pg);
    const long pbase = (long)pg * page_stride + head_off + (long)((j0 < S ? j0 : 0) & (P - 1)) * D;
    uint4 rk[U], rv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int jj = SPI * u + sub;             // slot inside the wave's 16
      const bool in = j0 + jj < S;
      const long o = pbase + (long)(in ? jj : 0) * D;  // clamp inside the page
      rk[u] = load16_stream(Kpool + o);
      rv[u] = load16_stream(Vpool + o);
    }
    float s[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      unpack8(rk[u], kf);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kf[e], d);
      d = group_sum<LPR>(d);
      s[u] = (j0 + SPI * u + sub < j_hi) ? d : -INFINITY;
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
      float vv[EPL];
      unpack8(rv[u], vv);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vv[e], acc[e]);
    }
    m = m_new;
  }

  // merge the SPI lane groups of the wave, then the waves
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

// splits of a (batch, head) -> output row; an empty split has m = -inf and weight 0
template <int D>
__global__ __launch_bounds__(D) void paged_combine_kernel(const float* __restrict__ partial,
                                                          bf16* __restrict__ O,
                                                          float* __restrict__ LSE, int n_splits) {
  const long bh = blockIdx.x;
  const int e = threadIdx.x;
  const float* p = partial + bh * n_splits * (long)(D + 2);
  float mn = -INFINITY;
  for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, p[s * (D + 2) + D]);
  float a = 0.f, z = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float ms = p[s * (D + 2) + D];
    const float w = ms == -INFINITY ? 0.f : fast_exp2(ms - mn);
    a = fmaf(p[s * (D + 2) + e], w, a);
    z = fmaf(p[s * (D + 2) + D + 1], w, z);
  }
  O[bh * D + e] = (bf16)(z > 0.f ? a / z : 0.f);  // an empty sequence gives O = 0, LSE = -inf
  if (LSE && e == 0) LSE[bh] = z > 0.f ? (mn + log2f(z)) * kLn2 : -INFINITY;
}

template <int D>
hipError_t launch_paged_t(const PagedDecodeArgs& a, hipStream_t st) {
  int logP = 0;
  while ((1 << logP) < a.P) ++logP;
  hipLaunchKernelGGL((paged_split_kernel<D>), dim3(a.n_splits, a.B * a.H), dim3(256), 0, st,
                     (const bf16*)a.q, (const bf16*)a.Kpool, (const bf16*)a.Vpool, a.table,
                     a.seq_len, a.partial, a.H, logP, a.max_pages, a.n_pages, a.scale * kLog2e);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((paged_combine_kernel<D>), dim3(a.B * a.H), dim3(D), 0, st, a.partial,
                     (bf16*)a.O, a.LSE, a.n_splits);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_paged_decode(const PagedDecodeArgs& a, hipStream_t st) {
  if (a.B == 0 || a.H == 0) return hipSuccess;
  return a.d == 128 ? launch_paged_t<128>(a, st) : launch_paged_t<64>(a, st);
}

}  // namespace mka
