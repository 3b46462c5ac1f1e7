// C-ABI layer: argument validation on the host, workspace carve-up, kernel launches.
// Every error is found before anything is enqueued; see include/mka.h for the contract.
#include <math.h>
#include <string.h>

#include <mutex>

#include "../../include/mka.h"
#include "mka_internal.h"

// Split-K partials of mka_fused_attn_decode_static: a fixed buffer in every GPU's memory image,
// held until the process ends.  On the host this name is only a handle for hipGetSymbolAddress;
// the address that kernels and copies may use is looked up once per device (each GPU has its
// own copy of the array at its own address) and is the only thing host code passes on.
static __device__ __align__(256) unsigned char scratch[MKA_DECODE_STATIC_SCRATCH_BYTES];

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks shared by route / forward / backward.  `empty` is set for a valid problem with no
// query rows, which the caller answers with MKA_OK without launching.
mka_status check_shape(const mka_shape* s, bool* empty) {
  if (!s) return MKA_ERR_NULL;
  if (s->dtype != MKA_F32 && s->dtype != MKA_BF16) return MKA_ERR_DTYPE;
  if (s->B < 0 || s->H < 0 || s->Tq < 0 || s->S < 0 || s->d <= 0) return MKA_ERR_SHAPE;
  if (s->S < s->Tq) return MKA_ERR_SHAPE;
  for (int l = 0; l < 3; ++l)
    if (s->len[l] < 0 || s->len[l] > s->S) return MKA_ERR_SHAPE;
  if (s->d != 64 && s->d != 128) return MKA_ERR_UNSUPPORTED;
  if (!(s->scale >= 0.f) || isinf(s->scale)) return MKA_ERR_UNSUPPORTED;
  if ((long long)s->S * s->d >= 0x7fffffffLL) return MKA_ERR_UNSUPPORTED;  // 32-bit offsets per head
  const long long bh = (long long)s->B * s->H;
  if (bh > 0x7fffffffLL / 4096) return MKA_ERR_UNSUPPORTED;  // grid index must fit
  if (bh * (long long)((s->Tq + 31) / 32) > 0x7fffffffLL) return MKA_ERR_UNSUPPORTED;
  *empty = (bh == 0 || s->Tq == 0);
  return MKA_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

constexpr size_t kStaticScratchBytes = MKA_DECODE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, null until looked up
std::mutex g_scratch_mutex;

// Device address of the scratch array on the current device (looked up on first use).
mka_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MKA_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
      return MKA_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MKA_OK;
}

}  // namespace

extern "C" {

int32_t mka_version(void) { return 100; }

const char* mka_status_string(mka_status st) {
  switch (st) {
    case MKA_OK: return "MKA_OK";
    case MKA_ERR_NULL: return "MKA_ERR_NULL: a required pointer is NULL";
    case MKA_ERR_SHAPE: return "MKA_ERR_SHAPE: inconsistent sizes";
    case MKA_ERR_DTYPE: return "MKA_ERR_DTYPE: unknown dtype";
    case MKA_ERR_ALIGN: return "MKA_ERR_ALIGN: pointer not 16-byte aligned";
    case MKA_ERR_WORKSPACE: return "MKA_ERR_WORKSPACE: workspace missing or too small";
    case MKA_ERR_UNSUPPORTED: return "MKA_ERR_UNSUPPORTED: no kernel for this request";
    case MKA_ERR_LAUNCH: return "MKA_ERR_LAUNCH: the HIP runtime refused a launch";
  }
  return "MKA_ERR_?: unknown status";
}

// Kf and Vf of the materialised forward: [B,H,S,d] bf16 each, 256-byte aligned.
static size_t fwd_materialise_bytes(const mka_shape* s) {
  if (s->dtype != MKA_BF16 || (s->d != 64 && s->d != 128) || s->S <= 0) return 0;
  return 2 * align256((size_t)s->B * s->H * (size_t)s->S * (size_t)s->d * 2);
}
// Fusing once costs one pass over the six K/V tensors; folding it into the attention kernel
// costs about a quarter of the attention time (every query tile fuses its K/V tiles again, in
// registers).  The two break even near 3072 causal query rows (half that without the mask).
static bool fwd_prefers_materialised(const mka_shape* s) {
  if (fwd_materialise_bytes(s) == 0) return false;
  return (long)s->Tq * (s->causal ? 1 : 2) >= 3072;
}

size_t mka_workspace_bytes(mka_op op, const mka_shape* s) {
  if (!s || s->B <= 0 || s->H <= 0 || s->d <= 0) return 0;
  const size_t bh = (size_t)s->B * s->H;
  switch (op) {
    case MKA_OP_ROUTE:
      return 0;
    case MKA_OP_FWD:
      return fwd_prefers_materialised(s) ? fwd_materialise_bytes(s) : 0;
    case MKA_OP_FWD_MATERIALISED:
      return fwd_materialise_bytes(s);
    case MKA_OP_FULL_MKA:
      if (s->dtype != MKA_BF16 || s->Tq <= 0) return 0;
      return 3 * align256(bh * (size_t)s->Tq * (size_t)s->d * 2);
    case MKA_OP_PREFIX_MEAN:
      if (s->dtype != MKA_BF16 || s->S <= 0) return 0;
      return mka::prefix_mean_workspace_bytes((int)bh, s->S, s->d);
    case MKA_OP_DECODE:
      return align256(bh * mka::kMaxSplits * (size_t)(s->d + 2) * sizeof(float));
    case MKA_OP_BWD: {  // the recommended route: stored dS where provided
      if (s->Tq <= 0 || s->S < s->Tq) return 0;
      const size_t stored = mka::bwd_workspace_bytes((int)bh, s->Tq, s->S, s->d, true);
      return stored ? stored : mka::bwd_workspace_bytes((int)bh, s->Tq, s->S, s->d, false);
    }
    case MKA_OP_BWD_RECOMPUTE:
      if (s->Tq <= 0 || s->S < s->Tq) return 0;
      return mka::bwd_workspace_bytes((int)bh, s->Tq, s->S, s->d, false);
    case MKA_OP_BWD_STORED_DS:  // 0 when the problem is too large for that route
      if (s->Tq <= 0 || s->S < s->Tq) return 0;
      return mka::bwd_workspace_bytes((int)bh, s->Tq, s->S, s->d, true);
  }
  return 0;
}

mka_status mka_route(const void* Q, const float* W_r, const float* b_r, float* G_out,
                     int32_t* idx_out, const mka_shape* shape, void* stream) {
  return mka_route_variant(Q, W_r, b_r, MKA_ROUTE_SOFT, G_out, idx_out, shape, stream);
}

mka_status mka_route_variant(const void* Q, const float* W_r, const float* b_r, int32_t mode,
                             float* G_out, int32_t* idx_out, const mka_shape* shape,
                             void* stream) {
  if (mode < MKA_ROUTE_SOFT || mode > MKA_ROUTE_TOP1) return MKA_ERR_UNSUPPORTED;
  bool empty = false;
  mka_shape tmp;
  if (!shape) return MKA_ERR_NULL;
  tmp = *shape;  // route reads only B,H,Tq,S,d,dtype
  tmp.len[0] = tmp.len[1] = tmp.len[2] = 0;
  tmp.scale = 1.f;
  const mka_status st = check_shape(&tmp, &empty);
  if (st != MKA_OK) return st;
  if (!Q || !W_r) return MKA_ERR_NULL;
  if (!aligned16(Q) || !aligned16(G_out) || (reinterpret_cast<uintptr_t>(W_r) & 3u) ||
      (reinterpret_cast<uintptr_t>(idx_out) & 3u))
    return MKA_ERR_ALIGN;
  if (empty || (!G_out && !idx_out)) return MKA_OK;
  mka::RouteArgs a;
  a.Q = Q; a.W_r = W_r; a.b_r = b_r; a.G = G_out; a.idx = idx_out;
  a.BH = shape->B * shape->H; a.Tq = shape->Tq; a.S = shape->S; a.d = shape->d;
  a.bf16 = shape->dtype == MKA_BF16;
  a.mode = mode;
  return mka::launch_route(a, (hipStream_t)stream) == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

mka_status mka_fused_attn_fwd(const void* Q, const void* const K[3], const void* const V[3],
                              const float* W_r, const float* b_r, float* G, void* O, float* LSE,
                              int32_t* idx_out, const mka_shape* shape, void* workspace,
                              size_t workspace_bytes, void* stream) {
  bool empty = false;
  const mka_status st = check_shape(shape, &empty);
  if (st != MKA_OK) return st;
  if (!Q || !K || !V || !G || !O) return MKA_ERR_NULL;
  if (idx_out && !W_r) return MKA_ERR_NULL;
  if (!aligned16(Q) || !aligned16(G) || !aligned16(O) || !aligned16(LSE)) return MKA_ERR_ALIGN;
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return MKA_ERR_ALIGN;
  mka::FwdArgs a;
  for (int l = 0; l < 3; ++l) {
    if (!aligned16(K[l]) || !aligned16(V[l])) return MKA_ERR_ALIGN;
    const bool present = K[l] && V[l];
    a.K[l] = present ? K[l] : nullptr;
    a.V[l] = present ? V[l] : nullptr;
    a.len[l] = present ? shape->len[l] : 0;
  }
  if (!a.K[0] && !a.K[1] && !a.K[2]) return MKA_ERR_NULL;  // at least one memory level
  if (empty) return MKA_OK;
  hipStream_t hs = (hipStream_t)stream;
  const int BH = shape->B * shape->H;
  const bool is_bf16 = shape->dtype == MKA_BF16;
  if (W_r) {
    mka::RouteArgs r;
    r.Q = Q; r.W_r = W_r; r.b_r = b_r; r.G = G; r.idx = idx_out;
    r.BH = BH; r.Tq = shape->Tq; r.S = shape->S; r.d = shape->d; r.bf16 = is_bf16;
    if (mka::launch_route(r, hs) != hipSuccess) return MKA_ERR_LAUNCH;
  }
  const size_t mat_bytes = fwd_materialise_bytes(shape);
  if (workspace && mat_bytes > 0 && workspace_bytes >= mat_bytes) {
    // Alg. 2 step 6 as written: Kf, Vf once to the workspace, then attention over that stream
    mka::PrefuseArgs pf;
    for (int l = 0; l < 3; ++l) {
      pf.K[l] = a.K[l]; pf.V[l] = a.V[l]; pf.len[l] = a.len[l];
    }
    pf.G = G;
    pf.Kf = workspace;
    pf.Vf = static_cast<char*>(workspace) + mat_bytes / 2;
    pf.BH = BH; pf.S = shape->S; pf.d = shape->d;
    if (mka::launch_prefuse(pf, hs) != hipSuccess) return MKA_ERR_LAUNCH;
    mka::MixArgs mx;
    mx.Q = Q;
    mx.K[0] = pf.Kf; mx.V[0] = pf.Vf; mx.S[0] = shape->S;
    mx.K[1] = mx.K[2] = mx.V[1] = mx.V[2] = nullptr;
    mx.S[1] = mx.S[2] = 0;
    mx.G = nullptr; mx.O = O; mx.LSE = LSE;
    mx.BH = BH; mx.Tq = shape->Tq; mx.d = shape->d;
    mx.causal = shape->causal ? 1 : 0;
    mx.scale = shape->scale;
    return mka::launch_mix_bf16(mx, hs) == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
  }
  a.Q = Q; a.G = G; a.O = O; a.LSE = LSE;
  a.BH = BH; a.Tq = shape->Tq; a.S = shape->S; a.d = shape->d;
  a.causal = shape->causal ? 1 : 0;
  a.scale = shape->scale;
  const hipError_t e = is_bf16 ? mka::launch_fwd_bf16(a, hs) : mka::launch_fwd_f32(a, hs);
  return e == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

mka_status mka_fuse_kv(const void* const K[3], const void* const V[3], const float* G, void* Kf,
                       void* Vf, const mka_shape* shape, void* stream) {
  if (!shape) return MKA_ERR_NULL;
  if (shape->dtype != MKA_F32 && shape->dtype != MKA_BF16) return MKA_ERR_DTYPE;
  if (shape->B < 0 || shape->H < 0 || shape->S < 0 || shape->d <= 0) return MKA_ERR_SHAPE;
  if (shape->d != 64 && shape->d != 128) return MKA_ERR_UNSUPPORTED;
  if (shape->dtype != MKA_BF16) return MKA_ERR_UNSUPPORTED;
  if (!K || !V || !G || !Kf || !Vf) return MKA_ERR_NULL;
  if (!aligned16(Kf) || !aligned16(Vf) || (reinterpret_cast<uintptr_t>(G) & 3u)) return MKA_ERR_ALIGN;
  mka::PrefuseArgs a;
  bool any = false;
  for (int l = 0; l < 3; ++l) {
    if (!aligned16(K[l]) || !aligned16(V[l])) return MKA_ERR_ALIGN;
    if (shape->len[l] < 0 || shape->len[l] > shape->S) return MKA_ERR_SHAPE;
    const bool present = K[l] && V[l];
    a.K[l] = present ? K[l] : nullptr;
    a.V[l] = present ? V[l] : nullptr;
    a.len[l] = present ? shape->len[l] : 0;
    any = any || present;
  }
  if (!any) return MKA_ERR_NULL;
  a.G = G; a.Kf = Kf; a.Vf = Vf;
  a.BH = shape->B * shape->H; a.S = shape->S; a.d = shape->d;
  return mka::launch_prefuse(a, (hipStream_t)stream) == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

mka_status mka_mixture_attn_fwd(const void* Q, const void* const K[3], const void* const V[3],
                                const float* G, void* O, float* LSE, const mka_shape* shape,
                                void* stream) {
  if (!shape) return MKA_ERR_NULL;
  if (shape->dtype != MKA_F32 && shape->dtype != MKA_BF16) return MKA_ERR_DTYPE;
  if (shape->B < 0 || shape->H < 0 || shape->Tq < 0 || shape->d <= 0) return MKA_ERR_SHAPE;
  if (shape->d != 64 && shape->d != 128) return MKA_ERR_UNSUPPORTED;
  if (shape->dtype != MKA_BF16) return MKA_ERR_UNSUPPORTED;  // bf16 MFMA path only
  if (!(shape->scale >= 0.f) || isinf(shape->scale)) return MKA_ERR_UNSUPPORTED;
  if (!Q || !K || !V || !O) return MKA_ERR_NULL;
  if (!aligned16(Q) || !aligned16(O) || (reinterpret_cast<uintptr_t>(G) & 3u) ||
      (reinterpret_cast<uintptr_t>(LSE) & 3u))
    return MKA_ERR_ALIGN;
  mka::MixArgs a;
  bool any = false;
  for (int l = 0; l < 3; ++l) {
    if (!aligned16(K[l]) || !aligned16(V[l])) return MKA_ERR_ALIGN;
    if (shape->len[l] < 0) return MKA_ERR_SHAPE;
    const bool present = K[l] && V[l] && shape->len[l] > 0;
    // bottom-right aligned causal mask: a memory shorter than the query block would leave its
    // first rows without a diagonal
    if (present && shape->causal && shape->len[l] < shape->Tq) return MKA_ERR_SHAPE;
    if (present && (long long)shape->len[l] * shape->d >= (1ll << 31)) return MKA_ERR_UNSUPPORTED;
    a.K[l] = present ? K[l] : nullptr;
    a.V[l] = present ? V[l] : nullptr;
    a.S[l] = present ? shape->len[l] : 0;
    any = any || present;
  }
  if (!any) return MKA_ERR_NULL;  // at least one memory
  if (shape->B == 0 || shape->H == 0 || shape->Tq == 0) return MKA_OK;
  a.Q = Q; a.G = G; a.O = O; a.LSE = LSE;
  a.BH = shape->B * shape->H; a.Tq = shape->Tq; a.d = shape->d;
  a.causal = shape->causal ? 1 : 0;
  a.scale = shape->scale;
  return mka::launch_mix_bf16(a, (hipStream_t)stream) == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

mka_status mka_full_attn_fwd(const void* Q, const void* const K[3], const void* const V[3],
                             const float* G, void* O, const mka_shape* shape, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (!shape) return MKA_ERR_NULL;
  if (shape->dtype != MKA_F32 && shape->dtype != MKA_BF16) return MKA_ERR_DTYPE;
  if (shape->B < 0 || shape->H < 0 || shape->Tq < 0 || shape->d <= 0) return MKA_ERR_SHAPE;
  if (shape->d != 64 && shape->d != 128) return MKA_ERR_UNSUPPORTED;
  if (shape->dtype != MKA_BF16) return MKA_ERR_UNSUPPORTED;  // bf16 MFMA path only
  if (!(shape->scale >= 0.f) || isinf(shape->scale)) return MKA_ERR_UNSUPPORTED;
  if (!Q || !K || !V || !G || !O) return MKA_ERR_NULL;
  if (!aligned16(Q) || !aligned16(O) || (reinterpret_cast<uintptr_t>(G) & 3u)) return MKA_ERR_ALIGN;
  bool present[3];
  bool any = false;
  for (int l = 0; l < 3; ++l) {
    if (!aligned16(K[l]) || !aligned16(V[l])) return MKA_ERR_ALIGN;
    if (shape->len[l] < 0) return MKA_ERR_SHAPE;
    present[l] = K[l] && V[l] && shape->len[l] > 0;
    if (present[l] && shape->causal && shape->len[l] < shape->Tq) return MKA_ERR_SHAPE;
    if (present[l] && (long long)shape->len[l] * shape->d >= (1ll << 31)) return MKA_ERR_UNSUPPORTED;
    any = any || present[l];
  }
  if (!any) return MKA_ERR_NULL;
  if (shape->B == 0 || shape->H == 0 || shape->Tq == 0) return MKA_OK;
  const size_t per = align256((size_t)shape->B * shape->H * (size_t)shape->Tq * (size_t)shape->d * 2);
  if (!workspace || workspace_bytes < 3 * per) return MKA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MKA_ERR_ALIGN;
  hipStream_t hs = (hipStream_t)stream;
  const void* A[3] = {nullptr, nullptr, nullptr};
  for (int l = 0; l < 3; ++l) {
    if (!present[l]) continue;
    void* a_l = static_cast<char*>(workspace) + l * per;
    mka::MixArgs a;
    a.Q = Q;
    a.K[0] = K[l]; a.V[0] = V[l]; a.S[0] = shape->len[l];
    a.K[1] = a.K[2] = a.V[1] = a.V[2] = nullptr;
    a.S[1] = a.S[2] = 0;
    a.G = nullptr; a.O = a_l; a.LSE = nullptr;
    a.BH = shape->B * shape->H; a.Tq = shape->Tq; a.d = shape->d;
    a.causal = shape->causal ? 1 : 0;
    a.scale = shape->scale;
    if (mka::launch_mix_bf16(a, hs) != hipSuccess) return MKA_ERR_LAUNCH;
    A[l] = a_l;
  }
  const long rows = (long)shape->B * shape->H * shape->Tq;
  return mka::launch_full_combine(A, G, O, rows, shape->d, hs) == hipSuccess ? MKA_OK
                                                                              : MKA_ERR_LAUNCH;
}

mka_status mka_paged_fused_decode(const void* q, const void* Kpool, const void* Vpool,
                                  const int32_t* table, const int32_t* seq_len, void* O, float* LSE,
                                  const mka_paged_shape* s, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (!s) return MKA_ERR_NULL;
  if (s->B < 0 || s->H < 0 || s->d <= 0 || s->n_pages <= 0 || s->max_pages <= 0) return MKA_ERR_SHAPE;
  if (s->d != 64 && s->d != 128) return MKA_ERR_UNSUPPORTED;
  const int P = s->page_size;
  if (P < 16 || P > 1024 || (P & (P - 1))) return MKA_ERR_SHAPE;
  if ((long long)s->max_pages * P >= (1ll << 31)) return MKA_ERR_UNSUPPORTED;
  if (s->n_splits < 0 || s->n_splits > mka::kMaxSplits) return MKA_ERR_SHAPE;
  if (!(s->scale >= 0.f) || isinf(s->scale)) return MKA_ERR_UNSUPPORTED;
  if (!q || !Kpool || !Vpool || !table || !seq_len || !O) return MKA_ERR_NULL;
  if (!aligned16(q) || !aligned16(Kpool) || !aligned16(Vpool) || !aligned16(O) ||
      (reinterpret_cast<uintptr_t>(table) & 3u) || (reinterpret_cast<uintptr_t>(seq_len) & 3u) ||
      (reinterpret_cast<uintptr_t>(LSE) & 3u))
    return MKA_ERR_ALIGN;
  if ((long long)s->B * s->H > 65535) return MKA_ERR_UNSUPPORTED;  // grid.y
  const int BH = s->B * s->H;
  if (BH == 0) return MKA_OK;
  int ns = s->n_splits ? s->n_splits : mka::decode_auto_splits(BH, s->max_pages * P);
  const size_t need = align256((size_t)BH * ns * (size_t)(s->d + 2) * sizeof(float));
  if (!workspace || workspace_bytes < need) return MKA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MKA_ERR_ALIGN;
  mka::PagedDecodeArgs a;
  a.q = q; a.Kpool = Kpool; a.Vpool = Vpool; a.table = table; a.seq_len = seq_len;
  a.partial = static_cast<float*>(workspace); a.O = O; a.LSE = LSE;
  a.B = s->B; a.H = s->H; a.d = s->d; a.P = P; a.max_pages = s->max_pages; a.n_pages = s->n_pages;
  a.n_splits = ns; a.scale = s->scale;
  return mka::launch_paged_decode(a, (hipStream_t)stream) == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

mka_status mka_prefix_mean(const void* X, void* M, const mka_shape* shape, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (!shape) return MKA_ERR_NULL;
  if (shape->dtype != MKA_F32 && shape->dtype != MKA_BF16) return MKA_ERR_DTYPE;
  if (shape->B < 0 || shape->H < 0 || shape->S < 0 || shape->d <= 0) return MKA_ERR_SHAPE;
  if (shape->d != 64 && shape->d != 128) return MKA_ERR_UNSUPPORTED;
  if (shape->dtype != MKA_BF16) return MKA_ERR_UNSUPPORTED;
  if (!X || !M) return MKA_ERR_NULL;
  if (!aligned16(X) || !aligned16(M)) return MKA_ERR_ALIGN;
  const int BH = shape->B * shape->H;
  if (BH == 0 || shape->S == 0) return MKA_OK;
  if (!workspace || workspace_bytes < mka::prefix_mean_workspace_bytes(BH, shape->S, shape->d))
    return MKA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MKA_ERR_ALIGN;
  return mka::launch_prefix_mean(X, M, BH, shape->S, shape->d, workspace, (hipStream_t)stream) ==
                 hipSuccess
             ? MKA_OK
             : MKA_ERR_LAUNCH;
}

// Argument validation and append bookkeeping shared by the two decode entry points: fills `a`
// (everything but the partials buffer and the final split count) and sets *noop for a valid
// problem without heads.  Touches no device.
static mka_status decode_prepare(const void* q, const void* const k_new[3],
                                 const void* const v_new[3], void* const Kc[3], void* const Vc[3],
                                 float* Gc, const int32_t len[3], const float* W_r,
                                 const float* b_r, void* O, float* LSE, int32_t* idx_out,
                                 const mka_decode_shape* s, mka::DecodeArgs* out, bool* noop) {
  if (!s) return MKA_ERR_NULL;
  if (s->dtype != MKA_F32 && s->dtype != MKA_BF16) return MKA_ERR_DTYPE;
  if (s->B < 0 || s->H < 0 || s->d <= 0 || s->capG <= 0 || s->n_splits < 0) return MKA_ERR_SHAPE;
  if (s->d != 64 && s->d != 128) return MKA_ERR_UNSUPPORTED;
  if (!(s->scale >= 0.f) || isinf(s->scale)) return MKA_ERR_UNSUPPORTED;
  if (s->n_splits > mka::kMaxSplits) return MKA_ERR_UNSUPPORTED;
  if (s->routing < MKA_ROUTE_SOFT || s->routing > MKA_ROUTE_TOP1) return MKA_ERR_UNSUPPORTED;
  if (!q || !k_new || !v_new || !Kc || !Vc || !Gc || !len || !O) return MKA_ERR_NULL;
  if (idx_out && !W_r) return MKA_ERR_NULL;  // the argmax needs the router
  const long long bh = (long long)s->B * s->H;
  if (bh > 65535) return MKA_ERR_UNSUPPORTED;  // grid.y
  // the kernels address a (batch, head)'s cache rows with 32-bit byte offsets
  const long long row_bytes = (long long)s->d * (s->dtype == MKA_BF16 ? 2 : 4);
  if ((long long)s->capG * 12 >= (1ll << 32)) return MKA_ERR_UNSUPPORTED;
  int j_new = 0;
  for (int l = 0; l < 3; ++l) {
    if (s->cap[l] < 0 || len[l] < 0 || len[l] > s->cap[l]) return MKA_ERR_SHAPE;
    if ((long long)s->cap[l] * row_bytes >= (1ll << 32)) return MKA_ERR_UNSUPPORTED;
    if (len[l] > j_new) j_new = len[l];
  }
  if (j_new >= s->capG) return MKA_ERR_SHAPE;
  mka::DecodeArgs& a = *out;
  bool any = false;
  for (int l = 0; l < 3; ++l) {
    const bool app = k_new[l] && v_new[l];
    if ((k_new[l] != nullptr) != (v_new[l] != nullptr)) return MKA_ERR_NULL;
    if (app) {
      if (len[l] != j_new || j_new >= s->cap[l]) return MKA_ERR_SHAPE;
      if (!Kc[l] || !Vc[l]) return MKA_ERR_NULL;
      any = true;
    }
    if (len[l] > 0 && (!Kc[l] || !Vc[l])) return MKA_ERR_NULL;
    if (!aligned16(k_new[l]) || !aligned16(v_new[l]) || !aligned16(Kc[l]) || !aligned16(Vc[l]))
      return MKA_ERR_ALIGN;
    a.k_new[l] = app ? k_new[l] : nullptr;
    a.v_new[l] = app ? v_new[l] : nullptr;
    a.Kc[l] = Kc[l];
    a.Vc[l] = Vc[l];
    a.cap[l] = s->cap[l];
    a.len[l] = app ? j_new + 1 : len[l];
  }
  if (!any) return MKA_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(O) || (reinterpret_cast<uintptr_t>(Gc) & 3u)) return MKA_ERR_ALIGN;
  *noop = bh == 0;
  a.S = j_new + 1;
  a.n_splits = s->n_splits > 0 ? s->n_splits : (bh > 0 ? mka::decode_auto_splits((int)bh, a.S) : 1);
  a.q = q; a.Gc = Gc; a.W_r = W_r; a.b_r = b_r; a.O = O; a.LSE = LSE; a.idx = idx_out;
  a.BH = (int)bh; a.d = s->d; a.capG = s->capG; a.j_new = j_new;
  a.scale = s->scale; a.bf16 = s->dtype == MKA_BF16; a.routing = s->routing;
  a.partial = nullptr;
  return MKA_OK;
}

static size_t decode_partial_bytes(const mka::DecodeArgs& a) {
  return (size_t)a.BH * a.n_splits * (size_t)(a.d + 2) * sizeof(float);
}

mka_status mka_fused_attn_decode(const void* q, const void* const k_new[3],
                                 const void* const v_new[3], void* const Kc[3], void* const Vc[3],
                                 float* Gc, int32_t len[3], const float* W_r, const float* b_r,
                                 void* O, float* LSE, int32_t* idx_out,
                                 const mka_decode_shape* s, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  mka::DecodeArgs a;
  bool noop = false;
  const mka_status st =
      decode_prepare(q, k_new, v_new, Kc, Vc, Gc, len, W_r, b_r, O, LSE, idx_out, s, &a, &noop);
  if (st != MKA_OK) return st;
  if (noop) return MKA_OK;
  if (!workspace || workspace_bytes < decode_partial_bytes(a)) return MKA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MKA_ERR_ALIGN;
  a.partial = static_cast<float*>(workspace);
  if (mka::launch_decode(a, (hipStream_t)stream) != hipSuccess) return MKA_ERR_LAUNCH;
  for (int l = 0; l < 3; ++l) len[l] = a.len[l];
  return MKA_OK;
}

mka_status mka_fused_attn_decode_static(const void* q, const void* const k_new[3],
                                        const void* const v_new[3], void* const Kc[3],
                                        void* const Vc[3], float* Gc, int32_t len[3],
                                        const float* W_r, const float* b_r, void* O, float* LSE,
                                        int32_t* idx_out, const mka_decode_shape* s, void* stream) {
  mka::DecodeArgs a;
  bool noop = false;
  const mka_status st =
      decode_prepare(q, k_new, v_new, Kc, Vc, Gc, len, W_r, b_r, O, LSE, idx_out, s, &a, &noop);
  if (st != MKA_OK) return st;
  if (noop) return MKA_OK;
  // the library's own split count is lowered until the partials fit the fixed buffer; a count
  // the caller fixed, or a batch that does not fit with one split, is refused
  if (s->n_splits == 0)
    while (a.n_splits > 1 && decode_partial_bytes(a) > kStaticScratchBytes) --a.n_splits;
  if (decode_partial_bytes(a) > kStaticScratchBytes) return MKA_ERR_WORKSPACE;
  void* buf = nullptr;
  const mka_status sb = static_scratch(&buf);  // this device's copy of `scratch`
  if (sb != MKA_OK) return sb;
  a.partial = static_cast<float*>(buf);
  if (mka::launch_decode(a, (hipStream_t)stream) != hipSuccess) return MKA_ERR_LAUNCH;
  for (int l = 0; l < 3; ++l) len[l] = a.len[l];
  return MKA_OK;
}

mka_status mka_fused_attn_bwd(const void* dO, const void* Q, const void* const K[3],
                              const void* const V[3], const float* G, const void* O,
                              const float* LSE, const float* W_r, void* dQ, void* const dK[3],
                              void* const dV[3], float* dW_r, float* db_r, const mka_shape* shape,
                              void* workspace, size_t workspace_bytes, void* stream) {
  bool empty = false;
  const mka_status st = check_shape(shape, &empty);
  if (st != MKA_OK) return st;
  if (shape->dtype != MKA_BF16) return MKA_ERR_UNSUPPORTED;
  if (!dO || !Q || !K || !V || !G || !O || !LSE || !dQ || !dK || !dV) return MKA_ERR_NULL;
  if (!aligned16(dO) || !aligned16(Q) || !aligned16(G) || !aligned16(O) || !aligned16(LSE) ||
      !aligned16(dQ))
    return MKA_ERR_ALIGN;
  mka::BwdArgs a;
  for (int l = 0; l < 3; ++l) {
    if (!aligned16(K[l]) || !aligned16(V[l]) || !aligned16(dK[l]) || !aligned16(dV[l]))
      return MKA_ERR_ALIGN;
    const bool present = K[l] && V[l];
    a.K[l] = present ? K[l] : nullptr;
    a.V[l] = present ? V[l] : nullptr;
    a.len[l] = present ? shape->len[l] : 0;
    a.dK[l] = dK[l];
    a.dV[l] = dV[l];
  }
  if (!a.K[0] && !a.K[1] && !a.K[2]) return MKA_ERR_NULL;  // at least one memory level
  if (empty) return MKA_OK;
  const int BH = shape->B * shape->H;
  const size_t need = mka::bwd_workspace_bytes(BH, shape->Tq, shape->S, shape->d, false);
  if (!workspace || workspace_bytes < need) return MKA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MKA_ERR_ALIGN;
  a.dO = dO; a.Q = Q; a.G = G; a.O = O; a.LSE = LSE; a.W_r = W_r; a.dQ = dQ;
  a.dW_r = W_r ? dW_r : nullptr;
  a.db_r = W_r ? db_r : nullptr;
  a.BH = BH; a.Tq = shape->Tq; a.S = shape->S; a.d = shape->d;
  a.causal = shape->causal ? 1 : 0;
  a.scale = shape->scale;
  a.workspace = workspace;
  a.workspace_bytes = workspace_bytes;
  const hipError_t e = mka::launch_bwd_bf16(a, (hipStream_t)stream);
  if (e == hipErrorNotSupported) return MKA_ERR_UNSUPPORTED;
  return e == hipSuccess ? MKA_OK : MKA_ERR_LAUNCH;
}

}  // extern "C"
