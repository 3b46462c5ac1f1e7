/*
 * mka.h — C ABI of the MI355X (gfx950) FastMKA route-fused attention library.
 *
 * The operations are those of the paper's Algorithm 2 ("FastMKA: Route-Fused
 * MKA"), restricted to head-level tensors:
 *   step 5   routing gates        lam = softmax_3(Q W_r + b_r), one triple per token
 *   step 6-7 route-fusion         Kf[j] = sum_l lam_l[j] K_l[j],  Vf[j] likewise
 *   step 8   cache update         append the new token's entries
 *   step 9   single attention     O = softmax(tau Q Kf^T, causal) Vf     (Eq. 1, tau of Eq. 3)
 * evaluated block-wise with the max-shift online softmax of the section
 * "Numerical Stability via Max-Shift".  The gate of slot j is the gate of the
 * token that produced slot j (token-aligned product of step 6), so the three
 * memories are slot-aligned: K_l, V_l all have S slots, the last Tq of which
 * belong to the Tq query rows of the call.
 *
 * Conventions, all entry points:
 *  - every tensor pointer is a DEVICE pointer owned by the caller, dense
 *    row-major, 16-byte aligned:  Q,O,dO,dQ [B,H,Tq,d];  K_l,V_l,dK_l,dV_l
 *    [B,H,S,d];  G [B,H,S,3] f32;  LSE [B,H,Tq] f32;  idx [B,H,Tq] int32;
 *    W_r [d,3] f32;  b_r [3] f32.  `dtype` is the element type of Q,K,V,O,dO
 *    and of the K/V/Q gradients; gates, LSE and router weights are always f32.
 *  - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work
 *    and return; they never synchronise, allocate, throw or abort.
 *  - scratch memory comes from the caller: `workspace` of at least
 *    mka_workspace_bytes(op, shape) bytes (device memory, 256-byte aligned).
 *  - every argument error is found on the host BEFORE anything is launched and
 *    reported as a status; nothing is written in that case.
 *  - supported: d in {64,128}; dtype MKA_BF16 (MFMA path) for every entry
 *    point, MKA_F32 (accuracy path) for route, forward and decode.
 *  - a level l with len[l] < S has no entry at slots j >= len[l]; it then
 *    contributes the zero vector there (Alg. 1's "M_3 <- 0") and the gates are
 *    not renormalised.  A NULL K[l]/V[l] pair means len[l] = 0.
 *  - causal masks are bottom-right aligned: row t sees slots j <= t + (S - Tq).
 */
#ifndef MKA_H_
#define MKA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MKA_OK = 0,
  MKA_ERR_NULL = 1,        /* a required pointer is NULL                           */
  MKA_ERR_SHAPE = 2,       /* non-positive size, S < Tq with causal, len[l] > S ... */
  MKA_ERR_DTYPE = 3,       /* unknown dtype                                        */
  MKA_ERR_ALIGN = 4,       /* a tensor pointer is not 16-byte aligned              */
  MKA_ERR_WORKSPACE = 5,   /* workspace missing or too small                       */
  MKA_ERR_UNSUPPORTED = 6, /* valid request this build has no kernel for           */
  MKA_ERR_LAUNCH = 7       /* the HIP runtime refused a launch                     */
} mka_status;

typedef enum { MKA_F32 = 0, MKA_BF16 = 1 } mka_dtype;

typedef enum {
  MKA_OP_ROUTE = 0,
  MKA_OP_FWD = 1,              /* what mka_fused_attn_fwd should be given for this shape  */
  MKA_OP_DECODE = 2,
  MKA_OP_BWD = 3,              /* what mka_fused_attn_bwd should be given for this shape  */
  MKA_OP_FWD_MATERIALISED = 4, /* what makes mka_fused_attn_fwd write Kf, Vf (see there)   */
  MKA_OP_FULL_MKA = 5,         /* mka_full_attn_fwd: three partial outputs [B,H,Tq,d]      */
  MKA_OP_PREFIX_MEAN = 6,      /* mka_prefix_mean: chunk sums                              */
  MKA_OP_BWD_STORED_DS = 7,    /* what makes mka_fused_attn_bwd store dS (see there)       */
  MKA_OP_BWD_RECOMPUTE = 8     /* the least mka_fused_attn_bwd accepts (see there)         */
} mka_op;

/* Problem shape of route / forward / backward. */
typedef struct {
  int32_t B, H;   /* batch, heads (K/V have the same H as Q)                         */
  int32_t Tq;     /* query rows of this call                                          */
  int32_t S;      /* visible slots, including the Tq new ones (S >= Tq)               */
  int32_t d;      /* head dimension                                                   */
  int32_t len[3]; /* valid slots of each level, 0 <= len[l] <= S                      */
  int32_t dtype;  /* mka_dtype                                                        */
  int32_t causal; /* 0: every row sees all S slots; 1: bottom-right aligned causal    */
  float scale;    /* tau                                                              */
} mka_shape;

/* Problem shape of one decode step. */
typedef struct {
  int32_t B, H, d;
  int32_t cap[3];   /* allocated slots per (b,h) of each level's K and V cache        */
  int32_t capG;     /* allocated rows per (b,h) of the gate cache                     */
  int32_t dtype;    /* mka_dtype of q, k_new, v_new, caches, O                        */
  int32_t n_splits; /* split-K factor along the slots; 0 = let the library choose     */
  float scale;      /* tau                                                            */
  int32_t routing;  /* mka_routing of the new slot's gate (0 = MKA_ROUTE_SOFT)         */
} mka_decode_shape;

/* Bytes of device scratch the given operation needs (0 if none, and 0 for an
 * invalid shape: the entry point itself reports what is wrong).  For
 * MKA_OP_DECODE pass a mka_shape with B,H,d,dtype filled and S = the largest
 * slot count the cache will reach; the answer covers any n_splits choice. */
size_t mka_workspace_bytes(mka_op op, const mka_shape* shape);

/* Alg. 2 step 5.  Logits g[t,l] = b_r[l] + sum_k Q[t,k] W_r[k,l] are an fp64 fma
 * chain in ascending k (so the argmax is reproducible bit for bit); gates are
 * the 3-way softmax of the logits.
 *   Q      in   [B,H,Tq,d] dtype
 *   W_r    in   [d,3] f32;  b_r in [3] f32, NULL = zeros
 *   G_out  out  [B,H,S,3] f32: rows S-Tq .. S-1 are written, others untouched; NULL = skip
 *   idx_out out [B,H,Tq] int32: argmax_l g[t,l], ties to the lowest l; NULL = skip
 * Only B,H,Tq,S,d,dtype of the shape are read. */
mka_status mka_route(const void* Q, const float* W_r, const float* b_r, float* G_out,
                     int32_t* idx_out, const mka_shape* shape, void* stream);

/* Routing variants of the paper's ablation (section "Routing Mechanism Ablation", table
 * "Routing mechanism ablation"); the paper names them without formulas, this is the reading:
 *   MKA_ROUTE_SOFT   the learned soft gates of Alg. 2 step 5 (= mka_route)
 *   MKA_ROUTE_FIXED  lam = 1/3 for every level
 *   MKA_ROUTE_TOP2   the level with the smallest logit gets 0, the other two soft gates are
 *                    renormalised to sum 1
 *   MKA_ROUTE_TOP1   the gate is the indicator of the largest logit
 * Ties go to the lower level (argmax: lowest index; dropped level: highest index among equal
 * minima); the decisions are taken on the fp64 logits of mka_route.  Arguments, layout and
 * errors as for mka_route (W_r is required in every mode: idx_out is the argmax of the logits);
 * an unknown mode gives MKA_ERR_UNSUPPORTED.  The gates are data for mka_fused_attn_fwd and
 * mka_fused_attn_bwd called without W_r (hard gates carry no router gradient). */
typedef enum {
  MKA_ROUTE_SOFT = 0,
  MKA_ROUTE_FIXED = 1,
  MKA_ROUTE_TOP2 = 2,
  MKA_ROUTE_TOP1 = 3
} mka_routing;
mka_status mka_route_variant(const void* Q, const float* W_r, const float* b_r, int32_t mode,
                             float* G_out, int32_t* idx_out, const mka_shape* shape,
                             void* stream);

/* Alg. 2 steps 5-7 and 9 for Tq query rows (prefill, or a training forward).
 *   Q     in     [B,H,Tq,d]
 *   K,V   in     three [B,H,S,d] each (entry NULL = level absent)
 *   W_r   in     router weights; NULL = take every row of G as given
 *   b_r   in     router bias, NULL = zeros
 *   G     in/out [B,H,S,3] f32, required.  With W_r: rows S-Tq..S-1 are computed
 *                from Q and written (rows below are the caller's, from earlier
 *                calls); without W_r: read only.
 *   O     out    [B,H,Tq,d] dtype
 *   LSE   out    [B,H,Tq] f32, log-sum-exp of the scaled visible scores; NULL = skip
 *   idx_out out  [B,H,Tq] int32 gate argmax (needs W_r); NULL = skip
 * Two routes compute the same thing (equal up to rounding order).  Folded: the
 * fusion happens tile by tile inside the attention kernel and Kf, Vf are never
 * written to memory; needs no workspace.  Materialised (bf16, d = 64 or 128): Kf
 * and Vf are written once to the workspace (step 6 as the algorithm states it)
 * and the attention kernel streams them; taken when `workspace` holds at least
 * mka_workspace_bytes(MKA_OP_FWD_MATERIALISED, shape) bytes (256-byte aligned),
 * else the folded route runs.  mka_workspace_bytes(MKA_OP_FWD, shape) is that
 * size when the library expects the materialised route to be the faster one
 * (long query blocks, where every query tile would fuse the same K/V tiles
 * again) and 0 otherwise, so a caller that sizes the workspace with it gets the
 * faster route.  The workspace contents are scratch: nothing is kept. */
mka_status mka_fused_attn_fwd(const void* Q, const void* const K[3], const void* const V[3],
                              const float* W_r, const float* b_r, float* G, void* O, float* LSE,
                              int32_t* idx_out, const mka_shape* shape, void* workspace,
                              size_t workspace_bytes, void* stream);

/* One decode step (Alg. 2 steps 5-9 with one query row per (b,h)):
 * the new token's slot is j_new = max_l len[l]; for every level with k_new[l] and
 * v_new[l] given, the entries are written to slot j_new of that level's cache
 * (requires len[l] == j_new < cap[l]) and len[l] becomes j_new+1; the new slot's
 * gate is the router on q and is written to Gc; then q attends over slots
 * 0..j_new of the fused stream (it sees itself), split along the slots.
 *   q        in      [B,H,1,d]
 *   k_new,v_new in   three [B,H,1,d] each, entry NULL = level gets no entry
 *   Kc,Vc    in/out  three caches [B,H,cap[l],d] each (NULL allowed if len[l]==0 and no k_new[l])
 *   Gc       in/out  [B,H,capG,3] f32 gate cache
 *   len      in/out  HOST array of 3: valid slots per level before / after the call
 *   W_r,b_r  in      router.  W_r NULL = row j_new of Gc is taken as the caller wrote it (as the
 *                    forward takes G without W_r); idx_out must then be NULL.  This is how a
 *                    cache of FUSED keys / values (section "Route-Fused MKA (FastMKA)": what the
 *                    paper caches; written by mka_fuse_kv) is decoded: the fused stream is level 1
 *                    alone, levels 2 and 3 NULL, every gate row (1,0,0), and k_new[0], v_new[0]
 *                    are the new token's fused rows.
 *   O        out     [B,H,1,d];  LSE out [B,H] f32 or NULL;  idx_out out [B,H] int32 or NULL
 * At least one level must be appended.  Per level cap[l] * d * sizeof(element) must stay below
 * 2^32 (MKA_ERR_UNSUPPORTED otherwise) and B * H below 65536.
 * shape->routing selects how the new slot's gate is formed from its logits (paper: section
 * "Routing Mechanism Ablation"; see mka_route_variant; an unknown value gives
 * MKA_ERR_UNSUPPORTED).  With hard routing (MKA_ROUTE_TOP2, MKA_ROUTE_TOP1) the attention does
 * not load the K / V rows of a level whose cached gate is exactly zero - they cannot contribute
 * - so a cache written with top-1 gates is read at a third of the bytes. */
mka_status mka_fused_attn_decode(const void* q, const void* const k_new[3],
                                 const void* const v_new[3], void* const Kc[3], void* const Vc[3],
                                 float* Gc, int32_t len[3], const float* W_r, const float* b_r,
                                 void* O, float* LSE, int32_t* idx_out,
                                 const mka_decode_shape* shape, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* mka_fused_attn_decode for callers that cannot allocate or hand over device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as mka_fused_attn_decode, without the workspace: the split-K partials live
 * in a fixed buffer of MKA_DECODE_STATIC_SCRATCH_BYTES inside the library's device image (every
 * GPU the library runs on holds its own copy until the process ends).  The call allocates
 * nothing and frees nothing.
 *  - limit: B * H * n_splits * (d + 2) * 4 bytes must fit the buffer.  With n_splits = 0 the
 *    library lowers its own split count until it fits; an explicit n_splits that does not fit,
 *    or a B * H that does not fit with one split, gives MKA_ERR_WORKSPACE and nothing runs.
 *    (Config C4 - B 16, H 32, d 128, 4 splits - needs 1.02 MiB.)
 *  - every call on a GPU shares that GPU's buffer and the buffer keeps the last call's contents:
 *    each call overwrites the partials it reads (nothing has to start at zero), but calls whose
 *    execution overlaps on one GPU - different streams, or a captured graph replayed while
 *    another call runs - race on it.  Serialise them on one stream. */
#define MKA_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
mka_status mka_fused_attn_decode_static(const void* q, const void* const k_new[3],
                                        const void* const v_new[3], void* const Kc[3],
                                        void* const Vc[3], float* Gc, int32_t len[3],
                                        const float* W_r, const float* b_r, void* O, float* LSE,
                                        int32_t* idx_out, const mka_decode_shape* shape,
                                        void* stream);

/* Backward of mka_fused_attn_fwd (chain rule through Alg. 2 steps 5-9) for the
 * loss sum(dO * O): gradients w.r.t. Q, every K_l, V_l, and the router.
 *   dO,Q,O in  [B,H,Tq,d];  K,V in three [B,H,S,d];  G in [B,H,S,3];  LSE in [B,H,Tq]
 *   W_r    in  [d,3] or NULL (gates were given: no router gradient, dW_r/db_r untouched)
 *   dQ     out [B,H,Tq,d] dtype (includes the path through the gates of the new slots)
 *   dK,dV  out three [B,H,S,d] dtype each (entry NULL = skip; zero where the level is absent)
 *   dW_r   out [d,3] f32, db_r out [3] f32 (set, not accumulated; NULL = skip)
 * Every output is a fixed-order sum: the same call gives the same bits (dQ is
 * accumulated in registers by a query-stationary kernel, dW_r/db_r by a
 * two-stage reduction).  The workspace holds the padded D / LSE rows, the gate gradients, the
 * router-gradient partial sums and the fused key / value streams.  Two routes to dQ:
 *  - stored score gradients: the key-stationary kernel (dK_l, dV_l, router gradient) also leaves
 *    dS in the workspace (bf16, 8 KiB per pair of a 128-slot key tile and a 32-row query tile, the
 *    full rectangle, streamed past the caches; config C5: 4 GiB) and the query-stationary dQ
 *    kernel reads them back - one product per pair.  Taken when the workspace holds at least
 *    mka_workspace_bytes(MKA_OP_BWD_STORED_DS, shape) bytes (0 = not provided for this shape: dS
 *    above 32 GiB in total or 4 GiB per head).
 *  - recomputation: the dQ kernel forms S, dP and dS a second time from the fused streams - three
 *    products per pair, a workspace of mka_workspace_bytes(MKA_OP_BWD_RECOMPUTE, shape) bytes,
 *    the least the call accepts (MKA_ERR_WORKSPACE below it).
 * Same result up to rounding order.  mka_workspace_bytes(MKA_OP_BWD, shape) is the size of the
 * route the library recommends: the first where it is provided (measured on MI355X in loops of
 * back-to-back calls: C5 2.22 against 2.37 ms, C2 0.374 against 0.390 ms), else the second. */
mka_status mka_fused_attn_bwd(const void* dO, const void* Q, const void* const K[3],
                              const void* const V[3], const float* G, const void* O,
                              const float* LSE, const float* W_r, void* dQ, void* const dK[3],
                              void* const dV[3], float* dW_r, float* db_r, const mka_shape* shape,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Route-fusion materialised (paper: Alg. 2 steps 6-7; the "single fused KV tensor" that the
 * paper caches): Kf[j] = sum_l [j < len[l]] G[j,l] K_l[j], Vf likewise, mixed in f32 and rounded
 * once to bf16.  K[l], V[l], Kf, Vf [B,H,S,d] (device, bf16, 16-byte aligned; Kf/Vf are fully
 * overwritten; a NULL K[l]/V[l] or slots j >= len[l] contribute the zero vector and the gates
 * are not renormalised; a level whose gate G[j,l] is exactly zero - hard routing - is not read
 * at that slot); G [B,H,S,3] f32 gates of the slots.  Reads shape->B,H,S,d,len,dtype.
 * Attention over the result is plain softmax attention: mka_mixture_attn_fwd with one memory
 * and G = NULL; it equals mka_fused_attn_fwd on the raw memories up to rounding order.
 * Enqueues on `stream` and returns; allocates nothing.  bf16 only, d in {64,128}. */
mka_status mka_fuse_kv(const void* const K[3], const void* const V[3], const float* G, void* Kf,
                       void* Vf, const mka_shape* shape, void* stream);

/* Gated mixture of exponentiated scores over up to three memories (paper: section "Theoretical
 * Formulation: Recursive MKA with Online Softmax", first equation, evaluated with the max-shift
 * recursion of that section) - the per-QUERY-gate formulation, a different function from the
 * route-fused path above:
 *
 *   O[t] = sum_l G[t,l] sum_j exp(scale Q[t].K_l[j]) V_l[j] / sum_l G[t,l] sum_j exp(scale Q[t].K_l[j])
 *
 * Q, O [B,H,Tq,d]; K[l], V[l] [B,H,len[l],d] (device, bf16, 16-byte aligned; a NULL entry or
 * len[l] == 0 means the memory is absent; the memories need not have equal lengths; shape->S is
 * not read); G [B,H,Tq,3] f32 gates of the query rows (e.g. from mka_route with S = Tq), or NULL
 * for all ones = softmax attention over the concatenation of the memories (with one memory:
 * plain attention, the kernel for a pre-fused K/V stream).  LSE [B,H,Tq] f32 (nullable) = log of
 * the denominator.  causal: every memory has its own bottom-right aligned mask (row t sees
 * slots j <= t + len[l] - Tq), which requires len[l] >= Tq (else MKA_ERR_SHAPE).  Rows that see
 * nothing (all visible memories gated off) give O = 0, LSE = -inf.  bf16 only
 * (MKA_ERR_UNSUPPORTED otherwise), d in {64, 128}.  Enqueues on `stream` and returns; allocates
 * nothing; O and LSE are fully overwritten.  Errors as for mka_fused_attn_fwd. */
mka_status mka_mixture_attn_fwd(const void* Q, const void* const K[3], const void* const V[3],
                                const float* G, void* O, float* LSE, const mka_shape* shape,
                                void* stream);

/* Symbolic (full) MKA, Alg. 1 of the paper - the three-path variant that FastMKA replaces: one
 * softmax attention per memory, mixed at the output with the gates of the QUERY rows:
 *
 *   a_l = softmax(scale Q K_l^T) V_l,      O[t] = sum_l G[t,l] a_l[t]
 *
 * Q, O [B,H,Tq,d]; K[l], V[l] [B,H,len[l],d] (device, bf16, 16-byte aligned; NULL entry or
 * len[l] == 0: the memory is absent and contributes a_l = 0, as the algorithm's M_3 = 0 does);
 * G [B,H,Tq,3] f32.  causal as for mka_mixture_attn_fwd (own bottom-right mask per memory,
 * len[l] >= Tq).  workspace: mka_workspace_bytes(MKA_OP_FULL_MKA, shape) bytes, 256-byte
 * aligned (the three partial outputs, bf16; scratch).  The launches are three plain attentions
 * and one combine pass.  bf16 only, d in {64,128}; errors as for mka_fused_attn_fwd. */
mka_status mka_full_attn_fwd(const void* Q, const void* const K[3], const void* const V[3],
                             const float* G, void* O, const mka_shape* shape, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Problem shape of a decode step over the paged fused-KV cache. */
typedef struct {
  int32_t B, H, d;
  int32_t page_size;  /* slots per page: a power of two, 16 <= page_size <= 1024            */
  int32_t n_pages;    /* pages in the pool                                                   */
  int32_t max_pages;  /* columns of the page table                                           */
  int32_t n_splits;   /* split-K factor along the slots, 1..64; 0 = let the library choose   */
  float scale;        /* tau                                                                 */
} mka_paged_shape;

/* Decode over the fused (routed) KV cache in a paged layout - what the paper caches (section
 * "Route-Fused MKA (FastMKA)": fused keys / values instead of raw token KV) in the layout it
 * uses for long contexts (section "Experimental Setup": contiguous up to 32K, paged beyond):
 *
 *   O[b,h] = softmax(scale q[b,h] . Kf[b,h,0..len[b]-1]^T) Vf[b,h,0..len[b]-1]
 *
 *   q        in  [B,H,1,d] bf16
 *   Kpool,Vpool in [n_pages,H,page_size,d] bf16: slot j of sequence b, head h lives in page
 *               table[b][j / page_size] at row j % page_size (e.g. written by mka_fuse_kv row by
 *               row as tokens arrive; filling the pool is the caller's)
 *   table    in  [B,max_pages] int32, device;  seq_len in [B] int32, device
 *   O        out [B,H,1,d] bf16;  LSE out [B,H] f32 or NULL
 * A length above max_pages * page_size and a page id outside the pool are clamped (the kernel
 * never reads outside the pool); a sequence of length 0 gives O = 0, LSE = -inf.
 * workspace: 64 * B*H * (d+2) * 4 bytes cover every n_splits (256-byte aligned).  bf16 only, d
 * in {64,128}.  Enqueues on `stream` and returns; allocates nothing. */
mka_status mka_paged_fused_decode(const void* q, const void* Kpool, const void* Vpool,
                                  const int32_t* table, const int32_t* seq_len, void* O, float* LSE,
                                  const mka_paged_shape* shape, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* Causal prefix-mean summary (Alg. 1: M_2[t] = Summary(X[1..t]), the "prefix mean" choice):
 * M[b,h,t,:] = mean over s <= t of X[b,h,s,:].  X, M [B,H,S,d] (device, bf16, 16-byte aligned,
 * M fully overwritten; B,H,S,d,dtype of the shape are read).  Applied to the L1 keys / values
 * it gives the L2 keys / values of Alg. 1 (the projections are linear).  Sums are f32 in a fixed
 * order (chunks of 64 rows); one rounding on store.  workspace:
 * mka_workspace_bytes(MKA_OP_PREFIX_MEAN, shape) bytes, 256-byte aligned. */
mka_status mka_prefix_mean(const void* X, void* M, const mka_shape* shape, void* workspace,
                           size_t workspace_bytes, void* stream);

/* Static, human-readable name of a status. */
const char* mka_status_string(mka_status status);

/* Library version as major*10000 + minor*100 + patch. */
int32_t mka_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MKA_H_ */
