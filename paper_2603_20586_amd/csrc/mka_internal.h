// Host-side declarations shared by the C-ABI layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mka {

struct RouteArgs {
  const void* Q;      // [rows = B*H*Tq, d]
  const float* W_r;   // [d,3]
  const float* b_r;   // [3] or null
  float* G;           // [B*H, S, 3] or null
  int32_t* idx;       // [B*H*Tq] or null
  int BH, Tq, S, d;
  bool bf16;
  int mode = 0;       // mka_routing
};
hipError_t launch_route(const RouteArgs& a, hipStream_t st);

struct FwdArgs {
  const void* Q;
  const void* K[3];
  const void* V[3];
  const float* G;
  void* O;
  float* LSE;  // or null
  int BH, Tq, S, d;
  int len[3];
  int causal;
  float scale;
};
hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t st);
hipError_t launch_fwd_f32(const FwdArgs& a, hipStream_t st);

// dQ of the backward = tau sum_j dS[t,j] Kf[j] + dg W_r^T, [B*H,Tq,d] bf16
struct BwdDqArgs {
  const void* Q;
  const void* dO;
  const void* Kf;   // fused stream [B*H,S,d] bf16, as written by the main backward kernel
  const void* Vf;
  const float* LSE2p;  // [B*H,Tqp] LSE in log2 units, rows padded per (b,h)
  const float* Dp;     // [B*H,Tqp] D = dO.O
  const float* dgate;  // [B*H,Tq,3] gradient of the router logits, or null (gates were given)
  const float* W_r;    // [d,3] or null
  void* dQ;
  int BH, Tq, Tqp, S, d;
  int causal;
  float scale;
};
hipError_t launch_bwd_dq_bf16(const BwdDqArgs& a, hipStream_t st);

// dQ from stored score gradients: dQ = tau sum_j dS[t,j] Kf[j] + dg W_r^T
struct BwdDqgArgs {
  const void* Kf;      // fused keys [B*H,S,d] bf16, as written by the main backward kernel
  const void* dS;      // [B*H][ceil(n_qt32/8)][n_kvt][8] blocks of 8 KiB (128 slots x 32 rows, bf16)
  const float* dgate;  // [B*H,Tq,3] or null
  const float* W_r;    // [d,3] or null
  void* dQ;
  int BH, Tq, S, d;
  int n_qt32, n_kvt;   // 32-row query tiles and 128-slot key tiles per head
  int causal;
  float scale;
};
hipError_t launch_bwd_dqg_bf16(const BwdDqgArgs& a, hipStream_t st);

struct MixArgs {
  const void* Q;
  const void* K[3];
  const void* V[3];
  const float* G;  // gates per QUERY row [BH,Tq,3], or null (all ones)
  void* O;
  float* LSE;      // or null
  int BH, Tq, d;
  int S[3];        // slots per level (0: absent)
  int causal;
  float scale;
};
hipError_t launch_mix_bf16(const MixArgs& a, hipStream_t st);

// full (three-path) MKA: O = sum_l G[:,l] * A_l over rows [B*H*Tq]; null A_l = level absent
hipError_t launch_full_combine(const void* const A[3], const float* G, void* O, long rows, int d,
                               hipStream_t st);
// causal prefix mean along S of X [B*H,S,d] bf16 -> M; workspace of prefix_mean_workspace_bytes
size_t prefix_mean_workspace_bytes(int BH, int S, int d);
hipError_t launch_prefix_mean(const void* X, void* M, int BH, int S, int d, void* workspace,
                              hipStream_t st);

// decode over the fused KV cache in a paged pool [n_pages,H,P,d] (bf16)
struct PagedDecodeArgs {
  const void* q;           // [B,H,1,d]
  const void* Kpool;
  const void* Vpool;
  const int32_t* table;    // [B,max_pages] device
  const int32_t* seq_len;  // [B] device
  float* partial;          // [B*H,n_splits,d+2]
  void* O;                 // [B,H,1,d]
  float* LSE;              // [B,H] or null
  int B, H, d, P, max_pages, n_pages, n_splits;
  float scale;
};
hipError_t launch_paged_decode(const PagedDecodeArgs& a, hipStream_t st);

struct PrefuseArgs {
  const void* K[3];
  const void* V[3];
  const float* G;  // [BH,S,3]
  void* Kf;
  void* Vf;
  int BH, S, d;
  int len[3];
};
hipError_t launch_prefuse(const PrefuseArgs& a, hipStream_t st);

struct DecodeArgs {
  const void* q;
  const void* k_new[3];
  const void* v_new[3];
  void* Kc[3];
  void* Vc[3];
  float* Gc;
  const float* W_r;
  const float* b_r;
  void* O;
  float* LSE;
  int32_t* idx;
  int BH, d;
  int cap[3], capG;
  int len[3];   // AFTER the append
  int j_new;    // slot of the new token
  int S;        // j_new + 1
  int n_splits;
  float scale;
  bool bf16;
  int routing;     // how the new slot's gate is formed; hard modes switch on gate-aware loads
  float* partial;  // workspace [BH, n_splits, d + 2]
};
hipError_t launch_decode(const DecodeArgs& a, hipStream_t st);
int decode_auto_splits(int BH, int S);
constexpr int kMaxSplits = 64;

struct BwdArgs {
  const void* dO;
  const void* Q;
  const void* K[3];
  const void* V[3];
  const float* G;
  const void* O;
  const float* LSE;
  const float* W_r;  // or null
  void* dQ;
  void* dK[3];
  void* dV[3];
  float* dW_r;
  float* db_r;
  int BH, Tq, S, d;
  int len[3];
  int causal;
  float scale;
  void* workspace;
  size_t workspace_bytes;
};
hipError_t launch_bwd_bf16(const BwdArgs& a, hipStream_t st);
// with_ds: room for the stored score gradients (one product instead of three in the dQ kernel);
// 0 is returned for with_ds when the problem is too large for that route
size_t bwd_workspace_bytes(int BH, int Tq, int S, int d, bool with_ds);

}  // namespace mka
