"""fp64 CPU oracle for FastMKA route-fused attention (TEST INFRASTRUCTURE ONLY).

Thin ctypes loader around ``oracle/mka_oracle.c``.  Nothing in the product
package imports this module; it is used by the tests, by the smoke check and by
the CPU-baseline leg of the benchmark.  It imports nothing from the HIP path.

Every function takes array-likes (numpy arrays or CPU torch tensors of any
float dtype, bf16 included), up-casts their exact values to fp64 and returns
fp64 numpy arrays.  Shapes: Q [B,H,Tq,d]; K_l, V_l [B,H,S,d]; G [B,H,S,3];
W_r [d,3]; b_r [3].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mka_oracle.c")
_LIB = os.path.join(_HERE, "libmka_oracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp contraction off so fma() is the only fused op)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.mka_oracle_num_threads.restype = ctypes.c_int
        _lib.mka_oracle_decode.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().mka_oracle_num_threads())


def f64(x) -> np.ndarray:
    """Exact up-cast of an array-like (numpy / torch, any float dtype) to contiguous fp64."""
    if x is None:
        return None
    if hasattr(x, "detach"):  # torch tensor, without importing torch here
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _p(a):
    return a.ctypes.data_as(_dp) if a is not None else None


def _ilen(len3, S):
    return np.ascontiguousarray(np.asarray(len3 if len3 is not None else (S, S, S), dtype=np.int32))


def route(Q, W_r, b_r=None, S=None, G_prev=None):
    """Router gates for the Tq new slots.  Returns (G [B,H,S,3], idx [B,H,Tq] int32)."""
    Q, W_r, b_r = f64(Q), f64(W_r), f64(b_r)
    B, H, Tq, d = Q.shape
    S = Tq if S is None else S
    G = np.zeros((B, H, S, 3)) if G_prev is None else f64(G_prev).copy()
    assert G.shape == (B, H, S, 3) and W_r.shape == (d, 3)
    idx = np.zeros((B, H, Tq), dtype=np.int32)
    lib().mka_oracle_route(_p(Q), _p(W_r), _p(b_r), B, H, Tq, S, d, _p(G),
                           idx.ctypes.data_as(_ip))
    return G, idx


ROUTE_SOFT, ROUTE_FIXED, ROUTE_TOP2, ROUTE_TOP1 = 0, 1, 2, 3


def route_variant(Q, W_r, b_r=None, mode=ROUTE_SOFT, S=None, G_prev=None):
    """Gates of the routing ablation (soft / fixed 1/3 / hard top-2 / hard top-1) for the Tq new
    slots.  Returns (G [B,H,S,3], idx [B,H,Tq] int32 = argmax of the logits in every mode)."""
    Q, W_r, b_r = f64(Q), f64(W_r), f64(b_r)
    B, H, Tq, d = Q.shape
    S = Tq if S is None else S
    G = np.zeros((B, H, S, 3)) if G_prev is None else f64(G_prev).copy()
    assert G.shape == (B, H, S, 3) and W_r.shape == (d, 3)
    idx = np.zeros((B, H, Tq), dtype=np.int32)
    lib().mka_oracle_route_variant(_p(Q), _p(W_r), _p(b_r), int(mode), B, H, Tq, S, d, _p(G),
                                   idx.ctypes.data_as(_ip))
    return G, idx


def fuse(X, G, len3=None):
    """Xf[j] = sum_l [j < len_l] G[j,l] X_l[j] for a triple of memories X = (X1, X2, X3)."""
    X = [f64(x) for x in X]
    G = f64(G)
    ref = next(x for x in X if x is not None)
    B, H, S, d = ref.shape
    out = np.empty((B, H, S, d))
    ln = _ilen(len3, S)
    lib().mka_oracle_fuse(_p(X[0]), _p(X[1]), _p(X[2]), _p(G), ln.ctypes.data_as(_ip), B, H, S, d,
                          _p(out))
    return out


def attn_fwd(Q, Kf, Vf, causal=True, tau=1.0, return_p=False):
    """Plain softmax attention of Q over one K/V stream.  Returns (O, LSE[, P])."""
    Q, Kf, Vf = f64(Q), f64(Kf), f64(Vf)
    B, H, Tq, d = Q.shape
    S = Kf.shape[2]
    O = np.empty((B, H, Tq, d))
    LSE = np.empty((B, H, Tq))
    P = np.empty((B, H, Tq, S)) if return_p else None
    lib().mka_oracle_attn_fwd(_p(Q), _p(Kf), _p(Vf), B, H, Tq, S, d, int(bool(causal)),
                              ctypes.c_double(tau), _p(O), _p(LSE), _p(P))
    return (O, LSE, P) if return_p else (O, LSE)


def mixture_fwd(Q, K, V, lam=None, causal=True, tau=1.0):
    """Gated mixture of exponentiated scores over up to three memories of their own lengths
    (entries of K/V may be None).  lam [B,H,Tq,3] per QUERY row, or None for all ones.
    Returns (O, LSE)."""
    Q = f64(Q)
    B, H, Tq, d = Q.shape
    Ks = [None if k is None else f64(k) for k in K]
    Vs = [None if v is None else f64(v) for v in V]
    S = (ctypes.c_int * 3)(*[0 if k is None else k.shape[2] for k in Ks])
    lam = None if lam is None else f64(lam)
    O = np.empty((B, H, Tq, d))
    LSE = np.empty((B, H, Tq))
    lib().mka_oracle_mixture_fwd(_p(Q), _p(Ks[0]), _p(Ks[1]), _p(Ks[2]), _p(Vs[0]), _p(Vs[1]),
                                 _p(Vs[2]), _p(lam), B, H, Tq, S, d, int(bool(causal)),
                                 ctypes.c_double(tau), _p(O), _p(LSE))
    return O, LSE


def full_mka_fwd(Q, K, V, lam, causal=True, tau=1.0):
    """Symbolic (full) MKA, Alg. 1: one softmax attention per memory, a_l = softmax(tau Q K_l^T) V_l
    (every memory with its own length and bottom-right causal mask), combined at the output with
    the per-QUERY gates: O[t] = sum_l lam[t,l] a_l[t].  A missing memory (None) contributes a_l = 0
    (the algorithm's M_3 = 0 gives k_3 = v_3 = 0, hence a_3 = 0).  Returns O."""
    Q, lam = f64(Q), f64(lam)
    O = np.zeros_like(Q)
    for l in range(3):
        if K[l] is None or V[l] is None:
            continue
        a_l, _ = attn_fwd(Q, K[l], V[l], causal=causal, tau=tau)
        O += lam[..., l:l + 1] * a_l
    return O


def prefix_mean(X):
    """Causal prefix-mean summary, Alg. 1 (the L2 memory: M_2[t] = Summary(X[1..t]) with the
    "prefix mean" choice): M[t] = (1/(t+1)) sum_{s<=t} X[s] along axis 2, one running sum in
    ascending s.  Because the K/V projections are linear, the L2 keys/values are the prefix
    mean of the L1 keys/values, which is how it is used here."""
    X = f64(X)
    out = np.empty_like(X)
    run = np.zeros(X.shape[:2] + X.shape[3:])
    for t in range(X.shape[2]):
        run = run + X[:, :, t]
        out[:, :, t] = run / (t + 1)
    return out


def paged_gather(pool, table, seq_len, b, h):
    """Rows 0..seq_len[b]-1 of sequence b, head h out of a paged pool [n_pages,H,P,d]: slot j
    lives in page table[b][j // P] at row j % P."""
    P = pool.shape[2]
    n = int(seq_len[b])
    out = np.empty((n, pool.shape[3]))
    for j in range(n):
        out[j] = pool[int(table[b, j // P]), h, j % P]
    return out


def paged_fused_decode(q, Kpool, Vpool, table, seq_len, tau=1.0):
    """One decode step over the fused KV cache in a paged layout (what the paper caches, section
    "Route-Fused MKA (FastMKA)", in the paged layout of its long-context runs): for every (b,h)
    softmax attention of the single query row over the sequence's own slots, gathered through
    the page table.  q [B,H,1,d]; returns (O [B,H,1,d], LSE [B,H]); an empty sequence gives
    O = 0, LSE = -inf."""
    q, Kpool, Vpool = f64(q), f64(Kpool), f64(Vpool)
    table, seq_len = np.asarray(table), np.asarray(seq_len)
    B, H, _, d = q.shape
    O = np.zeros((B, H, 1, d))
    LSE = np.full((B, H), -np.inf)
    for b in range(B):
        for h in range(H):
            if seq_len[b] <= 0:
                continue
            Kd = paged_gather(Kpool, table, seq_len, b, h)[None, None]
            Vd = paged_gather(Vpool, table, seq_len, b, h)[None, None]
            o, l = attn_fwd(q[b:b + 1, h:h + 1], Kd, Vd, causal=False, tau=tau)
            O[b, h] = o[0, 0]
            LSE[b, h] = l[0, 0, 0]
    return O, LSE


def attn_fwd_blockwise(Q, Kf, Vf, Bc, causal=True, tau=1.0):
    """Same result through the max-shift recursion over KV blocks of Bc slots."""
    Q, Kf, Vf = f64(Q), f64(Kf), f64(Vf)
    B, H, Tq, d = Q.shape
    S = Kf.shape[2]
    O = np.empty((B, H, Tq, d))
    LSE = np.empty((B, H, Tq))
    lib().mka_oracle_attn_fwd_blockwise(_p(Q), _p(Kf), _p(Vf), B, H, Tq, S, d, int(bool(causal)),
                                        ctypes.c_double(tau), int(Bc), _p(O), _p(LSE))
    return O, LSE


def fwd(Q, K, V, G, len3=None, causal=True, tau=1.0):
    """Route-fused attention forward on given gates.  K, V are triples.  Returns (O, LSE)."""
    Q, G = f64(Q), f64(G)
    K = [f64(x) for x in K]
    V = [f64(x) for x in V]
    B, H, Tq, d = Q.shape
    S = G.shape[2]
    ln = _ilen(len3, S)
    O = np.empty((B, H, Tq, d))
    LSE = np.empty((B, H, Tq))
    lib().mka_oracle_fwd(_p(Q), _p(K[0]), _p(K[1]), _p(K[2]), _p(V[0]), _p(V[1]), _p(V[2]), _p(G),
                         ln.ctypes.data_as(_ip), B, H, Tq, S, d, int(bool(causal)),
                         ctypes.c_double(tau), _p(O), _p(LSE))
    return O, LSE


def fwd_routed(Q, K, V, W_r, b_r=None, G_prev=None, len3=None, causal=True, tau=1.0):
    """Router on Q for the new slots, then the forward.  Returns (O, LSE, G, idx)."""
    S = f64(K[0]).shape[2] if K[0] is not None else None
    G, idx = route(Q, W_r, b_r, S=S, G_prev=G_prev)
    O, LSE = fwd(Q, K, V, G, len3=len3, causal=causal, tau=tau)
    return O, LSE, G, idx


def decode(q, k_new, v_new, Kc, Vc, Gc, len3, W_r, b_r=None, tau=1.0):
    """One decode step.  Kc, Vc: lists of fp64 numpy caches [B,H,cap_l,d] UPDATED IN PLACE,
    Gc fp64 [B,H,capG,3] updated in place, len3 a length-3 int list updated in place.
    k_new / v_new: triples with None for a level that gets no new entry.
    Returns (O [B,H,1,d], LSE [B,H,1], idx [B,H])."""
    q = f64(q)
    B, H, _, d = q.shape
    kn = [f64(x) for x in k_new]
    vn = [f64(x) for x in v_new]
    for a in list(Kc) + list(Vc) + [Gc]:
        assert a.dtype == np.float64 and a.flags.c_contiguous
    W_r, b_r = f64(W_r), f64(b_r)
    cap = np.asarray([a.shape[2] for a in Kc], dtype=np.int32)
    capG = int(Gc.shape[2])
    ln = np.asarray(len3, dtype=np.int32)
    arr3 = _dp * 3
    O = np.empty((B, H, 1, d))
    LSE = np.empty((B, H, 1))
    idx = np.zeros((B, H), dtype=np.int32)
    rc = lib().mka_oracle_decode(_p(q), arr3(*[_p(x) for x in kn]), arr3(*[_p(x) for x in vn]),
                                 arr3(*[_p(x) for x in Kc]), arr3(*[_p(x) for x in Vc]), _p(Gc),
                                 ln.ctypes.data_as(_ip), cap.ctypes.data_as(_ip), capG, _p(W_r),
                                 _p(b_r), B, H, d, ctypes.c_double(tau), _p(O), _p(LSE),
                                 idx.ctypes.data_as(_ip))
    if rc != 0:
        raise ValueError("inconsistent append or cache full")
    for l in range(3):
        len3[l] = int(ln[l])
    return O, LSE, idx


def decode_variant(q, k_new, v_new, Kc, Vc, Gc, len3, W_r, b_r=None, mode=ROUTE_SOFT, tau=1.0):
    """One decode step whose new slot is gated by a routing variant (paper: section "Routing
    Mechanism Ablation"); same in-place contract as `decode`.  Written out of the pinned pieces:
    append the new entries at slot j_new = max(len), gate of the new slot = route_variant on q,
    then the route-fused forward (Alg. 2 steps 6-9) of the one query row over slots 0..j_new
    (bottom-right causal mask: the row sees every slot, itself included)."""
    q = f64(q)
    B, H, _, d = q.shape
    j_new = int(max(len3))
    for l in range(3):
        if k_new[l] is not None:
            if len3[l] != j_new or j_new >= Kc[l].shape[2]:
                raise ValueError("inconsistent append or cache full")
            Kc[l][:, :, j_new] = f64(k_new[l])[:, :, 0]
            Vc[l][:, :, j_new] = f64(v_new[l])[:, :, 0]
            len3[l] = j_new + 1
    S = j_new + 1
    g_new, idx = route_variant(q, W_r, b_r, mode)     # [B,H,1,3], [B,H,1]
    Gc[:, :, j_new] = g_new[:, :, 0]
    K = [None if a is None else np.ascontiguousarray(a[:, :, :S]) for a in Kc]
    V = [None if a is None else np.ascontiguousarray(a[:, :, :S]) for a in Vc]
    # a level shorter than S contributes nothing beyond its length (the caches may hold anything there)
    for l in range(3):
        if K[l] is not None:
            K[l][:, :, len3[l]:] = 0.0
            V[l][:, :, len3[l]:] = 0.0
    ref = next(a for a in K if a is not None)
    K = [np.zeros_like(ref) if a is None else a for a in K]
    V = [np.zeros_like(ref) if a is None else a for a in V]
    O, LSE = fwd(q, K, V, np.ascontiguousarray(Gc[:, :, :S]), len3=list(len3), causal=True, tau=tau)
    return O, LSE, idx[:, :, 0]


def bwd(dO, Q, K, V, G, W_r, len3=None, causal=True, tau=1.0, want_dG=False):
    """Gradients of sum(dO*O).  Returns dict with dQ, dK (triple), dV (triple), dW_r, db_r[, dG]."""
    dO, Q, G, W_r = f64(dO), f64(Q), f64(G), f64(W_r)
    K = [f64(x) for x in K]
    V = [f64(x) for x in V]
    B, H, Tq, d = Q.shape
    S = G.shape[2]
    ln = _ilen(len3, S)
    dQ = np.empty_like(Q)
    dK = [np.empty((B, H, S, d)) for _ in range(3)]
    dV = [np.empty((B, H, S, d)) for _ in range(3)]
    dW = np.empty((d, 3))
    db = np.empty(3)
    dG = np.empty((B, H, S, 3)) if want_dG else None
    lib().mka_oracle_bwd(_p(dO), _p(Q), _p(K[0]), _p(K[1]), _p(K[2]), _p(V[0]), _p(V[1]), _p(V[2]),
                         _p(G), _p(W_r), ln.ctypes.data_as(_ip), B, H, Tq, S, d, int(bool(causal)),
                         ctypes.c_double(tau), _p(dQ), _p(dK[0]), _p(dK[1]), _p(dK[2]), _p(dV[0]),
                         _p(dV[1]), _p(dV[2]), _p(dW), _p(db), _p(dG))
    out = {"dQ": dQ, "dK": dK, "dV": dV, "dW_r": dW, "db_r": db}
    if want_dG:
        out["dG"] = dG
    return out
