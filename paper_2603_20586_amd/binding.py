"""ctypes binding of the C ABI in include/mka.h (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_float, c_int32, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmka.so")

MKA_F32, MKA_BF16 = 0, 1
MKA_OP_ROUTE, MKA_OP_FWD, MKA_OP_DECODE, MKA_OP_BWD, MKA_OP_FWD_MATERIALISED = 0, 1, 2, 3, 4
MKA_OP_FULL_MKA, MKA_OP_PREFIX_MEAN, MKA_OP_BWD_STORED_DS, MKA_OP_BWD_RECOMPUTE = 5, 6, 7, 8


class MkaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {status_string(status)}")


class MkaShape(ctypes.Structure):
    _fields_ = [("B", c_int32), ("H", c_int32), ("Tq", c_int32), ("S", c_int32), ("d", c_int32),
                ("len", c_int32 * 3), ("dtype", c_int32), ("causal", c_int32), ("scale", c_float)]


class MkaPagedShape(ctypes.Structure):
    _fields_ = [("B", c_int32), ("H", c_int32), ("d", c_int32), ("page_size", c_int32),
                ("n_pages", c_int32), ("max_pages", c_int32), ("n_splits", c_int32),
                ("scale", ctypes.c_float)]


class MkaDecodeShape(ctypes.Structure):
    _fields_ = [("B", c_int32), ("H", c_int32), ("d", c_int32), ("cap", c_int32 * 3),
                ("capG", c_int32), ("dtype", c_int32), ("n_splits", c_int32), ("scale", c_float),
                ("routing", c_int32)]


_P3 = c_void_p * 3
_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2603_20586_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        L = ctypes.CDLL(_LIB_PATH)
        L.mka_version.restype = c_int32
        L.mka_status_string.restype = ctypes.c_char_p
        L.mka_status_string.argtypes = [ctypes.c_int]
        L.mka_workspace_bytes.restype = c_size_t
        L.mka_workspace_bytes.argtypes = [ctypes.c_int, POINTER(MkaShape)]
        L.mka_route.restype = ctypes.c_int
        L.mka_route.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                POINTER(MkaShape), c_void_p]
        L.mka_full_attn_fwd.restype = ctypes.c_int
        L.mka_full_attn_fwd.argtypes = [c_void_p, POINTER(_P3), POINTER(_P3), c_void_p, c_void_p,
                                        POINTER(MkaShape), c_void_p, c_size_t, c_void_p]
        L.mka_prefix_mean.restype = ctypes.c_int
        L.mka_prefix_mean.argtypes = [c_void_p, c_void_p, POINTER(MkaShape), c_void_p, c_size_t,
                                      c_void_p]
        L.mka_paged_fused_decode.restype = ctypes.c_int
        L.mka_paged_fused_decode.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                             c_void_p, c_void_p, POINTER(MkaPagedShape), c_void_p,
                                             c_size_t, c_void_p]
        L.mka_route_variant.restype = ctypes.c_int
        L.mka_route_variant.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p,
                                        POINTER(MkaShape), c_void_p]
        L.mka_fused_attn_fwd.restype = ctypes.c_int
        L.mka_fused_attn_fwd.argtypes = [c_void_p, POINTER(_P3), POINTER(_P3), c_void_p, c_void_p,
                                         c_void_p, c_void_p, c_void_p, c_void_p,
                                         POINTER(MkaShape), c_void_p, c_size_t, c_void_p]
        L.mka_fused_attn_decode.restype = ctypes.c_int
        L.mka_fused_attn_decode.argtypes = [c_void_p, POINTER(_P3), POINTER(_P3), POINTER(_P3),
                                            POINTER(_P3), c_void_p, POINTER(c_int32 * 3),
                                            c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                            POINTER(MkaDecodeShape), c_void_p, c_size_t, c_void_p]
        L.mka_fused_attn_decode_static.restype = ctypes.c_int
        L.mka_fused_attn_decode_static.argtypes = [c_void_p, POINTER(_P3), POINTER(_P3), POINTER(_P3),
                                                   POINTER(_P3), c_void_p, POINTER(c_int32 * 3),
                                                   c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                                   POINTER(MkaDecodeShape), c_void_p]
        L.mka_fuse_kv.restype = ctypes.c_int
        L.mka_fuse_kv.argtypes = [POINTER(_P3), POINTER(_P3), c_void_p, c_void_p, c_void_p,
                                  POINTER(MkaShape), c_void_p]
        L.mka_mixture_attn_fwd.restype = ctypes.c_int
        L.mka_mixture_attn_fwd.argtypes = [c_void_p, POINTER(_P3), POINTER(_P3), c_void_p, c_void_p,
                                           c_void_p, POINTER(MkaShape), c_void_p]
        L.mka_fused_attn_bwd.restype = ctypes.c_int
        L.mka_fused_attn_bwd.argtypes = [c_void_p, c_void_p, POINTER(_P3), POINTER(_P3), c_void_p,
                                         c_void_p, c_void_p, c_void_p, c_void_p, POINTER(_P3),
                                         POINTER(_P3), c_void_p, c_void_p, POINTER(MkaShape),
                                         c_void_p, c_size_t, c_void_p]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().mka_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise MkaError(status, where)


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _p3(ts):
    return _P3(*[(t.data_ptr() if t is not None else None) for t in ts])


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return MKA_BF16
    if t.dtype == torch.float32:
        return MKA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> c_void_p:
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_check(*ts):
    for t in ts:
        if t is not None:
            if not t.is_cuda:
                raise ValueError("tensors must live in device memory")
            if not t.is_contiguous():
                raise ValueError("tensors must be contiguous")


def _f32_check(**ts):
    """Gates, LSE and router weights are float32 at the boundary whatever the tensor dtype."""
    for name, t in ts.items():
        if t is not None and t.dtype != torch.float32:
            raise TypeError(f"{name} must be float32, got {t.dtype}")


def _same_dtype(ref, **ts):
    """Q, K_l, V_l, O, dO and the caches share one element type (the shape's `dtype`)."""
    for name, t in ts.items():
        for x in (t if isinstance(t, (list, tuple)) else [t]):
            if x is not None and x.dtype != ref.dtype:
                raise TypeError(f"{name} must have the dtype of the queries ({ref.dtype}), got {x.dtype}")


def _shape(Q, S, len3, causal, scale) -> MkaShape:
    B, H, Tq, d = Q.shape
    s = MkaShape()
    s.B, s.H, s.Tq, s.S, s.d = B, H, Tq, S, d
    ln = len3 if len3 is not None else (S, S, S)
    for l in range(3):
        s.len[l] = int(ln[l])
    s.dtype = _dtype_code(Q)
    s.causal = int(bool(causal))
    s.scale = float(scale)
    return s


def mka_workspace_bytes(op: int, shape: MkaShape) -> int:
    return int(lib().mka_workspace_bytes(op, ctypes.byref(shape)))


def _workspace(nbytes: int, device):
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def mka_route(Q, W_r, b_r=None, S=None, G=None, want_idx=True):
    """Router gates (Alg. 2 step 5).  Returns (G [B,H,S,3] f32, idx [B,H,Tq] int32 or None).
    `G` may be an existing gate tensor whose rows S-Tq.. are overwritten."""
    _dev_check(Q, W_r, b_r, G)
    _f32_check(W_r=W_r, b_r=b_r, G=G)
    B, H, Tq, d = Q.shape
    S = Tq if S is None else S
    if G is None:
        G = torch.zeros((B, H, S, 3), dtype=torch.float32, device=Q.device)
    idx = torch.empty((B, H, Tq), dtype=torch.int32, device=Q.device) if want_idx else None
    s = _shape(Q, S, None, False, 1.0)
    _check(lib().mka_route(_ptr(Q), _ptr(W_r), _ptr(b_r), _ptr(G), _ptr(idx), ctypes.byref(s),
                           _stream()), "mka_route")
    return G, idx


MKA_ROUTE_SOFT, MKA_ROUTE_FIXED, MKA_ROUTE_TOP2, MKA_ROUTE_TOP1 = 0, 1, 2, 3


def mka_route_variant(Q, W_r, b_r=None, mode=MKA_ROUTE_SOFT, S=None, G=None, want_idx=True):
    """Gates of the routing ablation (soft / fixed 1/3 / hard top-2 / hard top-1).  Returns
    (G [B,H,S,3] f32, idx [B,H,Tq] int32 or None); arguments as for mka_route."""
    _dev_check(Q, W_r, b_r, G)
    _f32_check(W_r=W_r, b_r=b_r, G=G)
    B, H, Tq, d = Q.shape
    S = Tq if S is None else S
    if G is None:
        G = torch.zeros((B, H, S, 3), dtype=torch.float32, device=Q.device)
    idx = torch.empty((B, H, Tq), dtype=torch.int32, device=Q.device) if want_idx else None
    s = _shape(Q, S, None, False, 1.0)
    _check(lib().mka_route_variant(_ptr(Q), _ptr(W_r), _ptr(b_r), int(mode), _ptr(G), _ptr(idx),
                                   ctypes.byref(s), _stream()), "mka_route_variant")
    return G, idx


def mka_fused_attn_fwd(Q, K, V, W_r=None, b_r=None, G=None, len3=None, causal=True, scale=1.0,
                       want_lse=True, want_idx=True, O=None, LSE=None, idx=None, workspace=None,
                       materialise=None):
    """Route-fused attention forward.  K, V: sequences of three tensors (None = level absent).
    With W_r the router runs on Q and fills G's last Tq rows.  Returns (O, LSE, G, idx).
    `workspace`: uint8 device tensor handed to the library as it is.  Without one, `materialise`
    picks its size: None = what the library recommends for the shape, True = enough for the
    materialised route, False = none (folded route)."""
    _dev_check(Q, W_r, b_r, G, O, LSE, *K, *V)
    _f32_check(W_r=W_r, b_r=b_r, G=G, LSE=LSE)
    _same_dtype(Q, K=K, V=V, O=O)
    B, H, Tq, d = Q.shape
    ref = next(k for k in K if k is not None)
    S = ref.shape[2]
    if G is None:
        if W_r is None:
            raise ValueError("either W_r or G is required")
        G = torch.zeros((B, H, S, 3), dtype=torch.float32, device=Q.device)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None and want_lse:
        LSE = torch.empty((B, H, Tq), dtype=torch.float32, device=Q.device)
    if idx is None and want_idx and W_r is not None:
        idx = torch.empty((B, H, Tq), dtype=torch.int32, device=Q.device)
    s = _shape(Q, S, len3, causal, scale)
    k3, v3 = _p3(K), _p3(V)
    if workspace is None and materialise is not False:
        op = MKA_OP_FWD_MATERIALISED if materialise else MKA_OP_FWD
        nbytes = mka_workspace_bytes(op, s)
        if nbytes:
            workspace = _workspace(nbytes, Q.device)
    _check(lib().mka_fused_attn_fwd(_ptr(Q), ctypes.byref(k3), ctypes.byref(v3), _ptr(W_r),
                                    _ptr(b_r), _ptr(G), _ptr(O), _ptr(LSE), _ptr(idx),
                                    ctypes.byref(s), _ptr(workspace),
                                    workspace.numel() if workspace is not None else 0, _stream()),
           "mka_fused_attn_fwd")
    return O, LSE, G, idx


def mka_fused_attn_decode(q, k_new, v_new, Kc, Vc, Gc, len3, W_r, b_r=None, scale=1.0,
                          n_splits=0, workspace=None, O=None, LSE=None, idx=None, want_lse=True,
                          want_idx=True, routing=0):
    """One decode step; caches and `len3` (a python list of 3 ints) are updated in place.
    W_r None: the new slot's gate row in Gc is the caller's (fused-cache decode).  `routing`: MKA_ROUTE_* of the new slot's gate (hard modes read only the levels whose cached
    gate is not zero).  Returns (O [B,H,1,d], LSE [B,H] or None, idx [B,H] or None)."""
    _dev_check(q, W_r, b_r, Gc, O, LSE, *k_new, *v_new, *Kc, *Vc)
    _f32_check(W_r=W_r, b_r=b_r, Gc=Gc, LSE=LSE)
    _same_dtype(q, k_new=k_new, v_new=v_new, Kc=Kc, Vc=Vc, O=O)
    B, H, _, d = q.shape
    s = MkaDecodeShape()
    s.B, s.H, s.d = B, H, d
    for l in range(3):
        s.cap[l] = int(Kc[l].shape[2]) if Kc[l] is not None else 0
    s.capG = int(Gc.shape[2])
    s.dtype = _dtype_code(q)
    s.n_splits = int(n_splits)
    s.scale = float(scale)
    s.routing = int(routing)
    if workspace is None:
        qs = MkaShape()
        qs.B, qs.H, qs.d, qs.S, qs.Tq, qs.dtype = B, H, d, s.capG, 1, s.dtype
        workspace = _workspace(mka_workspace_bytes(MKA_OP_DECODE, qs), q.device)
    if O is None:
        O = torch.empty_like(q)
    if LSE is None and want_lse:
        LSE = torch.empty((B, H), dtype=torch.float32, device=q.device)
    if idx is None and want_idx and W_r is not None:
        idx = torch.empty((B, H), dtype=torch.int32, device=q.device)
    ln = (c_int32 * 3)(*[int(x) for x in len3])
    kn, vn, kc, vc = _p3(k_new), _p3(v_new), _p3(Kc), _p3(Vc)
    _check(lib().mka_fused_attn_decode(_ptr(q), ctypes.byref(kn), ctypes.byref(vn),
                                       ctypes.byref(kc), ctypes.byref(vc), _ptr(Gc),
                                       ctypes.byref(ln), _ptr(W_r), _ptr(b_r), _ptr(O), _ptr(LSE),
                                       _ptr(idx), ctypes.byref(s), _ptr(workspace),
                                       workspace.numel(), _stream()), "mka_fused_attn_decode")
    for l in range(3):
        len3[l] = int(ln[l])
    return O, LSE, idx


def mka_fused_attn_decode_static(q, k_new, v_new, Kc, Vc, Gc, len3, W_r, b_r, O, LSE=None, idx=None,
                                 scale=1.0, n_splits=0, routing=0):
    """mka_fused_attn_decode through the entry point that allocates nothing: the split-K partials
    live in the library's fixed device buffer, and every output tensor is the caller's (nothing
    is allocated here either).  Returns None; caches, `len3`, O, LSE, idx are updated in place."""
    _dev_check(q, W_r, b_r, Gc, O, LSE, idx, *k_new, *v_new, *Kc, *Vc)
    _f32_check(W_r=W_r, b_r=b_r, Gc=Gc, LSE=LSE)
    _same_dtype(q, k_new=k_new, v_new=v_new, Kc=Kc, Vc=Vc, O=O)
    B, H, _, d = q.shape
    s = MkaDecodeShape()
    s.B, s.H, s.d = B, H, d
    for l in range(3):
        s.cap[l] = int(Kc[l].shape[2]) if Kc[l] is not None else 0
    s.capG = int(Gc.shape[2])
    s.dtype = _dtype_code(q)
    s.n_splits, s.scale, s.routing = int(n_splits), float(scale), int(routing)
    ln = (c_int32 * 3)(*[int(x) for x in len3])
    kn, vn, kc, vc = _p3(k_new), _p3(v_new), _p3(Kc), _p3(Vc)
    _check(lib().mka_fused_attn_decode_static(_ptr(q), ctypes.byref(kn), ctypes.byref(vn),
                                              ctypes.byref(kc), ctypes.byref(vc), _ptr(Gc),
                                              ctypes.byref(ln), _ptr(W_r), _ptr(b_r), _ptr(O),
                                              _ptr(LSE), _ptr(idx), ctypes.byref(s), _stream()),
           "mka_fused_attn_decode_static")
    for l in range(3):
        len3[l] = int(ln[l])


def mka_fused_attn_bwd(dO, Q, K, V, G, O, LSE, W_r=None, len3=None, causal=True, scale=1.0,
                       workspace=None, grads_for=(True, True, True), stored_ds=None):
    """Backward of the forward.  Returns dict(dQ, dK[3], dV[3], dW_r, db_r).  Without a
    `workspace` one is allocated: of the size the library recommends (`stored_ds=None`), of the
    size with which the dQ kernel reads stored score gradients where the library provides that
    route (`True`), or of the smallest size, with which it recomputes them (`False`)."""
    _dev_check(dO, Q, G, O, LSE, W_r, *K, *V)
    _f32_check(W_r=W_r, G=G, LSE=LSE)
    _same_dtype(Q, dO=dO, O=O, K=K, V=V)
    B, H, Tq, d = Q.shape
    S = G.shape[2]
    s = _shape(Q, S, len3, causal, scale)
    if workspace is None:
        if stored_ds is None:
            nbytes = mka_workspace_bytes(MKA_OP_BWD, s)
        elif stored_ds:
            nbytes = max(mka_workspace_bytes(MKA_OP_BWD_RECOMPUTE, s),
                         mka_workspace_bytes(MKA_OP_BWD_STORED_DS, s))
        else:
            nbytes = mka_workspace_bytes(MKA_OP_BWD_RECOMPUTE, s)
        workspace = _workspace(nbytes, Q.device)
    dQ = torch.empty_like(Q)
    dK = [torch.empty_like(K[l]) if (K[l] is not None and grads_for[l]) else None
          for l in range(3)]
    dV = [torch.empty_like(V[l]) if (V[l] is not None and grads_for[l]) else None
          for l in range(3)]
    dW = torch.empty((d, 3), dtype=torch.float32, device=Q.device) if W_r is not None else None
    db = torch.empty((3,), dtype=torch.float32, device=Q.device) if W_r is not None else None
    k3, v3, dk3, dv3 = _p3(K), _p3(V), _p3(dK), _p3(dV)
    _check(lib().mka_fused_attn_bwd(_ptr(dO), _ptr(Q), ctypes.byref(k3), ctypes.byref(v3),
                                    _ptr(G), _ptr(O), _ptr(LSE), _ptr(W_r), _ptr(dQ),
                                    ctypes.byref(dk3), ctypes.byref(dv3), _ptr(dW), _ptr(db),
                                    ctypes.byref(s), _ptr(workspace), workspace.numel(),
                                    _stream()), "mka_fused_attn_bwd")
    return dict(dQ=dQ, dK=dK, dV=dV, dW_r=dW, db_r=db)


def mka_fuse_kv(K, V, G, len3=None, Kf=None, Vf=None):
    """Route-fusion materialised (Alg. 2 steps 6-7): returns (Kf, Vf), bf16 [B,H,S,d]."""
    _dev_check(G, Kf, Vf, *K, *V)
    _f32_check(G=G)
    ref = next(k for k in K if k is not None)
    _same_dtype(ref, K=K, V=V, Kf=Kf, Vf=Vf)
    B, H, S, d = ref.shape
    if Kf is None:
        Kf = torch.empty_like(ref)
    if Vf is None:
        Vf = torch.empty_like(ref)
    s = MkaShape()
    s.B, s.H, s.Tq, s.S, s.d = B, H, S, S, d
    ln = len3 if len3 is not None else (S, S, S)
    for l in range(3):
        s.len[l] = int(ln[l])
    s.dtype = _dtype_code(ref)
    s.causal, s.scale = 0, 1.0
    Kp, Vp = _p3(K), _p3(V)
    _check(lib().mka_fuse_kv(ctypes.byref(Kp), ctypes.byref(Vp), _ptr(G), _ptr(Kf), _ptr(Vf),
                             ctypes.byref(s), _stream()), "mka_fuse_kv")
    return Kf, Vf


def mka_mixture_attn_fwd(Q, K, V, G=None, causal=True, scale=1.0, want_lse=True, O=None, LSE=None):
    """Gated mixture of exponentiated scores over up to three memories of their own lengths
    (section "Recursive MKA with Online Softmax"); G [B,H,Tq,3] gates of the query rows or None.
    Returns (O, LSE)."""
    _dev_check(Q, G, O, LSE, *K, *V)
    _f32_check(G=G, LSE=LSE)
    _same_dtype(Q, K=K, V=V, O=O)
    B, H, Tq, d = Q.shape
    len3 = [0 if k is None else k.shape[2] for k in K]
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None and want_lse:
        LSE = torch.empty((B, H, Tq), dtype=torch.float32, device=Q.device)
    s = _shape(Q, max(len3 + [Tq]), len3, causal, scale)
    Kp, Vp = _p3(K), _p3(V)
    _check(lib().mka_mixture_attn_fwd(_ptr(Q), ctypes.byref(Kp), ctypes.byref(Vp), _ptr(G), _ptr(O),
                                      _ptr(LSE), ctypes.byref(s), _stream()), "mka_mixture_attn_fwd")
    return O, LSE


def mka_full_attn_fwd(Q, K, V, G, causal=True, scale=1.0, O=None, workspace=None):
    """Symbolic (full) MKA, Alg. 1: one attention per memory, outputs mixed with the gates of the
    query rows G [B,H,Tq,3].  Returns O."""
    _dev_check(Q, G, O, *K, *V)
    _f32_check(G=G)
    _same_dtype(Q, K=K, V=V, O=O)
    B, H, Tq, d = Q.shape
    len3 = [0 if k is None else k.shape[2] for k in K]
    if O is None:
        O = torch.empty_like(Q)
    s = _shape(Q, max(len3 + [Tq]), len3, causal, scale)
    if workspace is None:
        workspace = _workspace(mka_workspace_bytes(MKA_OP_FULL_MKA, s), Q.device)
    Kp, Vp = _p3(K), _p3(V)
    _check(lib().mka_full_attn_fwd(_ptr(Q), ctypes.byref(Kp), ctypes.byref(Vp), _ptr(G), _ptr(O),
                                   ctypes.byref(s), _ptr(workspace), workspace.numel(), _stream()),
           "mka_full_attn_fwd")
    return O


def mka_paged_fused_decode(q, Kpool, Vpool, table, seq_len, scale=1.0, n_splits=0, O=None,
                           want_lse=True, workspace=None):
    """One decode step over the fused KV cache in a paged pool [n_pages,H,P,d]; table [B,max_pages]
    int32 and seq_len [B] int32 on the device.  Returns (O [B,H,1,d], LSE [B,H] or None)."""
    _dev_check(q, Kpool, Vpool, table, seq_len, O)
    _same_dtype(q, Kpool=Kpool, Vpool=Vpool, O=O)
    if table.dtype != torch.int32 or seq_len.dtype != torch.int32:
        raise TypeError("table and seq_len must be int32")
    B, H, _, d = q.shape
    s = MkaPagedShape()
    s.B, s.H, s.d = B, H, d
    s.page_size, s.n_pages, s.max_pages = int(Kpool.shape[2]), int(Kpool.shape[0]), int(table.shape[1])
    s.n_splits, s.scale = int(n_splits), float(scale)
    if O is None:
        O = torch.empty_like(q)
    LSE = torch.empty((B, H), dtype=torch.float32, device=q.device) if want_lse else None
    if workspace is None:
        workspace = _workspace(64 * B * H * (d + 2) * 4, q.device)
    _check(lib().mka_paged_fused_decode(_ptr(q), _ptr(Kpool), _ptr(Vpool), _ptr(table), _ptr(seq_len),
                                        _ptr(O), _ptr(LSE), ctypes.byref(s), _ptr(workspace),
                                        workspace.numel(), _stream()), "mka_paged_fused_decode")
    return O, LSE


def mka_prefix_mean(X, M=None, workspace=None):
    """Causal prefix mean along the sequence axis of X [B,H,S,d] (the L2 summary of Alg. 1)."""
    _dev_check(X, M)
    B, H, S, d = X.shape
    if M is None:
        M = torch.empty_like(X)
    s = _shape(X, S, None, False, 1.0)
    if workspace is None:
        workspace = _workspace(mka_workspace_bytes(MKA_OP_PREFIX_MEAN, s), X.device)
    _check(lib().mka_prefix_mean(_ptr(X), _ptr(M), ctypes.byref(s), _ptr(workspace),
                                 workspace.numel(), _stream()), "mka_prefix_mean")
    return M
