"""Seeded synthetic inputs for the FastMKA hot path (shared by tests, smoke and bench).

This module holds no arithmetic of the method: it only draws random tensors of
the shapes, dtypes and distributions of the benchmark configurations and hands
the SAME bytes to whichever implementation is under test.  It stands in for
"one attention layer of a LLaMA-7B / Qwen-7B-shaped model at that context
length"; no dataset or trained weight is involved.

Recipe (every config): draw in fp32 from a torch.Generator on the target device
seeded with the config's seed, in the order Q, K1, V1, K2, V2, K3, V3, W_r, [dO],
then round to the config dtype.  Q, K_l, V_l, dO ~ N(0,1); W_r ~ N(0, 0.02^2)
(0.02 is the standard deviation); b_r = 0.  The tiny fp32 config multiplies Q by
1/sqrt(d) after drawing and uses softmax scale 1; the others leave Q alone and
use scale 1/sqrt(d).
"""
from __future__ import annotations

import math

import torch

# name -> shape of the benchmark configurations (one GPU each)
CONFIGS = {
    "C1": dict(kind="prefill", dtype="f32", B=1, H=2, d=64, Tq=128, S=128, causal=True, seed=0,
               q_prescale=True),
    "C2": dict(kind="prefill", dtype="bf16", B=4, H=16, d=128, Tq=2048, S=2048, causal=True,
               seed=1, q_prescale=False),
    "C3": dict(kind="prefill", dtype="bf16", B=1, H=32, d=128, Tq=8192, S=8192, causal=True,
               seed=2, q_prescale=False),
    "C4": dict(kind="decode", dtype="bf16", B=16, H=32, d=128, S0=32768, steps=64, seed=3),
    "C5": dict(kind="train", dtype="bf16", B=8, H=16, d=128, Tq=4096, S=4096, causal=True, seed=4,
               q_prescale=False),
}

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def torch_dtype(name: str) -> torch.dtype:
    return _TORCH_DTYPE[name]


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, g, device, dtype, std=1.0):
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(dtype).contiguous()


def prefill_inputs(B, H, Tq, S, d, dtype="bf16", seed=0, device="cpu", q_prescale=False,
                   with_dO=False, **_unused):
    """Inputs of a prefill / training call.  Returns a dict of tensors on `device`:
    Q [B,H,Tq,d]; K, V lists of three [B,H,S,d]; W_r [d,3] fp32; b_r [3] fp32 zeros;
    scale (python float); optionally dO [B,H,Tq,d]."""
    dt = torch_dtype(dtype)
    g = _gen(seed, device)
    Q32 = torch.randn((B, H, Tq, d), generator=g, device=device, dtype=torch.float32)
    if q_prescale:
        Q32 = Q32 * (1.0 / math.sqrt(d))
    Q = Q32.to(dt).contiguous()
    K, V = [], []
    for _ in range(3):
        K.append(_normal((B, H, S, d), g, device, dt))
        V.append(_normal((B, H, S, d), g, device, dt))
    W_r = _normal((d, 3), g, device, torch.float32, std=0.02)
    out = dict(Q=Q, K=K, V=V, W_r=W_r, b_r=torch.zeros(3, device=device, dtype=torch.float32),
               scale=(1.0 if q_prescale else 1.0 / math.sqrt(d)))
    if with_dO:
        out["dO"] = _normal((B, H, Tq, d), g, device, dt)
    return out


def config_inputs(name: str, device="cpu", **override):
    """Inputs for a named prefill/train configuration (C1, C2, C3, C5)."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    assert cfg["kind"] in ("prefill", "train")
    return prefill_inputs(device=device, with_dO=(cfg["kind"] == "train"), **cfg), cfg


def decode_caches(B, H, d, S0, cap_extra, dtype="bf16", seed=3, device="cpu", **_unused):
    """Pre-filled caches of a decode run: Kc, Vc lists of three [B,H,cap_l,d] with the first S0
    slots drawn N(0,1) (level 1 has room for `cap_extra` appended slots, levels 2 and 3 do not),
    and a gate cache Gc [B,H,S0+cap_extra,3] fp32 whose first S0 rows are softmax(z),
    z ~ N(0, (0.02*sqrt(d))^2) — the distribution the router's logits have for N(0,1) queries,
    standing in for the gates that the (absent) past queries would have produced."""
    dt = torch_dtype(dtype)
    g = _gen(seed, device)
    Kc, Vc = [], []
    for lvl in range(3):
        cap = S0 + (cap_extra if lvl == 0 else 0)
        k = torch.zeros((B, H, cap, d), device=device, dtype=dt)
        v = torch.zeros((B, H, cap, d), device=device, dtype=dt)
        # drawn per (level, tensor) in chunks over the batch to bound the fp32 temporary
        for b in range(B):
            k[b, :, :S0] = torch.randn((H, S0, d), generator=g, device=device,
                                       dtype=torch.float32).to(dt)
            v[b, :, :S0] = torch.randn((H, S0, d), generator=g, device=device,
                                       dtype=torch.float32).to(dt)
        Kc.append(k)
        Vc.append(v)
    z = torch.randn((B, H, S0, 3), generator=g, device=device, dtype=torch.float32) * (
        0.02 * math.sqrt(d))
    Gc = torch.zeros((B, H, S0 + cap_extra, 3), device=device, dtype=torch.float32)
    Gc[:, :, :S0] = torch.softmax(z, dim=-1)
    W_r = _normal((d, 3), g, device, torch.float32, std=0.02)
    return dict(Kc=Kc, Vc=Vc, Gc=Gc, W_r=W_r,
                b_r=torch.zeros(3, device=device, dtype=torch.float32),
                len=[S0, S0, S0], scale=1.0 / math.sqrt(d))


def decode_step_inputs(B, H, d, step, dtype="bf16", seed=3, device="cpu"):
    """The new token of decode step `step`: q, k1_new, v1_new [B,H,1,d] ~ N(0,1)."""
    dt = torch_dtype(dtype)
    g = _gen(seed * 1000003 + 17 + step, device)
    return tuple(_normal((B, H, 1, d), g, device, dt) for _ in range(3))
