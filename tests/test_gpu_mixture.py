"""GPU parity of the gated-mixture attention (section "Recursive MKA with Online Softmax") against
the fp64 oracle, through the C ABI: ragged shapes over several tiles and all three levels, levels
of unequal length, absent levels, zero gates, no gates (plain attention), and the full-size
prefill shape on sampled heads."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from util import BF16_ATOL, announce, cpu_list, max_abs, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mka():
    import paper_2603_20586_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _inputs(B, H, Tq, S3, d, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    def rnd(*shape):
        return torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    Q = rnd(B, H, Tq, d)
    K = [None if s is None else rnd(B, H, s, d) for s in S3]
    V = [None if s is None else rnd(B, H, s, d) for s in S3]
    G = torch.softmax(torch.randn((B, H, Tq, 3), generator=gen, device="cuda") * 2.0, -1)
    return Q, K, V, G


def _check(mka, oracle, Q, K, V, G, causal, scale):
    O, LSE = mka.mka_mixture_attn_fwd(Q, K, V, G, causal=causal, scale=scale)
    torch.cuda.synchronize()
    Oref, Lref = oracle.mixture_fwd(Q.cpu(), cpu_list(K), cpu_list(V),
                                    None if G is None else G.cpu(), causal=causal, tau=scale)
    eo = max_abs(O, Oref)
    fin = np.isfinite(Lref)
    el = float(np.max(np.abs(to_np(LSE)[fin] - Lref[fin]))) if fin.any() else 0.0
    assert eo <= BF16_ATOL and el <= BF16_ATOL, (eo, el)
    assert np.array_equal(np.isfinite(to_np(LSE)), fin)
    return eo, el


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("Tq,S3,causal", [
    (300, (300, 300, 300), True),     # several query tiles, 15 stream tiles, ragged tails
    (130, (333, 130, 200), True),     # unequal lengths, each with its own diagonal
    (200, (260, 70, 1), False),       # non-causal, a one-slot memory
    (257, (257, None, 300), True),    # a memory absent
    (64, (64, None, None), True),     # one memory, one tile
    (520, (520, 600, None), True),    # three query tiles: a heavy / light pair and the middle one
    (1, (1, 1, 1), True), (1, (70, 3, 129), False)])
def test_mixture_shapes(mka, oracle, d, Tq, S3, causal):
    announce(f"mixture d={d} Tq={Tq} S={S3} causal={causal}")
    Q, K, V, G = _inputs(2, 2, Tq, S3, d, seed=31)
    _check(mka, oracle, Q, K, V, G, causal, 1.0 / np.sqrt(d))


@pytest.mark.parametrize("d", [128, 64])
def test_mixture_reference_exponent_moves_along_the_stream(mka, oracle, d):
    """Keys that grow with the slot index in every memory, so that the reference exponent of the
    lazy max-shift moves in many units of the stream, not just in the first (the kernel's rare
    path), and drops back at each level change relative to the new level's scores."""
    announce(f"mixture growing keys d={d}")
    Q, K, V, G = _inputs(2, 2, 260, (500, 333, 400), d, seed=37)
    K = [(k.float() * torch.linspace(1.0, 12.0, k.shape[2], device="cuda").view(1, 1, -1, 1)).to(torch.bfloat16)
         for k in K]
    V = [(v.float() * 0.25).to(torch.bfloat16) for v in V]   # |O| <= 1: the output's own rounding
    for causal in (True, False):
        O, LSE = mka.mka_mixture_attn_fwd(Q, K, V, G, causal=causal, scale=1.0 / np.sqrt(d))
        torch.cuda.synchronize()
        Oref, Lref = oracle.mixture_fwd(Q.cpu(), cpu_list(K), cpu_list(V), G.cpu(), causal=causal,
                                        tau=1.0 / np.sqrt(d))
        assert max_abs(O, Oref) <= BF16_ATOL, max_abs(O, Oref)
        assert float(np.max(np.abs(to_np(LSE) - Lref))) <= BF16_ATOL


def test_mixture_without_gates_is_attention_over_the_concatenation(mka, oracle):
    announce("mixture no gates")
    Q, K, V, _ = _inputs(1, 3, 190, (190, 200, 250), 128, seed=32)
    _check(mka, oracle, Q, K, V, None, True, 0.09)


def test_mixture_zero_gates_switch_levels_off_per_row(mka, oracle):
    announce("mixture zero gates")
    Q, K, V, G = _inputs(1, 2, 150, (150, 150, 150), 128, seed=33)
    G[:, :, ::2, 0] = 0.0          # even rows never look at memory 1
    G[:, :, 5, :] = 0.0            # a row that sees nothing: O = 0, LSE = -inf
    O, LSE = mka.mka_mixture_attn_fwd(Q, K, V, G, causal=True, scale=0.1)
    torch.cuda.synchronize()
    assert float(O[:, :, 5].float().abs().max()) == 0.0
    assert bool(torch.isinf(LSE[:, :, 5]).all())
    _check(mka, oracle, Q, K, V, G, True, 0.1)


def test_mixture_one_memory_matches_the_route_fused_forward_with_one_hot_gates(mka):
    """Two different kernels of the library on a case where the two formulations coincide."""
    announce("mixture vs route-fused, one memory")
    inp = si.prefill_inputs(1, 2, 260, 260, 128, dtype="bf16", seed=34, device="cuda")
    G = torch.zeros((1, 2, 260, 3), device="cuda")
    G[..., 0] = 1.0
    O1, L1, _, _ = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], None, None, G=G,
                                          causal=True, scale=inp["scale"])
    O2, L2 = mka.mka_mixture_attn_fwd(inp["Q"], [inp["K"][0], None, None], [inp["V"][0], None, None],
                                      None, causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    assert float((O1.float() - O2.float()).abs().max()) <= 1e-2
    assert float((L1 - L2).abs().max()) <= 1e-2


def test_mixture_full_prefill_shape_sampled_heads(mka, oracle):
    """C2 shape (B4 H16 T2048 d128), all three memories: every head runs, 3 are compared."""
    announce("mixture C2 shape")
    inp, cfg = si.config_inputs("C2", device="cuda")
    G, _ = mka.mka_route(inp["Q"], inp["W_r"] * 30.0, inp["b_r"], want_idx=False)
    O, LSE = mka.mka_mixture_attn_fwd(inp["Q"], inp["K"], inp["V"], G, causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    for (b, h) in [(0, 0), (2, 7), (3, 15)]:
        sl = (slice(b, b + 1), slice(h, h + 1))
        Oref, Lref = oracle.mixture_fwd(inp["Q"][sl].cpu(), [k[sl].cpu() for k in inp["K"]],
                                        [v[sl].cpu() for v in inp["V"]], G[sl].cpu(),
                                        causal=True, tau=inp["scale"])
        assert max_abs(O[sl], Oref) <= BF16_ATOL
        assert max_abs(LSE[sl], Lref) <= BF16_ATOL


def _one_row(x, b, h, lo, hi):
    return None if x is None else x[b:b + 1, h:h + 1, lo:hi].cpu()


def test_mixture_long_prefill_shape_sampled_rows(mka, oracle):
    """C3 shape (B1 H32 T8192 d128), three memories of 8192 slots, the size bench.py times: the
    oracle computes sampled query rows one by one (row t of a causal problem is a one-row
    problem over slots 0..t of every memory)."""
    announce("mixture C3 shape, sampled rows")
    inp, cfg = si.config_inputs("C3", device="cuda")
    G, _ = mka.mka_route(inp["Q"], inp["W_r"] * 30.0, inp["b_r"], want_idx=False)
    O, LSE = mka.mka_mixture_attn_fwd(inp["Q"], inp["K"], inp["V"], G, causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    worst = 0.0
    for (b, h) in [(0, 0), (0, 31), (0, 13)]:
        for t in [0, 1, 63, 64, 255, 256, 257, 4095, 4096, 8000, 8191]:
            Oref, Lref = oracle.mixture_fwd(
                _one_row(inp["Q"], b, h, t, t + 1), [_one_row(k, b, h, 0, t + 1) for k in inp["K"]],
                [_one_row(v, b, h, 0, t + 1) for v in inp["V"]], _one_row(G, b, h, t, t + 1),
                causal=True, tau=inp["scale"])
            worst = max(worst, max_abs(O[b:b + 1, h:h + 1, t:t + 1], Oref))
            assert abs(float(LSE[b, h, t]) - float(Lref[0, 0, 0])) <= BF16_ATOL
    assert worst <= BF16_ATOL, worst
    assert torch.isfinite(O.float()).all()


# ------------------------------------------------------------------ materialised route-fusion
@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("S,len3", [(300, None), (257, [257, 100, 0]), (1, None)])
def test_fuse_kv_against_the_oracle(mka, oracle, d, S, len3):
    announce(f"fuse_kv d={d} S={S} len={len3}")
    inp = si.prefill_inputs(2, 2, S, S, d, dtype="bf16", seed=41, device="cuda")
    G = torch.softmax(torch.randn((2, 2, S, 3), device="cuda") * 2, -1)
    Kf, Vf = mka.mka_fuse_kv(inp["K"], inp["V"], G, len3=len3)
    torch.cuda.synchronize()
    Kr = oracle.fuse(cpu_list(inp["K"]), G.cpu(), len3=len3)
    Vr = oracle.fuse(cpu_list(inp["V"]), G.cpu(), len3=len3)
    # one bf16 rounding of a value of magnitude <= ~5
    assert max_abs(Kf, Kr) <= BF16_ATOL and max_abs(Vf, Vr) <= BF16_ATOL


@pytest.mark.parametrize("mode", [2, 3])   # hard top-2, hard top-1: gates with exact zeros
def test_fuse_kv_with_hard_gates(mka, oracle, mode):
    """Zero-gated levels are not loaded by the kernel; the oracle multiplies by the zero.  With
    top-1 gates the fused row is the selected level's row, bit for bit."""
    announce(f"fuse_kv hard gates mode={mode}")
    S, d = 300, 128
    inp = si.prefill_inputs(2, 2, S, S, d, dtype="bf16", seed=43, device="cuda")
    G, idx = mka.mka_route_variant(inp["Q"], inp["W_r"] * 20.0, inp["b_r"], mode=mode)
    assert int((G == 0).sum()) == 2 * 2 * S * (mode - 1)   # one (top-2) or two (top-1) zeros per slot
    Kf, Vf = mka.mka_fuse_kv(inp["K"], inp["V"], G)
    torch.cuda.synchronize()
    Kr = oracle.fuse(cpu_list(inp["K"]), G.cpu())
    Vr = oracle.fuse(cpu_list(inp["V"]), G.cpu())
    assert max_abs(Kf, Kr) <= BF16_ATOL and max_abs(Vf, Vr) <= BF16_ATOL
    if mode == 3:
        sel = idx.long()[..., None, None].expand(-1, -1, -1, 1, d)      # [B,H,S,1,d]
        Ks = torch.stack(inp["K"], 3).gather(3, sel)[:, :, :, 0]
        Vs = torch.stack(inp["V"], 3).gather(3, sel)[:, :, :, 0]
        assert torch.equal(Kf, Ks) and torch.equal(Vf, Vs)


def test_prefuse_then_plain_attention_equals_the_folded_forward(mka, oracle):
    """The materialised alternative to in-kernel fusion: same fused bf16 stream, so the two GPU
    paths agree far inside the bound, and both match the oracle's route-fused forward."""
    announce("prefuse + plain attention vs folded forward")
    inp = si.prefill_inputs(1, 3, 400, 400, 128, dtype="bf16", seed=42, device="cuda")
    O1, L1, G, _ = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"] * 20.0, inp["b_r"],
                                          causal=True, scale=inp["scale"])
    Kf, Vf = mka.mka_fuse_kv(inp["K"], inp["V"], G)
    O2, L2 = mka.mka_mixture_attn_fwd(inp["Q"], [Kf, None, None], [Vf, None, None], None,
                                      causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    assert float((O1.float() - O2.float()).abs().max()) <= 5e-3
    assert float((L1 - L2).abs().max()) <= 5e-3
    Oref, Lref = oracle.fwd(inp["Q"].cpu(), cpu_list(inp["K"]), cpu_list(inp["V"]), G.cpu(),
                            causal=True, tau=inp["scale"])[:2]
    assert max_abs(O2, Oref) <= BF16_ATOL and max_abs(L2, Lref) <= BF16_ATOL
