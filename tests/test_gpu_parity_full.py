"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The fp64 oracle cannot finish these sizes in seconds, so it computes sampled outputs one by
one: whole (batch, head) pairs where a head fits in seconds, otherwise single query rows (a
row t of a causal problem is a 1-row problem over slots 0..t).  Router outputs (gates, argmax)
are cheap and are compared in full."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from util import BF16_ATOL, F32_RTOL, GATE_ATOL, announce, max_abs, rel_err, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mka():
    import paper_2603_20586_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _rows_check(oracle, inp, G, O, LSE, heads, rows, tau):
    """Oracle on single rows: row t of head (b,h) sees slots 0..t."""
    worst = 0.0
    for (b, h) in heads:
        for t in rows:
            q = inp["Q"][b:b + 1, h:h + 1, t:t + 1].cpu()
            K = [k[b:b + 1, h:h + 1, :t + 1].cpu() for k in inp["K"]]
            V = [v[b:b + 1, h:h + 1, :t + 1].cpu() for v in inp["V"]]
            g = G[b:b + 1, h:h + 1, :t + 1].cpu()
            Oref, LSEref = oracle.fwd(q, K, V, g, causal=True, tau=tau)
            worst = max(worst, max_abs(O[b:b + 1, h:h + 1, t:t + 1], Oref))
            assert abs(float(LSE[b, h, t]) - float(LSEref[0, 0, 0])) <= BF16_ATOL
    return worst


def test_C2_prefill_full(mka, oracle):
    announce("C2 prefill full size")
    inp, cfg = si.config_inputs("C2", device="cuda")
    O, LSE, G, idx = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"],
                                            causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    Gref, idxref = oracle.route(inp["Q"].cpu(), inp["W_r"].cpu(), inp["b_r"].cpu())
    np.testing.assert_array_equal(idx.cpu().numpy(), idxref)  # all 131072 rows, bit-exact
    assert max_abs(G, Gref) <= GATE_ATOL
    for (b, h) in [(0, 0), (3, 15), (1, 7)]:  # whole heads
        sl = (slice(b, b + 1), slice(h, h + 1))
        Oref, LSEref = oracle.fwd(inp["Q"][sl].cpu(), [k[sl].cpu() for k in inp["K"]],
                                  [v[sl].cpu() for v in inp["V"]], Gref[sl], causal=True,
                                  tau=inp["scale"])
        assert max_abs(O[sl], Oref) <= BF16_ATOL
        assert max_abs(LSE[sl], LSEref) <= BF16_ATOL


@pytest.mark.parametrize("materialise", [None, False], ids=["library-default-route", "folded-route"])
def test_C3_long_prefill_sampled_rows(mka, oracle, materialise):
    """Both forward routes at the full C3 size: the one the library picks by itself for this shape
    (Kf, Vf materialised once, then plain attention) and the folded kernel (fusion inside the
    attention kernel's tile loads, no workspace)."""
    announce(f"C3 long prefill full size, sampled rows, materialise={materialise}")
    inp, cfg = si.config_inputs("C3", device="cuda")
    O, LSE, G, idx = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"],
                                            causal=True, scale=inp["scale"], materialise=materialise)
    torch.cuda.synchronize()
    Gref, idxref = oracle.route(inp["Q"].cpu(), inp["W_r"].cpu(), inp["b_r"].cpu())
    np.testing.assert_array_equal(idx.cpu().numpy(), idxref)
    assert max_abs(G, Gref) <= GATE_ATOL
    rows = [0, 1, 63, 64, 255, 256, 257, 4095, 4096, 8000, 8191]
    worst = _rows_check(oracle, inp, G, O, LSE, [(0, 0), (0, 31), (0, 13)], rows, inp["scale"])
    assert worst <= BF16_ATOL, worst
    # property that holds at any size: every output row is a convex combination of fused values
    assert torch.isfinite(O.float()).all()


def test_C5_forward_folded_route_sampled_heads(mka, oracle):
    """The folded forward kernel at the full C5 size (the library's default there is the
    materialised route, which the training test below runs): two whole heads."""
    announce("C5 forward, folded route, sampled heads")
    inp, cfg = si.config_inputs("C5", device="cuda")
    O, LSE, G, idx = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"],
                                            causal=True, scale=inp["scale"], materialise=False)
    torch.cuda.synchronize()
    for (b, h) in [(0, 0), (5, 9)]:
        sl = (slice(b, b + 1), slice(h, h + 1))
        Oref, LSEref, Gref, idxref = oracle.fwd_routed(
            inp["Q"][sl].cpu(), [k[sl].cpu() for k in inp["K"]], [v[sl].cpu() for v in inp["V"]],
            inp["W_r"].cpu(), inp["b_r"].cpu(), causal=True, tau=inp["scale"])
        np.testing.assert_array_equal(idx[sl].cpu().numpy(), idxref)
        assert max_abs(O[sl], Oref) <= BF16_ATOL
        assert max_abs(LSE[sl], LSEref) <= BF16_ATOL


def test_C5_training_all_heads(mka, oracle):
    """Config C5 in full: dQ, dK_l, dV_l of all 128 heads on the raw 2e-2, dW_r / db_r of the whole
    problem on the normalised 2e-2 (about a minute of oracle time on the machine's host cores)."""
    announce("C5 training full size, all heads")
    inp, cfg = si.config_inputs("C5", device="cuda")
    O, LSE, G, idx = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"],
                                            causal=True, scale=inp["scale"])
    g = mka.mka_fused_attn_bwd(inp["dO"], inp["Q"], inp["K"], inp["V"], G, O, LSE, inp["W_r"],
                               causal=True, scale=inp["scale"], stored_ds=False)
    # the alternative route stores dS for the dQ kernel instead of recomputing the scores: same
    # main kernel (bit-identical dK / dV / dW_r), its dQ is checked below as well
    dQ_rec = mka.mka_fused_attn_bwd(inp["dO"], inp["Q"], inp["K"], inp["V"], G, O, LSE, inp["W_r"],
                                    causal=True, scale=inp["scale"], stored_ds=True,
                                    grads_for=(False, False, False))["dQ"]
    torch.cuda.synchronize()
    # Router gradients of the configured problem: they sum over all 128 heads and 524 288 rows
    # (two-stage fixed-order reduction on the GPU).  The oracle runs every head, one batch entry
    # (16 heads) at a time to bound its memory, and its per-head sums are added in fp64.
    B = cfg["B"]
    dW_ref = np.zeros((cfg["d"], 3))
    db_ref = np.zeros(3)
    for b in range(B):
        sl = slice(b, b + 1)
        print(f"[case] C5 oracle backward, batch entry {b + 1}/{B}", flush=True)
        Gref, _ = oracle.route(inp["Q"][sl].cpu(), inp["W_r"].cpu(), inp["b_r"].cpu())
        ref = oracle.bwd(inp["dO"][sl].cpu(), inp["Q"][sl].cpu(), [k[sl].cpu() for k in inp["K"]],
                         [v[sl].cpu() for v in inp["V"]], Gref, inp["W_r"].cpu(), causal=True,
                         tau=inp["scale"])
        dW_ref += ref["dW_r"]
        db_ref += ref["db_r"]
        if True:  # every head's dQ / dK_l / dV_l on the raw bound while the reference is here
            assert max_abs(g["dQ"][sl], ref["dQ"]) <= BF16_ATOL
            assert max_abs(dQ_rec[sl], ref["dQ"]) <= BF16_ATOL
            for l in range(3):
                assert max_abs(g["dK"][l][sl], ref["dK"][l]) <= BF16_ATOL
                assert max_abs(g["dV"][l][sl], ref["dV"][l]) <= BF16_ATOL
        del ref
    # sums of 524 288 rows: judged on the scale-normalised error of each gradient's own reference
    eW = max_abs(g["dW_r"], dW_ref) / max(1.0, float(np.abs(dW_ref).max()))
    eb = max_abs(g["db_r"], db_ref) / max(1.0, float(np.abs(db_ref).max()))
    print(f"[case] C5 dW_r normalised error {eW:.3e} (max|ref| {np.abs(dW_ref).max():.3e}), "
          f"db_r {eb:.3e} (max|ref| {np.abs(db_ref).max():.3e})", flush=True)
    assert eW <= BF16_ATOL, eW
    assert eb <= BF16_ATOL, eb
    # the same call again gives the same bits (fixed-order sums everywhere)
    g2 = mka.mka_fused_attn_bwd(inp["dO"], inp["Q"], inp["K"], inp["V"], G, O, LSE, inp["W_r"],
                                causal=True, scale=inp["scale"], stored_ds=False)
    # ... on either route (the default workspace is the recommended route's: stored dS here)
    dQ_rec2 = mka.mka_fused_attn_bwd(inp["dO"], inp["Q"], inp["K"], inp["V"], G, O, LSE, inp["W_r"],
                                     causal=True, scale=inp["scale"],
                                     grads_for=(False, False, False))["dQ"]
    torch.cuda.synchronize()
    assert torch.equal(g2["dW_r"], g["dW_r"]) and torch.equal(g2["db_r"], g["db_r"])
    assert torch.equal(g2["dQ"], g["dQ"])
    assert torch.equal(dQ_rec2, dQ_rec)
    for l in range(3):
        assert torch.equal(g2["dK"][l], g["dK"][l]) and torch.equal(g2["dV"][l], g["dV"][l])


def test_C4_decode_full_sampled_heads(mka, oracle):
    announce("C4 decode full size: 64 steps, sampled heads checked at every step")
    cfg = si.CONFIGS["C4"]
    B, H, d, S0, steps = cfg["B"], cfg["H"], cfg["d"], cfg["S0"], cfg["steps"]
    c = si.decode_caches(B, H, d, S0, cap_extra=steps, device="cuda", seed=cfg["seed"])
    heads = [(0, 0), (15, 31), (6, 17)]
    pick = lambda x: torch.stack([x[b, h] for (b, h) in heads], 0)[None]  # noqa: E731
    Kc_o = [to_np(pick(x)).copy() for x in c["Kc"]]
    Vc_o = [to_np(pick(x)).copy() for x in c["Vc"]]
    Gc_o = to_np(pick(c["Gc"])).copy()
    len_g, len_o = list(c["len"]), list(c["len"])
    worst = 0.0
    for step in range(steps):
        q, k1, v1 = si.decode_step_inputs(B, H, d, step, device="cuda", seed=cfg["seed"])
        O, LSE, idx = mka.mka_fused_attn_decode(q, [k1, None, None], [v1, None, None], c["Kc"],
                                                c["Vc"], c["Gc"], len_g, c["W_r"], c["b_r"],
                                                scale=c["scale"])
        torch.cuda.synchronize()
        Oref, LSEref, idxref = oracle.decode(pick(q).cpu(), [pick(k1).cpu(), None, None],
                                             [pick(v1).cpu(), None, None], Kc_o, Vc_o, Gc_o, len_o,
                                             c["W_r"].cpu(), c["b_r"].cpu(), tau=c["scale"])
        assert len_g == len_o
        np.testing.assert_array_equal(pick(idx).cpu().numpy()[0], idxref[0])
        worst = max(worst, max_abs(pick(O), Oref))
        assert max_abs(pick(LSE), LSEref[:, :, 0]) <= BF16_ATOL
    assert worst <= BF16_ATOL, worst
    assert len_g == [S0 + steps, S0, S0]
    assert max_abs(pick(c["Gc"]), Gc_o) <= GATE_ATOL


def test_C1_tiny_fp32_config(mka, oracle):
    announce("C1 tiny fp32 (also in the small suite; kept here as the config list's first entry)")
    inp, cfg = si.config_inputs("C1", device="cuda")
    O, LSE, G, idx = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"],
                                            causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    Oref, LSEref, Gref, idxref = oracle.fwd_routed(
        inp["Q"].cpu(), [k.cpu() for k in inp["K"]], [v.cpu() for v in inp["V"]],
        inp["W_r"].cpu(), inp["b_r"].cpu(), causal=True, tau=inp["scale"])
    assert rel_err(O, Oref) <= F32_RTOL
    np.testing.assert_array_equal(idx.cpu().numpy(), idxref)
