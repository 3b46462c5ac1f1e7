"""Pins of the oracle's routing variants (paper: section "Routing Mechanism Ablation", table
"Routing mechanism ablation": learned soft routing, fixed lam = 1/3, hard top-2, hard top-1).
The paper names the variants without formulas; the reading (hard top-k keeps the k largest
logits and renormalises their soft gates, ties to the lower level) is pinned here by values
worked out by hand, by the properties that define it, by scipy's softmax on the kept levels, and
end to end: top-1 routed attention is plain attention over the per-slot selected memory."""
import numpy as np
import pytest
from scipy.special import softmax

SOFT, FIXED, TOP2, TOP1 = 0, 1, 2, 3


def _logit_problem(logits):
    """Q, W_r such that row t has exactly the logits[t] (Q = unit vectors, W_r = the logits)."""
    logits = np.asarray(logits, dtype=np.float64)
    n = logits.shape[0]
    Q = np.eye(n)[None, None]            # [1,1,n,n]
    return Q, logits.copy()              # W_r [n,3]


def test_hand_worked_gates(oracle):
    # logits (ln 4, ln 2, ln 1): soft = (4/7, 2/7, 1/7); top-2 = (2/3, 1/3, 0); top-1 = (1, 0, 0)
    # logits (0, ln 3, ln 3 + ln 2): soft = (1, 3, 6)/10; top-2 = (0, 1/3, 2/3); top-1 = (0, 0, 1)
    L = [[np.log(4.0), np.log(2.0), 0.0], [0.0, np.log(3.0), np.log(6.0)]]
    Q, W = _logit_problem(L)
    want = {SOFT: [[4 / 7, 2 / 7, 1 / 7], [0.1, 0.3, 0.6]],
            FIXED: [[1 / 3] * 3, [1 / 3] * 3],
            TOP2: [[2 / 3, 1 / 3, 0.0], [0.0, 1 / 3, 2 / 3]],
            TOP1: [[1.0, 0.0, 0.0], [0.0, 0.0, 1.0]]}
    for mode, w in want.items():
        G, idx = oracle.route_variant(Q, W, None, mode)
        np.testing.assert_allclose(G[0, 0], np.array(w), rtol=0, atol=1e-15)
        np.testing.assert_array_equal(idx[0, 0], [0, 2])


def test_ties_go_to_the_lower_level(oracle):
    L = [[0.5, 0.5, 0.5], [1.0, 2.0, 2.0], [3.0, 1.0, 1.0]]
    Q, W = _logit_problem(L)
    G1, idx = oracle.route_variant(Q, W, None, TOP1)
    G2, _ = oracle.route_variant(Q, W, None, TOP2)
    np.testing.assert_array_equal(idx[0, 0], [0, 1, 0])
    np.testing.assert_array_equal(G1[0, 0], [[1, 0, 0], [0, 1, 0], [1, 0, 0]])
    # all equal: levels 1 and 2 kept; equal maxima both kept; equal minima: the higher one dropped
    e = np.exp(-2.0)
    np.testing.assert_allclose(G2[0, 0], [[0.5, 0.5, 0.0], [0.0, 0.5, 0.5],
                                          [1 / (1 + e), e / (1 + e), 0.0]], atol=1e-15)


def test_defining_properties_on_random_logits(oracle):
    rng = np.random.default_rng(5)
    B, H, T, d = 2, 3, 17, 8
    Q = rng.standard_normal((B, H, T, d))
    W = rng.standard_normal((d, 3))
    b = rng.standard_normal(3)
    logits = Q @ W + b
    soft, idx = oracle.route(Q, W, b)            # pinned elsewhere
    for mode in (SOFT, FIXED, TOP2, TOP1):
        G, idx_m = oracle.route_variant(Q, W, b, mode)
        np.testing.assert_array_equal(idx_m, idx)          # the argmax does not depend on the mode
        np.testing.assert_allclose(G.sum(-1), 1.0, atol=1e-14)
        assert (G >= 0).all()
    np.testing.assert_allclose(oracle.route_variant(Q, W, b, SOFT)[0], soft, atol=1e-15)
    np.testing.assert_array_equal(oracle.route_variant(Q, W, b, FIXED)[0], np.full(soft.shape, 1 / 3))
    G1 = oracle.route_variant(Q, W, b, TOP1)[0]
    np.testing.assert_array_equal(G1, np.eye(3)[logits.argmax(-1)])
    # top-2: exactly one zero, at the smallest logit; the kept pair is the library softmax of
    # the two kept logits (= the soft gates in the same ratio)
    G2 = oracle.route_variant(Q, W, b, TOP2)[0]
    drop = logits.argmin(-1)
    assert ((G2 == 0).sum(-1) == 1).all()
    np.testing.assert_array_equal(np.take_along_axis(G2, drop[..., None], -1)[..., 0], 0.0)
    masked = np.where(np.arange(3) == drop[..., None], -np.inf, logits)
    np.testing.assert_allclose(G2, softmax(masked, axis=-1), atol=1e-14)


def test_a_level_that_is_never_chosen_makes_top2_equal_soft(oracle):
    rng = np.random.default_rng(6)
    Q = rng.standard_normal((1, 2, 9, 4))
    W = rng.standard_normal((4, 3))
    b = np.array([0.0, -800.0, 0.0])             # exp(-800) underflows: level 2 has soft gate 0
    soft = oracle.route_variant(Q, W, b, SOFT)[0]
    top2 = oracle.route_variant(Q, W, b, TOP2)[0]
    np.testing.assert_array_equal(soft[..., 1], 0.0)
    np.testing.assert_allclose(top2, soft, atol=1e-15)


def test_rows_below_the_new_slots_are_kept(oracle):
    rng = np.random.default_rng(7)
    Q = rng.standard_normal((1, 1, 3, 4))
    W = rng.standard_normal((4, 3))
    prev = rng.random((1, 1, 8, 3))
    G, _ = oracle.route_variant(Q, W, None, TOP1, S=8, G_prev=prev)
    np.testing.assert_array_equal(G[:, :, :5], prev[:, :, :5])
    np.testing.assert_array_equal(G[:, :, 5:].sum(-1), 1.0)


@pytest.mark.parametrize("causal", [True, False])
def test_top1_routed_attention_is_attention_over_the_selected_memory(oracle, causal):
    """End to end: with hard top-1 gates the fused stream of Alg. 2 step 6 is, slot by slot, the
    chosen level's row, so the route-fused forward equals plain attention over that stream."""
    rng = np.random.default_rng(8)
    B, H, T, d = 1, 2, 11, 4
    Q = rng.standard_normal((B, H, T, d))
    K = [rng.standard_normal((B, H, T, d)) for _ in range(3)]
    V = [rng.standard_normal((B, H, T, d)) for _ in range(3)]
    W = rng.standard_normal((d, 3)) * 3
    G, idx = oracle.route_variant(Q, W, None, TOP1)
    O, LSE = oracle.fwd(Q, K, V, G, causal=causal, tau=0.6)
    sel = idx[..., None]                                   # [B,H,T,1]
    Ks = np.choose(sel, [K[0], K[1], K[2]])
    Vs = np.choose(sel, [V[0], V[1], V[2]])
    Oref, LSEref = oracle.attn_fwd(Q, Ks, Vs, causal=causal, tau=0.6)
    np.testing.assert_allclose(O, Oref, atol=1e-13)
    np.testing.assert_allclose(LSE, LSEref, atol=1e-13)


# ------------------------------------------------------------------ decode with a routing variant
def _decode_problem(rng, B, H, d, S0, cap, lens=None):
    Kc = [np.ascontiguousarray(rng.standard_normal((B, H, cap, d))) for _ in range(3)]
    Vc = [np.ascontiguousarray(rng.standard_normal((B, H, cap, d))) for _ in range(3)]
    q = rng.standard_normal((B, H, 1, d))
    kn = [rng.standard_normal((B, H, 1, d)) for _ in range(3)]
    vn = [rng.standard_normal((B, H, 1, d)) for _ in range(3)]
    W = rng.standard_normal((d, 3)) * 2
    b = rng.standard_normal(3)
    return q, kn, vn, Kc, Vc, W, b, (list(lens) if lens else [S0, S0, S0])


def test_decode_variant_soft_is_the_decode_oracle(oracle):
    """The composition (append, variant gate, forward of one row) against the stand-alone decode
    oracle, which is pinned on its own: soft routing must give the same step, also with a level
    that lags behind and gets no entry."""
    import copy
    rng = np.random.default_rng(21)
    for lens, drop in (([5, 5, 5], None), ([5, 3, 5], 1)):
        q, kn, vn, Kc, Vc, W, b, l1 = _decode_problem(rng, 2, 2, 8, 5, 9, lens)
        if drop is not None:
            kn[drop] = None
            vn[drop] = None
        Gc = rng.random((2, 2, 9, 3))
        Gc /= Gc.sum(-1, keepdims=True)
        Kc2, Vc2, Gc2, l2 = copy.deepcopy(Kc), copy.deepcopy(Vc), Gc.copy(), list(l1)
        O1, L1, i1 = oracle.decode(q, kn, vn, Kc, Vc, Gc, l1, W, b, tau=0.3)
        O2, L2, i2 = oracle.decode_variant(q, kn, vn, Kc2, Vc2, Gc2, l2, W, b, mode=SOFT, tau=0.3)
        np.testing.assert_allclose(O2, O1, atol=1e-14)
        np.testing.assert_allclose(L2, L1, atol=1e-14)
        np.testing.assert_array_equal(i2, i1)
        np.testing.assert_array_equal(Gc2, Gc)
        assert l1 == l2
        for a, c in zip(Kc + Vc, Kc2 + Vc2):
            np.testing.assert_array_equal(a, c)


def test_decode_top1_is_attention_over_the_selected_rows(oracle):
    """With one-hot gates in the cache and a top-1 gate for the new slot, the step is plain
    attention of q over the stream that holds, slot by slot, the selected level's row."""
    rng = np.random.default_rng(22)
    B, H, d, S0, cap = 1, 3, 8, 6, 8
    q, kn, vn, Kc, Vc, W, b, lens = _decode_problem(rng, B, H, d, S0, cap)
    sel_old = rng.integers(0, 3, size=(B, H, S0))
    Gc = np.zeros((B, H, cap, 3))
    Gc[:, :, :S0] = np.eye(3)[sel_old]
    O, LSE, idx = oracle.decode_variant(q, kn, vn, Kc, Vc, Gc, lens, W, b, mode=TOP1, tau=0.7)
    logits = q[:, :, 0] @ W + b
    np.testing.assert_array_equal(idx, logits.argmax(-1))
    np.testing.assert_array_equal(Gc[:, :, S0], np.eye(3)[idx])       # the new slot's gate
    sel = np.concatenate([sel_old, idx[..., None]], -1)[..., None]     # [B,H,S0+1,1]
    S = S0 + 1
    Ks = np.choose(sel, [a[:, :, :S] for a in Kc])
    Vs = np.choose(sel, [a[:, :, :S] for a in Vc])
    Oref, Lref = oracle.attn_fwd(q, Ks, Vs, causal=False, tau=0.7)
    np.testing.assert_allclose(O, Oref, atol=1e-13)
    np.testing.assert_allclose(LSE, Lref, atol=1e-13)
    assert lens == [S, S, S]


def test_decode_top2_gate_of_the_new_slot_by_hand(oracle):
    # one head, d = 3, W = I: the logits are q.  q = (ln 4, ln 2, 0) -> top-2 gate (2/3, 1/3, 0)
    q = np.array([np.log(4.0), np.log(2.0), 0.0]).reshape(1, 1, 1, 3)
    Kc = [np.zeros((1, 1, 2, 3)) for _ in range(3)]
    Vc = [np.zeros((1, 1, 2, 3)) for _ in range(3)]
    Gc = np.zeros((1, 1, 2, 3))
    one = [np.ones((1, 1, 1, 3)) * (l + 1) for l in range(3)]
    lens = [0, 0, 0]
    O, LSE, idx = oracle.decode_variant(q, one, one, Kc, Vc, Gc, lens, np.eye(3), None, mode=TOP2)
    np.testing.assert_allclose(Gc[0, 0, 0], [2 / 3, 1 / 3, 0.0], atol=1e-15)
    # a single slot: O is its fused value row = 2/3 * 1 + 1/3 * 2 = 4/3 in every component
    np.testing.assert_allclose(O[0, 0, 0], 4 / 3, atol=1e-14)
    assert idx[0, 0] == 0 and lens == [1, 1, 1]
