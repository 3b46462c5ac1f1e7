"""Pins of the oracle's symbolic (full) MKA forward (paper: Alg. 1 "Symbolic MKA": one attention
per memory level, outputs mixed with the per-query gates) and of the causal prefix-mean summary
that produces the L2 memory there.  Checked against brute-force numpy / scipy evaluations, the
special cases that reduce to plain attention, and linearity of the projection."""
import numpy as np
import pytest
from scipy.special import softmax


def _problem(rng, B=1, H=2, Tq=6, S=(6, 8, 7), d=4):
    Q = rng.standard_normal((B, H, Tq, d))
    K = [rng.standard_normal((B, H, s, d)) for s in S]
    V = [rng.standard_normal((B, H, s, d)) for s in S]
    lam = softmax(rng.standard_normal((B, H, Tq, 3)), axis=-1)
    return Q, K, V, lam


@pytest.mark.parametrize("causal", [False, True])
def test_algorithm_by_brute_force(oracle, causal):
    rng = np.random.default_rng(0)
    Q, K, V, lam = _problem(rng)
    tau = 0.8
    O = oracle.full_mka_fwd(Q, K, V, lam, causal=causal, tau=tau)
    B, H, Tq, d = Q.shape
    ref = np.zeros_like(Q)
    for l in range(3):
        S = K[l].shape[2]
        s = tau * np.einsum("bhtd,bhjd->bhtj", Q, K[l])
        if causal:
            t = np.arange(Tq)[:, None]
            j = np.arange(S)[None, :]
            s = np.where(j <= t + (S - Tq), s, -np.inf)
        a = np.einsum("bhtj,bhjd->bhtd", softmax(s, axis=-1), V[l])
        ref += lam[..., l][..., None] * a
    np.testing.assert_allclose(O, ref, atol=1e-13)


def test_one_hot_gates_give_that_memory_s_attention(oracle):
    rng = np.random.default_rng(1)
    Q, K, V, _ = _problem(rng)
    for l in range(3):
        lam = np.zeros(Q.shape[:3] + (3,))
        lam[..., l] = 1.0
        O = oracle.full_mka_fwd(Q, K, V, lam, causal=True, tau=0.5)
        a, _ = oracle.attn_fwd(Q, K[l], V[l], causal=True, tau=0.5)
        np.testing.assert_allclose(O, a, atol=1e-14)


def test_equal_memories_give_plain_attention_whatever_the_gates(oracle):
    rng = np.random.default_rng(2)
    Q, K, V, lam = _problem(rng, S=(7, 7, 7))
    O = oracle.full_mka_fwd(Q, [K[0]] * 3, [V[0]] * 3, lam, causal=True, tau=0.9)
    a, _ = oracle.attn_fwd(Q, K[0], V[0], causal=True, tau=0.9)
    np.testing.assert_allclose(O, a, atol=1e-13)


def test_missing_memory_equals_zero_memory(oracle):
    # Alg. 1 sets M_3 = 0: zero keys and values give a_3 = 0, the same as leaving the level out
    rng = np.random.default_rng(3)
    Q, K, V, lam = _problem(rng)
    Z = np.zeros_like(K[2])
    O0 = oracle.full_mka_fwd(Q, [K[0], K[1], Z], [V[0], V[1], Z], lam, causal=True, tau=0.7)
    O1 = oracle.full_mka_fwd(Q, [K[0], K[1], None], [V[0], V[1], None], lam, causal=True, tau=0.7)
    np.testing.assert_allclose(O0, O1, atol=1e-15)


def test_differs_from_route_fusion_and_from_the_mixture(oracle):
    """Three functions of the same inputs: full MKA mixes outputs, the gated mixture mixes
    exponentials under one normalisation, route-fusion mixes keys / values.  A planted mix-up
    between them would pass the special cases above; this one separates them."""
    rng = np.random.default_rng(4)
    Q, K, V, lam = _problem(rng, S=(6, 6, 6))
    full = oracle.full_mka_fwd(Q, K, V, lam, causal=True, tau=1.0)
    mix, _ = oracle.mixture_fwd(Q, K, V, lam, causal=True, tau=1.0)
    fused, _ = oracle.fwd(Q, K, V, lam, causal=True, tau=1.0)
    assert np.abs(full - mix).max() > 1e-2
    assert np.abs(full - fused).max() > 1e-2


def test_prefix_mean_against_cumsum_and_by_hand(oracle):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((2, 3, 9, 4))
    M = oracle.prefix_mean(X)
    ref = np.cumsum(X, axis=2) / np.arange(1, 10)[None, None, :, None]
    np.testing.assert_allclose(M, ref, atol=1e-14)
    np.testing.assert_array_equal(M[:, :, 0], X[:, :, 0])
    hand = oracle.prefix_mean(np.array([1.0, 3.0, 8.0, 0.0]).reshape(1, 1, 4, 1))
    np.testing.assert_allclose(hand.ravel(), [1.0, 2.0, 4.0, 3.0], atol=1e-15)
    # causal: changing a later row never changes an earlier summary
    X2 = X.copy()
    X2[:, :, 5:] += 1.0
    np.testing.assert_array_equal(oracle.prefix_mean(X2)[:, :, :5], M[:, :, :5])


def test_prefix_mean_commutes_with_a_linear_projection(oracle):
    # why the L2 keys can be produced from the L1 keys: mean(X) W = mean(X W)
    rng = np.random.default_rng(6)
    X = rng.standard_normal((1, 1, 7, 5))
    W = rng.standard_normal((5, 3))
    np.testing.assert_allclose(oracle.prefix_mean(X) @ W, oracle.prefix_mean(X @ W), atol=1e-13)
