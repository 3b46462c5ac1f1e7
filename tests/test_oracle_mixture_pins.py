"""Pins of the oracle's gated-mixture attention (paper: section "Theoretical Formulation:
Recursive MKA with Online Softmax").  Each test checks the oracle against something it did not
compute itself: a brute-force numpy evaluation of the section's first equation, the section's
max-shift recursion over the levels written out here, softmax attention over the concatenated
memories (with log-gate biases), and the special cases that reduce to one memory."""
import numpy as np
import pytest


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _problem(rng, B=1, H=2, Tq=5, S=(5, 7, 6), d=4):
    Q = _rand(rng, B, H, Tq, d)
    K = [_rand(rng, B, H, s, d) for s in S]
    V = [_rand(rng, B, H, s, d) for s in S]
    g = _rand(rng, B, H, Tq, 3)
    lam = np.exp(g) / np.exp(g).sum(-1, keepdims=True)
    return Q, K, V, lam


def _mask(Tq, S, causal):
    t = np.arange(Tq)[:, None]
    j = np.arange(S)[None, :]
    return (j <= t + (S - Tq)) if causal else np.ones((Tq, S), bool)


@pytest.mark.parametrize("causal", [False, True])
def test_first_equation_by_brute_force(oracle, causal):
    rng = np.random.default_rng(0)
    Q, K, V, lam = _problem(rng)
    tau = 0.7
    O, LSE = oracle.mixture_fwd(Q, K, V, lam, causal=causal, tau=tau)
    B, H, Tq, d = Q.shape
    for b in range(B):
        for h in range(H):
            num = np.zeros((Tq, d))
            den = np.zeros(Tq)
            for l in range(3):
                e = np.exp(tau * Q[b, h] @ K[l][b, h].T) * _mask(Tq, K[l].shape[2], causal)
                num += lam[b, h, :, l:l + 1] * (e @ V[l][b, h])
                den += lam[b, h, :, l] * e.sum(-1)
            np.testing.assert_allclose(O[b, h], num / den[:, None], rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(LSE[b, h], np.log(den), rtol=1e-12, atol=1e-13)


def test_max_shift_recursion_over_levels(oracle):
    """mu, z, alpha of the section's max-shift recursion, one level at a time."""
    rng = np.random.default_rng(1)
    Q, K, V, lam = _problem(rng, Tq=4, S=(6, 4, 9), d=3)
    Q = Q * 30.0  # exponents far outside exp()'s comfortable range without the shift
    O, _ = oracle.mixture_fwd(Q, K, V, lam, causal=False, tau=1.0)
    q, la = Q[0, 0], lam[0, 0]
    mu = np.full(4, -np.inf)
    z = np.zeros(4)
    alpha = np.zeros((4, 3))
    for l in range(3):
        s = q @ K[l][0, 0].T
        mu_new = np.maximum(mu, s.max(-1))
        sl = np.exp(s - mu_new[:, None])
        r = np.exp(mu - mu_new)
        z = z * r + la[:, l] * sl.sum(-1)
        alpha = alpha * r[:, None] + la[:, l:l + 1] * (sl @ V[l][0, 0])
        mu = mu_new
    np.testing.assert_allclose(O[0, 0], alpha / z[:, None], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_equals_softmax_over_concatenation_with_log_gate_bias(oracle, causal):
    """The mixture is softmax attention over [K1;K2;K3] with log lam_l[t] added to the scores of
    level l: checked with the oracle-independent numpy softmax."""
    rng = np.random.default_rng(2)
    Q, K, V, lam = _problem(rng, Tq=6, S=(6, 8, 6), d=5)
    O, _ = oracle.mixture_fwd(Q, K, V, lam, causal=causal, tau=0.5)
    for h in range(2):
        s = np.concatenate([0.5 * Q[0, h] @ K[l][0, h].T + np.log(lam[0, h, :, l:l + 1])
                            for l in range(3)], -1)
        msk = np.concatenate([_mask(6, K[l].shape[2], causal) for l in range(3)], -1)
        s = np.where(msk, s, -np.inf)
        p = np.exp(s - s.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        ref = p @ np.concatenate([V[l][0, h] for l in range(3)], 0)
        np.testing.assert_allclose(O[0, h], ref, rtol=1e-12, atol=1e-13)


def test_one_hot_gate_is_attention_over_that_memory(oracle):
    rng = np.random.default_rng(3)
    Q, K, V, _ = _problem(rng, Tq=7, S=(7, 9, 8), d=4)
    for l in range(3):
        lam = np.zeros((1, 2, 7, 3))
        lam[..., l] = 1.0
        O, LSE = oracle.mixture_fwd(Q, K, V, lam, causal=True, tau=0.3)
        Oref, Lref = oracle.attn_fwd(Q, K[l], V[l], causal=True, tau=0.3)
        np.testing.assert_allclose(O, Oref, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(LSE, Lref, rtol=1e-12, atol=1e-13)


def test_equal_memories_do_not_depend_on_the_gate(oracle):
    rng = np.random.default_rng(4)
    Q, K, V, lam = _problem(rng, Tq=5, S=(6, 6, 6), d=4)
    K = [K[0]] * 3
    V = [V[0]] * 3
    O, LSE = oracle.mixture_fwd(Q, K, V, lam, causal=True, tau=1.0)
    Oref, Lref = oracle.attn_fwd(Q, K[0], V[0], causal=True, tau=1.0)
    np.testing.assert_allclose(O, Oref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(LSE, Lref, rtol=1e-12, atol=1e-13)  # gates sum to one


def test_gate_scale_invariance_absent_level_and_no_gate(oracle):
    rng = np.random.default_rng(5)
    Q, K, V, lam = _problem(rng, Tq=4, S=(4, 5, 6), d=3)
    O1, L1 = oracle.mixture_fwd(Q, K, V, lam, causal=False, tau=1.0)
    O2, L2 = oracle.mixture_fwd(Q, K, V, 3.0 * lam, causal=False, tau=1.0)
    np.testing.assert_allclose(O1, O2, rtol=1e-12, atol=1e-13)       # the quotient is scale free
    np.testing.assert_allclose(L2 - L1, np.log(3.0), rtol=1e-12)
    # a level with a zero gate everywhere == that level absent
    lam0 = lam.copy()
    lam0[..., 2] = 0.0
    Oa, La = oracle.mixture_fwd(Q, K, V, lam0, causal=False, tau=1.0)
    Ob, Lb = oracle.mixture_fwd(Q, [K[0], K[1], None], [V[0], V[1], None], lam0, causal=False, tau=1.0)
    np.testing.assert_allclose(Oa, Ob, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(La, Lb, rtol=1e-13, atol=1e-14)
    # no gate == plain attention over the concatenation
    Oc, _ = oracle.mixture_fwd(Q, K, V, None, causal=False, tau=1.0)
    Kc = np.concatenate(K, 2)
    Vc = np.concatenate(V, 2)
    Od, _ = oracle.attn_fwd(Q, Kc, Vc, causal=False, tau=1.0)
    np.testing.assert_allclose(Oc, Od, rtol=1e-12, atol=1e-13)
