"""Pins for the fp64 oracle against things the paper and the mathematics fix.

None of these tests compares the oracle with itself through the same formula:
each one checks a closed form, an invariant, a special case that reduces to a
textbook/library routine, or a brute-force evaluation written separately.
Citations refer to the paper: Alg. 2 (FastMKA), Eq. (1) (standard attention),
the max-shift recursion of the "Numerical Stability via Max-Shift" subsection.
"""
import math

import numpy as np
import pytest
import torch

RNG = np.random.default_rng(1234)


def rand(*shape, scale=1.0):
    return RNG.standard_normal(shape) * scale


def make(B=2, H=2, Tq=9, S=9, d=4, wscale=0.5):
    Q = rand(B, H, Tq, d)
    K = [rand(B, H, S, d) for _ in range(3)]
    V = [rand(B, H, S, d) for _ in range(3)]
    W = rand(d, 3, scale=wscale)
    b = rand(3, scale=0.3)
    return Q, K, V, W, b


def textbook_attention(Q, K, V, causal, tau):
    """Independent 15-line softmax attention (Eq. 1), numpy, bottom-right causal mask."""
    B, H, Tq, d = Q.shape
    S = K.shape[2]
    s = tau * np.einsum("bhtk,bhjk->bhtj", Q, K)
    if causal:
        t = np.arange(Tq)[:, None]
        j = np.arange(S)[None, :]
        s = np.where(j <= t + (S - Tq), s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("bhtj,bhjk->bhtk", p, V), p


# ---------------------------------------------------------------- brute force
def brute_force(Q, K, V, W, b, causal, tau):
    """Everything written as explicit nested Python sums for B=H=1 (separate code)."""
    Tq, d = len(Q), len(Q[0])
    S = len(K[0])
    G, idx = [], []
    for t in range(Tq):
        g = [b[l] + sum(Q[t][k] * W[k][l] for k in range(d)) for l in range(3)]
        mx = max(g)
        e = [math.exp(x - mx) for x in g]
        G.append([x / sum(e) for x in e])
        idx.append(g.index(mx))
    Kf = [[sum(G[j][l] * K[l][j][k] for l in range(3)) for k in range(d)] for j in range(S)]
    Vf = [[sum(G[j][l] * V[l][j][k] for l in range(3)) for k in range(d)] for j in range(S)]
    O = []
    for t in range(Tq):
        vis = [j for j in range(S) if (not causal) or j <= t + S - Tq]
        w = [math.exp(tau * sum(Q[t][k] * Kf[j][k] for k in range(d))) for j in vis]
        z = sum(w)
        O.append([sum(w[i] / z * Vf[j][k] for i, j in enumerate(vis)) for k in range(d)])
    return G, idx, O


@pytest.mark.parametrize("T,d,causal", [(1, 1, True), (3, 2, True), (4, 2, True), (4, 2, False)])
def test_brute_force_tiny(oracle, T, d, causal):
    Q, K, V, W, b = make(1, 1, T, T, d)
    tau = 0.7
    G, idx, O = brute_force(Q[0, 0].tolist(), [k[0, 0].tolist() for k in K],
                            [v[0, 0].tolist() for v in V], W.tolist(), b.tolist(), causal, tau)
    O2, LSE2, G2, idx2 = oracle.fwd_routed(Q, K, V, W, b, causal=causal, tau=tau)
    np.testing.assert_allclose(G2[0, 0], np.array(G), rtol=0, atol=1e-14)
    assert idx2[0, 0].tolist() == idx
    np.testing.assert_allclose(O2[0, 0], np.array(O), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- closed forms
def test_single_slot_closed_form(oracle):
    # Tq=S=1: p=1, so O = Vf[0] = sum_l lam_l V_l[0] whatever Q.K is
    Q, K, V, W, b = make(2, 3, 1, 1, 5)
    O, LSE, G, idx = oracle.fwd_routed(Q, K, V, W, b, tau=0.3)
    g = np.einsum("bhtk,kl->bhtl", Q, W) + b
    lam = np.exp(g) / np.exp(g).sum(-1, keepdims=True)
    expect = sum(lam[..., l:l + 1] * V[l] for l in range(3))
    np.testing.assert_allclose(O, expect, atol=1e-14)
    np.testing.assert_allclose(G, lam, atol=1e-15)


def test_zero_router_uniform_gates_and_tie_rule(oracle):
    Q, K, V, W, b = make(1, 2, 7, 7, 4)
    W0, b0 = np.zeros_like(W), np.zeros(3)
    O, LSE, G, idx = oracle.fwd_routed(Q, K, V, W0, b0, tau=0.5)
    assert np.all(G == 1.0 / 3.0)  # exactly equal logits
    assert np.all(idx == 0)  # ties go to the lowest level
    Kf = oracle.fuse(K, G)
    np.testing.assert_allclose(Kf, (K[0] + K[1] + K[2]) / 3.0, atol=1e-15)
    ref, _ = textbook_attention(Q, (K[0] + K[1] + K[2]) / 3, (V[0] + V[1] + V[2]) / 3, True, 0.5)
    np.testing.assert_allclose(O, ref, atol=1e-13)


@pytest.mark.parametrize("level", [0, 1, 2])
@pytest.mark.parametrize("causal", [True, False])
def test_one_hot_gates_reduce_to_standard_attention(oracle, level, causal):
    # bias +1000 on one level: exp(-1000) underflows to 0 in fp64, so lam is exactly one-hot and
    # the result must be textbook (and library) attention over that one memory.
    Q, K, V, W, b = make(2, 2, 11, 11, 8)
    W0 = np.zeros_like(W)
    b1 = np.zeros(3)
    b1[level] = 1000.0
    tau = 1.0 / math.sqrt(8)
    O, LSE, G, idx = oracle.fwd_routed(Q, K, V, W0, b1, causal=causal, tau=tau)
    onehot = np.zeros(3)
    onehot[level] = 1.0
    assert np.all(G == onehot)
    assert np.all(idx == level)
    ref, p = textbook_attention(Q, K[level], V[level], causal, tau)
    np.testing.assert_allclose(O, ref, atol=1e-13)
    lib = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K[level]), torch.from_numpy(V[level]),
        is_causal=causal, scale=tau)
    np.testing.assert_allclose(O, lib.numpy(), atol=1e-12)
    # LSE against its definition
    s = tau * np.einsum("bhtk,bhjk->bhtj", Q, K[level])
    if causal:
        s = np.where(np.tril(np.ones((11, 11), dtype=bool)), s, -np.inf)
    np.testing.assert_allclose(LSE, np.log(np.exp(s).sum(-1)), atol=1e-12)


def test_equal_memories_make_gates_irrelevant(oracle):
    Q, K, V, W, b = make(1, 2, 10, 10, 4)
    K = [K[0]] * 3
    V = [V[0]] * 3
    O1, *_ = oracle.fwd_routed(Q, K, V, W, b, tau=0.5)
    O2, *_ = oracle.fwd_routed(Q, K, V, rand(4, 3, scale=3.0), rand(3), tau=0.5)
    ref, _ = textbook_attention(Q, K[0], V[0], True, 0.5)
    np.testing.assert_allclose(O1, ref, atol=1e-13)
    np.testing.assert_allclose(O2, ref, atol=1e-13)


def test_zero_keys_give_prefix_means(oracle):
    Q, K, V, W, b = make(1, 1, 8, 8, 3)
    K = [np.zeros_like(k) for k in K]
    O, LSE, G, idx = oracle.fwd_routed(Q, K, V, W, b, tau=1.0)
    Vf = oracle.fuse(V, G)
    expect = np.cumsum(Vf, axis=2) / np.arange(1, 9)[None, None, :, None]
    np.testing.assert_allclose(O, expect, atol=1e-13)
    np.testing.assert_allclose(LSE[0, 0], np.log(np.arange(1, 9)), atol=1e-13)
    # tau -> 0 gives the same thing for any keys
    Q2, K2, V2, W2, b2 = make(1, 1, 8, 8, 3)
    O2, _, G2, _ = oracle.fwd_routed(Q2, K2, V2, W2, b2, tau=0.0)
    Vf2 = oracle.fuse(V2, G2)
    np.testing.assert_allclose(O2, np.cumsum(Vf2, 2) / np.arange(1, 9)[None, None, :, None],
                               atol=1e-13)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("Tq,S", [(12, 12), (5, 12), (1, 12)])
def test_probabilities_and_gates_are_distributions(oracle, Tq, S):
    Q, K, V, W, b = make(2, 2, Tq, S, 4)
    Gprev = np.abs(rand(2, 2, S, 3)) + 0.1
    Gprev /= Gprev.sum(-1, keepdims=True)
    G, idx = oracle.route(Q, W, b, S=S, G_prev=Gprev)
    np.testing.assert_allclose(G.sum(-1), 1.0, atol=1e-15)
    assert np.all(G >= 0)
    np.testing.assert_array_equal(G[:, :, :S - Tq], Gprev[:, :, :S - Tq])  # old slots untouched
    Kf, Vf = oracle.fuse(K, G), oracle.fuse(V, G)
    O, LSE, P = oracle.attn_fwd(Q, Kf, Vf, causal=True, tau=0.4, return_p=True)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-14)
    assert np.all(P >= 0)
    t = np.arange(Tq)[:, None]
    j = np.arange(S)[None, :]
    assert np.all(P[:, :, j > t + (S - Tq)] == 0)  # bottom-right aligned causal mask
    assert np.all(P[:, :, j <= t + (S - Tq)] > 0)
    np.testing.assert_allclose(np.einsum("bhtj,bhjk->bhtk", P, Vf), O, atol=1e-13)


@pytest.mark.parametrize("Bc", [1, 3, 16, 64, 70])
@pytest.mark.parametrize("causal", [True, False])
def test_block_size_independence_of_max_shift_recursion(oracle, Bc, causal):
    Q, K, V, W, b = make(1, 2, 70, 70, 8)
    Q = Q * 4.0  # large logits so that the running max really moves
    G, _ = oracle.route(Q, W, b)
    Kf, Vf = oracle.fuse(K, G), oracle.fuse(V, G)
    O, LSE = oracle.attn_fwd(Q, Kf, Vf, causal=causal, tau=0.9)
    Ob, LSEb = oracle.attn_fwd_blockwise(Q, Kf, Vf, Bc, causal=causal, tau=0.9)
    np.testing.assert_allclose(Ob, O, rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSEb, LSE, rtol=0, atol=1e-12)


def test_level_permutation_symmetry(oracle):
    Q, K, V, W, b = make(1, 2, 9, 9, 4)
    perm = [2, 0, 1]
    O1, _, G1, idx1 = oracle.fwd_routed(Q, K, V, W, b, tau=0.5)
    O2, _, G2, idx2 = oracle.fwd_routed(Q, [K[p] for p in perm], [V[p] for p in perm],
                                        W[:, perm], b[perm], tau=0.5)
    np.testing.assert_allclose(O2, O1, atol=1e-13)
    np.testing.assert_allclose(G2, G1[..., perm], atol=1e-15)
    inv = np.argsort(perm)
    np.testing.assert_array_equal(idx2, inv[idx1])


def test_bias_shift_and_value_linearity(oracle):
    Q, K, V, W, b = make(1, 2, 9, 9, 4)
    O1, _, G1, _ = oracle.fwd_routed(Q, K, V, W, b, tau=0.5)
    O2, _, G2, _ = oracle.fwd_routed(Q, K, V, W, b + 2.5, tau=0.5)
    np.testing.assert_allclose(G2, G1, atol=1e-15)
    np.testing.assert_allclose(O2, O1, atol=1e-13)
    V2 = [rand(*v.shape) for v in V]
    Oa, *_ = oracle.fwd_routed(Q, K, V2, W, b, tau=0.5)
    Ob, *_ = oracle.fwd_routed(Q, K, [2 * V[l] - 3 * V2[l] for l in range(3)], W, b, tau=0.5)
    np.testing.assert_allclose(Ob, 2 * O1 - 3 * Oa, atol=1e-12)


def test_absent_level_is_zero_memory_without_renormalisation(oracle):
    # a level with no entry at a slot contributes the zero vector (Alg. 1: M_3 <- 0)
    Q, K, V, W, b = make(1, 2, 10, 10, 4)
    len3 = [10, 6, 0]
    G, _ = oracle.route(Q, W, b)
    O1, L1 = oracle.fwd(Q, K, V, G, len3=len3, tau=0.5)
    Kz = [K[0].copy(), K[1].copy(), np.zeros_like(K[2])]
    Vz = [V[0].copy(), V[1].copy(), np.zeros_like(V[2])]
    Kz[1][:, :, 6:] = 0
    Vz[1][:, :, 6:] = 0
    O2, L2 = oracle.fwd(Q, Kz, Vz, G, tau=0.5)
    np.testing.assert_allclose(O1, O2, atol=1e-14)
    np.testing.assert_allclose(L1, L2, atol=1e-14)
    # a missing pointer is the same as length 0
    O3, _ = oracle.fwd(Q, [K[0], K[1], None], [V[0], V[1], None], G, len3=[10, 6, 10], tau=0.5)
    np.testing.assert_allclose(O3, O1, atol=1e-14)


def test_cache_prefix_is_bottom_right_aligned(oracle):
    # Tq new rows over S slots == the last Tq rows of the full S x S causal problem
    S, Tq = 13, 4
    Qf, K, V, W, b = make(1, 2, S, S, 4)
    Of, _, Gf, idxf = oracle.fwd_routed(Qf, K, V, W, b, tau=0.5)
    Qn = Qf[:, :, S - Tq:]
    On, _, Gn, idxn = oracle.fwd_routed(Qn, K, V, W, b, G_prev=Gf, tau=0.5)
    np.testing.assert_allclose(On, Of[:, :, S - Tq:], atol=1e-14)
    np.testing.assert_array_equal(Gn, Gf)
    np.testing.assert_array_equal(idxn, idxf[:, :, S - Tq:])


# ---------------------------------------------------------------- decode
def test_decode_equals_last_prefill_row_and_appends(oracle):
    B, H, d, S0, steps = 2, 2, 4, 6, 3
    Q, K, V, W, b = make(B, H, S0 + steps, S0 + steps, d)
    # prefill over the first S0 tokens gives the gate cache
    G0, _ = oracle.route(Q[:, :, :S0], W, b)
    cap = S0 + steps
    Kc = [np.zeros((B, H, cap if l == 0 else S0, d)) for l in range(3)]
    Vc = [np.zeros((B, H, cap if l == 0 else S0, d)) for l in range(3)]
    for l in range(3):
        Kc[l][:, :, :S0] = K[l][:, :, :S0]
        Vc[l][:, :, :S0] = V[l][:, :, :S0]
    Gc = np.zeros((B, H, cap, 3))
    Gc[:, :, :S0] = G0
    len3 = [S0, S0, S0]
    for s in range(steps):
        j = S0 + s
        q = Q[:, :, j:j + 1]
        O, LSE, idx = oracle.decode(q, [K[0][:, :, j:j + 1], None, None],
                                    [V[0][:, :, j:j + 1], None, None], Kc, Vc, Gc, len3, W, b,
                                    tau=0.5)
        assert len3 == [j + 1, S0, S0]
        # reference: prefill over j+1 slots where levels 2,3 stop at S0
        Sn = j + 1
        Gall, idxall = oracle.route(Q[:, :, :Sn], W, b)
        Oref, LSEref = oracle.fwd(Q[:, :, :Sn], [x[:, :, :Sn] for x in K],
                                  [x[:, :, :Sn] for x in V], Gall, len3=[Sn, S0, S0], tau=0.5)
        np.testing.assert_allclose(O[:, :, 0], Oref[:, :, -1], atol=1e-13)
        np.testing.assert_allclose(LSE[:, :, 0], LSEref[:, :, -1], atol=1e-13)
        np.testing.assert_array_equal(idx, idxall[:, :, -1])
        np.testing.assert_array_equal(Gc[:, :, :Sn], Gall)
        np.testing.assert_array_equal(Kc[0][:, :, :Sn], K[0][:, :, :Sn])
    with pytest.raises(ValueError):  # level 2 skipped tokens: it cannot rejoin
        oracle.decode(Q[:, :, :1], [K[0][:, :, :1], K[1][:, :, :1], None],
                      [V[0][:, :, :1], V[1][:, :, :1], None], Kc, Vc, Gc, len3, W, b)


# ---------------------------------------------------------------- backward
def _loss(oracle, Q, K, V, W, b, dO, len3, Tq, S, tau, Gprev):
    O, _, _, _ = oracle.fwd_routed(Q, K, V, W, b, G_prev=Gprev, len3=len3, tau=tau)
    return float((O * dO).sum())


@pytest.mark.parametrize("Tq,S,len3", [(5, 5, None), (3, 6, None), (5, 5, [5, 3, 0])])
def test_backward_matches_central_finite_differences(oracle, Tq, S, len3):
    B, H, d, tau = 1, 2, 3, 0.6
    Q, K, V, W, b = make(B, H, Tq, S, d)
    dO = rand(B, H, Tq, d)
    Gprev = np.abs(rand(B, H, S, 3)) + 0.1
    Gprev /= Gprev.sum(-1, keepdims=True)
    G, _ = oracle.route(Q, W, b, S=S, G_prev=Gprev)
    g = oracle.bwd(dO, Q, K, V, G, W, len3=len3, tau=tau)
    h = 1e-5

    def fd(arr, setter):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h
            lp = _loss(oracle, Q, K, V, W, b, dO, len3, Tq, S, tau, Gprev)
            arr[i] = old - h
            lm = _loss(oracle, Q, K, V, W, b, dO, len3, Tq, S, tau, Gprev)
            arr[i] = old
            out[i] = (lp - lm) / (2 * h)
        return out

    def close(a, ref):
        np.testing.assert_allclose(a, ref, rtol=1e-6, atol=1e-8 * max(1.0, np.abs(ref).max()))

    close(g["dQ"], fd(Q, None))
    for l in range(3):
        close(g["dK"][l], fd(K[l], None))
        close(g["dV"][l], fd(V[l], None))
    close(g["dW_r"], fd(W, None))
    close(g["db_r"], fd(b, None))
    assert abs(g["db_r"].sum()) < 1e-12  # softmax Jacobian: sum_l dg = 0


def test_backward_matches_autograd_second_opinion(oracle):
    # the same forward written with fp64 torch CPU ops; autograd is the library routine
    B, H, Tq, S, d, tau = 2, 2, 7, 10, 4, 0.5
    Q, K, V, W, b = make(B, H, Tq, S, d)
    dO = rand(B, H, Tq, d)
    len3 = [10, 8, 10]
    Gprev = np.abs(rand(B, H, S, 3)) + 0.1
    Gprev /= Gprev.sum(-1, keepdims=True)
    G, _ = oracle.route(Q, W, b, S=S, G_prev=Gprev)
    got = oracle.bwd(dO, Q, K, V, G, W, len3=len3, tau=tau, want_dG=True)

    tq = torch.tensor(Q, requires_grad=True)
    tk = [torch.tensor(x, requires_grad=True) for x in K]
    tv = [torch.tensor(x, requires_grad=True) for x in V]
    tw = torch.tensor(W, requires_grad=True)
    tb = torch.tensor(b, requires_grad=True)
    lam_new = torch.softmax(tq @ tw + tb, dim=-1)
    tg = torch.cat([torch.tensor(Gprev[:, :, :S - Tq]), lam_new], dim=2)
    tg.retain_grad()
    mask = torch.stack([(torch.arange(S) < len3[l]).double() for l in range(3)], -1)  # [S,3]
    kf = sum((tg[..., l] * mask[:, l])[..., None] * tk[l] for l in range(3))
    vf = sum((tg[..., l] * mask[:, l])[..., None] * tv[l] for l in range(3))
    s = tau * tq @ kf.transpose(-1, -2)
    vis = torch.arange(S)[None, :] <= torch.arange(Tq)[:, None] + (S - Tq)
    p = torch.softmax(s.masked_fill(~vis, float("-inf")), dim=-1)
    ((p @ vf) * torch.tensor(dO)).sum().backward()
    np.testing.assert_allclose(got["dQ"], tq.grad.numpy(), atol=1e-12)
    for l in range(3):
        np.testing.assert_allclose(got["dK"][l], tk[l].grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(got["dV"][l], tv[l].grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(got["dW_r"], tw.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(got["db_r"], tb.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(got["dG"], tg.grad.numpy(), atol=1e-12)


def test_planted_mistakes_are_caught(oracle):
    """A transposed W_r, a dropped level or a top-left mask would each break a pin above;
    show it on the brute-force case by planting them in the *expected* side."""
    Q, K, V, W, b = make(1, 1, 4, 4, 3)
    O, _, G, _ = oracle.fwd_routed(Q, K, V, W, b, tau=0.7)
    # dropped level
    O_bad, _ = oracle.fwd(Q, [K[0], K[1], None], [V[0], V[1], None], G, tau=0.7)
    assert np.abs(O - O_bad).max() > 1e-3
    # wrong sign of the shift in the softmax would not change p; wrong tau would
    O_bad2, *_ = oracle.fwd_routed(Q, K, V, W, b, tau=0.71)
    assert np.abs(O - O_bad2).max() > 1e-5
