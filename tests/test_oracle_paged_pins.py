"""Pins of the oracle's decode over the paged fused-KV cache (paper: fused keys / values are what
is cached, section "Route-Fused MKA (FastMKA)"; paged layout for long contexts, section
"Experimental Setup").  The attention itself is the oracle's plain attention (pinned elsewhere);
what is new is the page-table gather, pinned against dense layouts, a permutation of the
physical pages, per-sequence lengths and scipy's softmax."""
import numpy as np
from scipy.special import softmax


def _paged(rng, B, H, P, d, lens, shuffle=True):
    max_pages = max(1, max((n + P - 1) // P for n in lens))
    n_pages = B * max_pages + 3
    ids = rng.permutation(n_pages) if shuffle else np.arange(n_pages)
    table = ids[:B * max_pages].reshape(B, max_pages).astype(np.int32)
    Kpool = rng.standard_normal((n_pages, H, P, d))
    Vpool = rng.standard_normal((n_pages, H, P, d))
    return Kpool, Vpool, table, np.asarray(lens, dtype=np.int32)


def _dense(pool, table, n, b, h):
    P = pool.shape[2]
    pages = [pool[table[b, i], h] for i in range((n + P - 1) // P)]
    return np.concatenate(pages, 0)[:n] if pages else np.zeros((0, pool.shape[3]))


def test_against_scipy_softmax_on_the_gathered_rows(oracle):
    rng = np.random.default_rng(0)
    B, H, P, d = 2, 3, 16, 8
    Kp, Vp, table, lens = _paged(rng, B, H, P, d, [37, 16])
    q = rng.standard_normal((B, H, 1, d))
    O, LSE = oracle.paged_fused_decode(q, Kp, Vp, table, lens, tau=0.4)
    for b in range(B):
        for h in range(H):
            K = _dense(Kp, table, lens[b], b, h)
            V = _dense(Vp, table, lens[b], b, h)
            s = 0.4 * K @ q[b, h, 0]
            np.testing.assert_allclose(O[b, h, 0], softmax(s) @ V, atol=1e-13)
            np.testing.assert_allclose(LSE[b, h], np.log(np.exp(s - s.max()).sum()) + s.max(), atol=1e-13)


def test_identity_table_is_the_contiguous_decode(oracle):
    # pages in order = a contiguous cache: the same numbers as plain attention over [B,H,S,d]
    rng = np.random.default_rng(1)
    B, H, P, d, S = 2, 2, 16, 4, 48
    Kd = rng.standard_normal((B, H, S, d))
    Vd = rng.standard_normal((B, H, S, d))
    q = rng.standard_normal((B, H, 1, d))
    n = S // P
    Kp = Kd.reshape(B, H, n, P, d).transpose(0, 2, 1, 3, 4).reshape(B * n, H, P, d)
    Vp = Vd.reshape(B, H, n, P, d).transpose(0, 2, 1, 3, 4).reshape(B * n, H, P, d)
    table = np.arange(B * n, dtype=np.int32).reshape(B, n)
    O, LSE = oracle.paged_fused_decode(q, Kp, Vp, table, [S, S], tau=0.7)
    Oref, Lref = oracle.attn_fwd(q, Kd, Vd, causal=False, tau=0.7)
    np.testing.assert_allclose(O, Oref, atol=1e-14)
    np.testing.assert_allclose(LSE, Lref[..., 0], atol=1e-14)


def test_moving_pages_with_their_table_entries_changes_nothing(oracle):
    rng = np.random.default_rng(2)
    B, H, P, d = 2, 2, 16, 4
    Kp, Vp, table, lens = _paged(rng, B, H, P, d, [40, 21], shuffle=False)
    q = rng.standard_normal((B, H, 1, d))
    O1, L1 = oracle.paged_fused_decode(q, Kp, Vp, table, lens, tau=1.0)
    perm = rng.permutation(Kp.shape[0])           # new physical position of every page
    Kp2, Vp2 = np.empty_like(Kp), np.empty_like(Vp)
    Kp2[perm], Vp2[perm] = Kp, Vp
    O2, L2 = oracle.paged_fused_decode(q, Kp2, Vp2, perm[table].astype(np.int32), lens, tau=1.0)
    np.testing.assert_array_equal(O1, O2)
    np.testing.assert_array_equal(L1, L2)


def test_rows_past_a_sequence_s_length_are_not_read(oracle):
    rng = np.random.default_rng(3)
    B, H, P, d = 2, 1, 16, 4
    Kp, Vp, table, lens = _paged(rng, B, H, P, d, [19, 0])
    q = rng.standard_normal((B, H, 1, d))
    O1, L1 = oracle.paged_fused_decode(q, Kp, Vp, table, lens, tau=1.0)
    Kp2, Vp2 = Kp.copy(), Vp.copy()
    Kp2[table[0, 1], :, 3:] = np.nan               # rows 19.. of the second page of sequence 0
    Vp2[table[0, 1], :, 3:] = np.nan
    O2, L2 = oracle.paged_fused_decode(q, Kp2, Vp2, table, lens, tau=1.0)
    np.testing.assert_array_equal(O1, O2)
    assert np.all(O1[1] == 0.0) and np.all(np.isneginf(L1[1]))    # empty sequence
