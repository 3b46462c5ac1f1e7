"""GPU parity of the symbolic (full) MKA forward (Alg. 1: one attention per memory, outputs mixed
with the per-query gates) and of the causal prefix-mean summary (the L2 producer of Alg. 1)
against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from util import BF16_ATOL, announce, cpu_list, max_abs

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


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("Tq,S3,causal", [
    (300, (300, 300, 300), True),     # several query tiles and KV tiles, ragged tails
    (130, (333, 130, 200), True),     # memories of their own lengths and diagonals
    (200, (260, 70, 1), False),       # non-causal, a one-slot memory
    (257, (257, None, 300), True),    # a memory absent: contributes nothing
    (1, (1, 1, 1), True)])
def test_full_mka_shapes(mka, oracle, d, Tq, S3, causal):
    announce(f"full MKA d={d} Tq={Tq} S={S3} causal={causal}")
    Q, K, V, G = _inputs(2, 2, Tq, S3, d, seed=41)
    scale = 1.0 / np.sqrt(d)
    O = mka.mka_full_attn_fwd(Q, K, V, G, causal=causal, scale=scale)
    torch.cuda.synchronize()
    Oref = oracle.full_mka_fwd(Q.cpu(), cpu_list(K), cpu_list(V), G.cpu(), causal=causal, tau=scale)
    assert max_abs(O, Oref) <= BF16_ATOL, max_abs(O, Oref)


def test_full_mka_one_hot_gates_equal_plain_attention(mka):
    """Needs no oracle: with one-hot gates the output is the attention kernel's output over that
    memory, bit for bit (the combine step multiplies by 1 and adds zeros)."""
    announce("full MKA one-hot")
    Q, K, V, _ = _inputs(1, 2, 200, (200, 230, 260), 128, seed=42)
    for l in range(3):
        G = torch.zeros((1, 2, 200, 3), device="cuda")
        G[..., l] = 1.0
        O = mka.mka_full_attn_fwd(Q, K, V, G, causal=True, scale=0.09)
        Kl = [K[l], None, None]
        Vl = [V[l], None, None]
        A, _ = mka.mka_mixture_attn_fwd(Q, Kl, Vl, None, causal=True, scale=0.09)
        torch.cuda.synchronize()
        assert torch.equal(O, A)


def test_full_mka_rejects_missing_workspace(mka):
    import ctypes
    from paper_2603_20586_amd.binding import _p3, _ptr, _shape, _stream

    Q, K, V, G = _inputs(1, 1, 64, (64, 64, 64), 64, seed=43)
    O = torch.empty_like(Q)
    s = _shape(Q, 64, [64, 64, 64], True, 0.1)
    Kp, Vp = _p3(K), _p3(V)
    rc = mka.lib().mka_full_attn_fwd(_ptr(Q), ctypes.byref(Kp), ctypes.byref(Vp), _ptr(G), _ptr(O),
                                     ctypes.byref(s), None, 0, _stream())
    assert rc == 5


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("S", [1, 63, 64, 65, 200, 1000])
def test_prefix_mean(mka, oracle, d, S):
    announce(f"prefix mean d={d} S={S}")
    gen = torch.Generator(device="cuda").manual_seed(50 + S)
    X = (torch.randn((2, 3, S, d), generator=gen, device="cuda") + 0.5).to(torch.bfloat16)
    M = mka.mka_prefix_mean(X)
    torch.cuda.synchronize()
    ref = oracle.prefix_mean(X.cpu())
    assert max_abs(M, ref) <= BF16_ATOL, max_abs(M, ref)
    assert torch.equal(M[:, :, 0], X[:, :, 0])      # the mean of one row is the row


def test_full_mka_with_prefix_mean_memory(mka, oracle):
    """Alg. 1 end to end on the memories it defines: L1 = the keys / values, L2 = their causal
    prefix mean (produced on the GPU), L3 absent."""
    announce("full MKA with prefix-mean L2")
    Q, K, V, G = _inputs(1, 2, 180, (180, None, None), 128, seed=44)
    K2, V2 = mka.mka_prefix_mean(K[0]), mka.mka_prefix_mean(V[0])
    O = mka.mka_full_attn_fwd(Q, [K[0], K2, None], [V[0], V2, None], G, causal=True, scale=0.09)
    torch.cuda.synchronize()
    K2r = oracle.prefix_mean(K[0].cpu()); V2r = oracle.prefix_mean(V[0].cpu())
    Oref = oracle.full_mka_fwd(Q.cpu(), [K[0].cpu(), K2r, None], [V[0].cpu(), V2r, None], G.cpu(),
                               causal=True, tau=0.09)
    assert max_abs(O, Oref) <= BF16_ATOL


def test_full_mka_long_prefill_shape_sampled_rows(mka, oracle):
    """C3 shape (B1 H32 T8192 d128), the size bench.py times: sampled query rows, each a one-row
    problem over slots 0..t of every memory for the oracle."""
    import synth_inputs as si
    from util import announce as _announce

    _announce("full MKA C3 shape, sampled rows")
    inp, cfg = si.config_inputs("C3", device="cuda")
    G, _ = mka.mka_route(inp["Q"], inp["W_r"] * 30.0, inp["b_r"], want_idx=False)
    O = mka.mka_full_attn_fwd(inp["Q"], inp["K"], inp["V"], G, causal=True, scale=inp["scale"])
    torch.cuda.synchronize()
    worst = 0.0
    for (b, h) in [(0, 0), (0, 31), (0, 13)]:
        for t in [0, 1, 63, 64, 255, 256, 257, 4095, 4096, 8000, 8191]:
            cut = lambda x, lo, hi: x[b:b + 1, h:h + 1, lo:hi].cpu()  # noqa: E731
            Oref = oracle.full_mka_fwd(cut(inp["Q"], t, t + 1), [cut(k, 0, t + 1) for k in inp["K"]],
                                       [cut(v, 0, t + 1) for v in inp["V"]], cut(G, t, t + 1),
                                       causal=True, tau=inp["scale"])
            worst = max(worst, max_abs(O[b:b + 1, h:h + 1, t:t + 1], Oref))
    assert worst <= BF16_ATOL, worst
