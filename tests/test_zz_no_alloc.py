"""GPU test of the decode entry point that allocates nothing (mka_fused_attn_decode_static):
through the C ABI, its outputs against those of mka_fused_attn_decode (same kernels, the split-K
partials in the library's fixed device buffer instead of a caller workspace), on two calls in a
row, the second with a smaller input - the buffer then still holds the first call's partials."""
import pytest
import torch

import synth_inputs as si
from util import BF16_ATOL, announce

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mka():
    import paper_2603_20586_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _both(mka, B, H, d, S0, seed, n_splits):
    """One decode step through each entry point on identical caches; returns the two results."""
    outs = []
    for static in (False, True):
        c = si.decode_caches(B, H, d, S0, cap_extra=2, dtype="bf16", seed=seed, device="cuda")
        q, k1, v1 = si.decode_step_inputs(B, H, d, 0, dtype="bf16", seed=seed, device="cuda")
        ln = list(c["len"])
        if static:
            O = torch.empty_like(q)
            LSE = torch.empty((B, H), dtype=torch.float32, device="cuda")
            idx = torch.empty((B, H), dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            before = torch.cuda.memory_stats()["allocation.all.allocated"]
            mka.mka_fused_attn_decode_static(q, [k1, None, None], [v1, None, None], c["Kc"], c["Vc"],
                                             c["Gc"], ln, c["W_r"], c["b_r"], O, LSE, idx,
                                             scale=c["scale"], n_splits=n_splits)
            assert torch.cuda.memory_stats()["allocation.all.allocated"] == before  # torch's allocator idle
        else:
            O, LSE, idx = mka.mka_fused_attn_decode(q, [k1, None, None], [v1, None, None], c["Kc"],
                                                    c["Vc"], c["Gc"], ln, c["W_r"], c["b_r"],
                                                    scale=c["scale"], n_splits=n_splits)
        torch.cuda.synchronize()
        outs.append((O, LSE, idx, ln, c["Gc"][:, :, S0].clone(), c["Kc"][0][:, :, S0].clone()))
    return outs


def _compare(a, b):
    (O0, L0, i0, ln0, g0, k0), (O1, L1, i1, ln1, g1, k1) = a, b
    assert ln0 == ln1
    assert torch.equal(i0, i1) and torch.equal(g0, g1) and torch.equal(k0, k1)   # index / byte work
    assert float((O0.float() - O1.float()).abs().max()) <= BF16_ATOL
    assert float((L0 - L1).abs().max()) <= BF16_ATOL
    # same kernels, same split count, same order of every sum: the bits agree too
    assert torch.equal(O0, O1) and torch.equal(L0, L1)


def test_static_decode_matches_workspace_decode_twice_in_a_row(mka):
    announce("decode without allocation: large call, then a smaller one")
    big = _both(mka, 3, 8, 128, 5000, seed=7, n_splits=0)       # 24 heads, several splits
    _compare(*big)
    small = _both(mka, 1, 2, 128, 300, seed=8, n_splits=0)      # fewer heads, one split: the
    _compare(*small)                                            # buffer still holds the big call's partials
    d64 = _both(mka, 2, 2, 64, 1000, seed=9, n_splits=3)        # another head dim, explicit splits
    _compare(*d64)


def test_static_decode_rejects_what_does_not_fit(mka):
    announce("decode without allocation: size limit")
    B, H, d = 64, 64, 128       # 4096 heads x 130 floats = 2.03 MiB per split: 3 fit, 5 do not
    c = si.decode_caches(B, H, d, 64, cap_extra=1, dtype="bf16", seed=3, device="cuda")
    q, k1, v1 = si.decode_step_inputs(B, H, d, 0, dtype="bf16", seed=3, device="cuda")
    O = torch.empty_like(q)
    ln = list(c["len"])
    with pytest.raises(mka.MkaError) as e:
        mka.mka_fused_attn_decode_static(q, [k1, None, None], [v1, None, None], c["Kc"], c["Vc"],
                                         c["Gc"], ln, c["W_r"], c["b_r"], O, scale=c["scale"], n_splits=5)
    assert e.value.status == 5 and ln == list(c["len"])          # MKA_ERR_WORKSPACE, nothing ran
    mka.mka_fused_attn_decode_static(q, [k1, None, None], [v1, None, None], c["Kc"], c["Vc"],
                                     c["Gc"], ln, c["W_r"], c["b_r"], O, scale=c["scale"], n_splits=3)
    torch.cuda.synchronize()
    assert ln[0] == c["len"][0] + 1 and torch.isfinite(O.float()).all()
