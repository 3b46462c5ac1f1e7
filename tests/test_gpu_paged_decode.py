"""GPU parity of the decode over the paged fused-KV cache against the fp64 oracle, through the C
ABI: shuffled page tables, per-sequence lengths (ragged, page-aligned, one slot, empty), several
page sizes and split counts; and end to end: a cache written by mka_fuse_kv, read through pages,
equals the contiguous route-fused decode's numbers."""
import numpy as np
import pytest
import torch

from util import BF16_ATOL, announce, max_abs, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mka():
    import paper_2603_20586_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _pool(B, H, P, d, lens, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    max_pages = max(1, max((n + P - 1) // P for n in lens))
    n_pages = B * max_pages + 5
    perm = torch.randperm(n_pages, generator=gen, device="cuda")
    table = perm[:B * max_pages].reshape(B, max_pages).to(torch.int32).contiguous()
    Kp = torch.randn((n_pages, H, P, d), generator=gen, device="cuda").to(torch.bfloat16)
    Vp = torch.randn((n_pages, H, P, d), generator=gen, device="cuda").to(torch.bfloat16)
    q = torch.randn((B, H, 1, d), generator=gen, device="cuda").to(torch.bfloat16)
    return q, Kp, Vp, table, torch.tensor(lens, dtype=torch.int32, device="cuda")


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("P,lens,n_splits", [
    (16, [37, 16, 1], 0),          # ragged, exactly one page, one slot
    (64, [700, 333, 64], 3),       # several trips and pages, three splits (some slices empty)
    (128, [1000, 0, 129], 4),      # an empty sequence
    (256, [2500, 2500, 2500], 0)])
def test_paged_decode(mka, oracle, d, P, lens, n_splits):
    announce(f"paged decode d={d} P={P} lens={lens} splits={n_splits}")
    q, Kp, Vp, table, sl = _pool(len(lens), 3, P, d, lens, seed=60 + P)
    scale = 1.0 / np.sqrt(d)
    O, LSE = mka.mka_paged_fused_decode(q, Kp, Vp, table, sl, scale=scale, n_splits=n_splits)
    torch.cuda.synchronize()
    Oref, Lref = oracle.paged_fused_decode(q.cpu(), Kp.cpu(), Vp.cpu(), table.cpu().numpy(), lens,
                                           tau=scale)
    assert max_abs(O, Oref) <= BF16_ATOL, max_abs(O, Oref)
    fin = np.isfinite(Lref)
    assert np.array_equal(np.isfinite(to_np(LSE)), fin)
    assert float(np.abs(to_np(LSE)[fin] - Lref[fin]).max()) <= BF16_ATOL


def test_bad_table_entries_are_clamped_not_followed(mka):
    """Page ids outside the pool and a length beyond the table must not take the kernel outside
    the pool: the call completes and returns finite numbers."""
    announce("paged decode hostile table")
    q, Kp, Vp, table, sl = _pool(2, 2, 16, 64, [40, 40], seed=70)
    table[0, 1] = 10 ** 6
    table[1, 0] = -5
    sl[1] = 10 ** 6
    O, LSE = mka.mka_paged_fused_decode(q, Kp, Vp, table, sl, scale=0.1)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all() and torch.isfinite(LSE).all()


def test_paged_fused_cache_equals_contiguous_route_fused_decode(mka):
    """End to end: route, fuse the three memories once (mka_fuse_kv), scatter the fused rows into
    shuffled pages, decode through the table - against the contiguous decode that fuses the
    three raw caches at read time.  Same function, different rounding order (Kf / Vf are rounded
    to bf16 once in the fused cache)."""
    announce("paged fused cache vs contiguous raw-cache decode")
    import synth_inputs as si

    B, H, S, d, P = 2, 4, 300, 128, 64
    inp = si.prefill_inputs(B, H, S, S, d, dtype="bf16", seed=71, device="cuda")
    G, _ = mka.mka_route(inp["Q"], inp["W_r"] * 10, inp["b_r"])
    Kf = torch.empty_like(inp["K"][0]); Vf = torch.empty_like(inp["V"][0])
    mka.mka_fuse_kv(inp["K"], inp["V"], G, Kf=Kf, Vf=Vf)
    # reference: prefill forward's last row = attention of the last query over all S fused slots
    O, LSE, _, _ = mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], None, None, G=G, causal=True,
                                          scale=inp["scale"], materialise=False)
    n = (S + P - 1) // P
    perm = torch.randperm(B * n + 2, device="cuda")
    table = perm[:B * n].reshape(B, n).to(torch.int32).contiguous()
    Kp = torch.zeros((B * n + 2, H, P, d), device="cuda", dtype=torch.bfloat16)
    Vp = torch.zeros_like(Kp)
    for b in range(B):
        for i in range(n):
            rows = slice(i * P, min(S, (i + 1) * P))
            cnt = rows.stop - rows.start
            Kp[table[b, i], :, :cnt] = Kf[b, :, rows]
            Vp[table[b, i], :, :cnt] = Vf[b, :, rows]
    sl = torch.full((B,), S, dtype=torch.int32, device="cuda")
    q = inp["Q"][:, :, -1:, :].contiguous()
    Od, Ld = mka.mka_paged_fused_decode(q, Kp, Vp, table, sl, scale=inp["scale"])
    torch.cuda.synchronize()
    assert float((Od.float() - O[:, :, -1:].float()).abs().max()) <= BF16_ATOL
    assert float((Ld - LSE[:, :, -1]).abs().max()) <= BF16_ATOL
