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


def _big_pool(B, H, P, d, S, seed):
    """Pool of B*ceil(S/P) pages in a shuffled table, filled chunk by chunk (a single randn call
    over the whole pool would need an f32 temporary of twice its size)."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    npg = (S + P - 1) // P
    n_pages = B * npg
    Kp = torch.empty((n_pages, H, P, d), device="cuda", dtype=torch.bfloat16)
    Vp = torch.empty_like(Kp)
    step = max(1, (1 << 27) // (H * P * d))
    for i in range(0, n_pages, step):
        n = min(step, n_pages - i)
        Kp[i:i + n] = torch.randn((n, H, P, d), generator=gen, device="cuda").to(torch.bfloat16)
        Vp[i:i + n] = torch.randn((n, H, P, d), generator=gen, device="cuda").to(torch.bfloat16)
    table = torch.randperm(n_pages, generator=gen, device="cuda").reshape(B, npg).to(torch.int32).contiguous()
    q = torch.randn((B, H, 1, d), generator=gen, device="cuda").to(torch.bfloat16)
    return q, Kp, Vp, table


@pytest.mark.timeout(600)
@pytest.mark.parametrize("S", [32768, 131072], ids=["C4-shape-32K", "128K-slots"])
def test_paged_decode_full_size_sampled_heads(mka, oracle, S):
    """The decode shape of config C4 (B16 H32 d128) over the paged fused cache at 32K slots and at
    the context length the paper pages for (128K; sequences of unequal length), in the launch
    configuration bench.py times.  Every head runs; three are compared: the oracle gets that
    head's slice of the whole pool and the sequence's row of the shuffled table."""
    announce(f"paged decode full size B16 H32 d128 S={S}")
    B, H, d, P = 16, 32, 128, 128
    q, Kp, Vp, table = _big_pool(B, H, P, d, S, seed=80)
    lens = [S] * B
    lens[6] = S - 77          # ragged: ends inside a page
    lens[15] = S - P          # ends on a page boundary
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    scale = 1.0 / np.sqrt(d)
    O, LSE = mka.mka_paged_fused_decode(q, Kp, Vp, table, sl, scale=scale)
    torch.cuda.synchronize()
    for (b, h) in [(0, 0), (15, 31), (6, 17)]:
        print(f"[case] oracle head ({b},{h})", flush=True)
        Oref, Lref = oracle.paged_fused_decode(
            q[b:b + 1, h:h + 1].cpu(), Kp[:, h:h + 1].cpu(), Vp[:, h:h + 1].cpu(),
            table[b:b + 1].cpu().numpy(), [lens[b]], tau=scale)
        assert max_abs(O[b:b + 1, h:h + 1], Oref) <= BF16_ATOL
        assert abs(float(LSE[b, h]) - float(Lref[0, 0])) <= BF16_ATOL
    assert torch.isfinite(O.float()).all()


@pytest.mark.parametrize("d", [128, 64])
def test_contiguous_fused_cache_decode_end_to_end(mka, oracle, d):
    """Decode over a single FUSED cache (what the paper caches), end to end from mka_fuse_kv:
    route, fuse the three raw memories once, then three decode steps in which the new token's
    rows are fused with its own gate and appended to the fused cache (level 1 alone, levels 2
    and 3 NULL, gate rows (1,0,0), no router weights).  Reference: the oracle's route-fused
    decode over the three RAW caches - the same function; the fused cache only adds one bf16
    rounding of Kf / Vf."""
    import synth_inputs as si

    announce(f"contiguous fused-cache decode d={d}")
    B, H, S0, steps = 2, 3, 700, 3
    inp = si.prefill_inputs(B, H, S0, S0, d, dtype="bf16", seed=90, device="cuda")
    W = inp["W_r"] * 10
    G, _ = mka.mka_route(inp["Q"], W, inp["b_r"])
    cap = S0 + steps
    Kfc = torch.zeros((B, H, cap, d), device="cuda", dtype=torch.bfloat16)
    Vfc = torch.zeros_like(Kfc)
    Kf, Vf = mka.mka_fuse_kv(inp["K"], inp["V"], G)
    Kfc[:, :, :S0], Vfc[:, :, :S0] = Kf, Vf
    Gone = torch.zeros((B, H, cap, 3), device="cuda")
    Gone[..., 0] = 1.0
    # the oracle keeps the three raw caches and the real gates
    grow = lambda x: np.concatenate([to_np(x), np.zeros((B, H, steps, d))], 2)  # noqa: E731
    Kc_o = [grow(k) for k in inp["K"]]
    Vc_o = [grow(v) for v in inp["V"]]
    Gc_o = np.concatenate([to_np(G), np.zeros((B, H, steps, 3))], 2)
    len_g, len_o = [S0, 0, 0], [S0, S0, S0]
    for step in range(steps):
        q, _, _ = si.decode_step_inputs(B, H, d, step, device="cuda", seed=91)
        kn = [si.decode_step_inputs(B, H, d, step, device="cuda", seed=92 + l)[1] for l in range(3)]
        vn = [si.decode_step_inputs(B, H, d, step, device="cuda", seed=92 + l)[2] for l in range(3)]
        g_new, _ = mka.mka_route(q, W, inp["b_r"])                       # [B,H,1,3]
        kf_new, vf_new = mka.mka_fuse_kv(kn, vn, g_new)                  # the new token's fused rows
        O, LSE, idx = mka.mka_fused_attn_decode(q, [kf_new, None, None], [vf_new, None, None],
                                                [Kfc, None, None], [Vfc, None, None], Gone, len_g,
                                                None, None, scale=inp["scale"])
        torch.cuda.synchronize()
        assert idx is None and len_g == [S0 + step + 1, 0, 0]
        Oref, Lref, _ = oracle.decode(q.cpu(), [k.cpu() for k in kn], [v.cpu() for v in vn], Kc_o,
                                      Vc_o, Gc_o, len_o, W.cpu(), inp["b_r"].cpu(), tau=inp["scale"])
        assert max_abs(O, Oref) <= BF16_ATOL, (step, max_abs(O, Oref))
        assert max_abs(LSE, Lref[:, :, 0]) <= BF16_ATOL
    assert bool((Gone[..., 0] == 1).all()) and bool((Gone[..., 1:] == 0).all())  # gate rows untouched
