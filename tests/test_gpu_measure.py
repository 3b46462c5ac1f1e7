"""The measurement micro-benchmarks (libmka_measure.so, not product surface) on the GPU: the MFMA
loops are checked against the closed form of their checksum, so that the flop count bench.py
credits them with is the work they really do."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_mfma_loop_on_supplied_operands_matches_its_closed_form():
    from paper_2603_20586_amd import measure

    iters, wgs = 5, 3
    n = measure.FRAG_BYTES // 2
    fr = torch.ones(n, dtype=torch.float32, device="cuda").view(16, 512, 8)
    for j in range(8):
        fr[2 * j] = float(j + 1)      # A fragment j of every lane: all elements j + 1
    frags = fr.reshape(-1).to(torch.bfloat16)
    out = torch.zeros(wgs * 512, dtype=torch.float32, device="cuda")
    flops = measure.mfma_loop_data(out, frags, wgs, iters)
    torch.cuda.synchronize()
    # every MFMA adds 16 (j + 1) to each element of its accumulator; a lane sums 4 chains x 16
    # registers, each chain sees every j once per iteration
    expect = 64 * 16 * sum(range(1, 9)) * iters
    assert torch.equal(out, torch.full_like(out, float(expect)))
    assert flops == wgs * 8 * iters * 32 * 2 * 32 * 32 * 16


def test_mfma_loop_and_read_loop_run():
    from paper_2603_20586_amd import measure

    out = torch.zeros(4 * 512, dtype=torch.float32, device="cuda")
    flops = measure.mfma_loop(out, 4, 10)
    src = torch.ones(1 << 20, dtype=torch.int32, device="cuda")
    nbytes = measure.stream_read(src)
    torch.cuda.synchronize()
    assert flops == 4 * 8 * 10 * 4 * 2 * 32 * 32 * 16
    assert torch.isfinite(out).all()
    assert 0 < nbytes <= src.numel() * 4
