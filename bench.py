#!/usr/bin/env python3
"""Benchmark of the FastMKA route-fused attention hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input at the shape of
benchmark config C2 (B=4, H=16, d=128, T=2048, bf16, causal):
    forward  (router + route-fusion + attention)         mka_fused_attn_fwd
    backward (dQ, dK_l, dV_l, dW_r, db_r)                mka_fused_attn_bwd
    decode   (append one token, attend over the caches)  mka_fused_attn_decode
`value` = algorithmic attention flops of the step / step time, inputs resident in HBM.
The larger configurations (C3 long prefill, C5 training, C4 bandwidth-bound decode) are timed
with a few iterations each and reported under "workloads"; the roofline objects are measured
live with HIP events on the launch stream.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--quick] [--no-cpu]
prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E


def attn_pairs(Tq, S, causal=True):
    """Unmasked (row, slot) pairs per head: bottom-right aligned causal mask."""
    if not causal:
        return Tq * S
    off = S - Tq
    return Tq * off + Tq * (Tq + 1) // 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--quick", action="store_true", help="skip the larger workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB elementwise copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not provided "
              "(every (batch, head) is independent: the path would shard over batch x heads)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2603_20586_amd as mka  # raises if libmka.so is not built: no fallback
    import synth_inputs as si

    mka.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def time_region(fn, iters, warm):
        """Average ms per call, HIP events recorded on the stream the kernels are launched on."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record(stream)
        for _ in range(iters):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    # ------------------------------------------------------------------ the step (config C2)
    inp, cfg = si.config_inputs("C2", device=dev)
    B, H, T, d = cfg["B"], cfg["H"], cfg["Tq"], cfg["d"]
    inp["dO"] = torch.randn((B, H, T, d), device=dev,
                            generator=torch.Generator(dev).manual_seed(101)).bfloat16()
    G = torch.zeros((B, H, T, 3), device=dev)
    O = torch.empty_like(inp["Q"])
    LSE = torch.empty((B, H, T), device=dev)
    idx = torch.empty((B, H, T), dtype=torch.int32, device=dev)
    from paper_2603_20586_amd.binding import MKA_OP_BWD, MKA_OP_DECODE, _shape

    shp = _shape(inp["Q"], T, None, True, inp["scale"])
    ws_bwd = torch.empty(mka.mka_workspace_bytes(MKA_OP_BWD, shp), dtype=torch.uint8, device=dev)
    # decode caches of the same shape: the prefill's memories with room for the appended tokens
    n_app = args.steps + args.warmup + 64
    Kc = [torch.cat([k, torch.zeros((B, H, n_app, d), device=dev, dtype=k.dtype)], 2).contiguous()
          if l == 0 else k for l, k in enumerate(inp["K"])]
    Vc = [torch.cat([v, torch.zeros((B, H, n_app, d), device=dev, dtype=v.dtype)], 2).contiguous()
          if l == 0 else v for l, v in enumerate(inp["V"])]
    Gc = torch.zeros((B, H, T + n_app, 3), device=dev)
    qd, k1d, v1d = si.decode_step_inputs(B, H, d, 0, device=dev, seed=1)
    shp_dec = _shape(qd, T + n_app, None, False, inp["scale"])
    ws_dec = torch.empty(mka.mka_workspace_bytes(MKA_OP_DECODE, shp_dec), dtype=torch.uint8,
                         device=dev)
    Od = torch.empty_like(qd)
    len_dec = [T, T, T]

    def fwd():
        mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"], G=G,
                               causal=True, scale=inp["scale"], O=O, LSE=LSE, idx=idx)

    def fwd_kernel_only():  # gates given: exactly one kernel launch
        mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], None, None, G=G, causal=True,
                               scale=inp["scale"], O=O, LSE=LSE, want_idx=False)

    def bwd():
        mka.mka_fused_attn_bwd(inp["dO"], inp["Q"], inp["K"], inp["V"], G, O, LSE, inp["W_r"],
                               causal=True, scale=inp["scale"], workspace=ws_bwd)

    def dec():
        mka.mka_fused_attn_decode(qd, [k1d, None, None], [v1d, None, None], Kc, Vc, Gc, len_dec,
                                  inp["W_r"], inp["b_r"], scale=inp["scale"], workspace=ws_dec,
                                  O=Od, want_lse=False, want_idx=False)

    def step():
        fwd()
        bwd()
        dec()

    fwd()
    Gc[:, :, :T] = G  # gate cache of the prefilled slots
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    pairs = attn_pairs(T, T) * B * H
    fl_fwd, fl_bwd = 4 * d * pairs, 10 * d * pairs
    fl_dec = 4 * d * (T + 1) * B * H
    value = (fl_fwd + fl_bwd + fl_dec) / (ms_step * 1e-3) / 1e12

    # per-phase timings with HIP events on the launch stream
    len_dec[:] = [T, T, T]
    ms_fwd = time_region(fwd, args.steps, 2)
    ms_fwdk = time_region(fwd_kernel_only, args.steps, 2)
    ms_bwd = time_region(bwd, args.steps, 2)
    len_dec[:] = [T, T, T]

    def dec_fixed():
        len_dec[:] = [T, T, T]
        dec()

    ms_dec = time_region(dec_fixed, args.steps, 2)
    phases = {
        "fwd_ms": ms_fwd, "fwd_tflops": fl_fwd / ms_fwd / 1e9,
        "fwd_kernel_ms": ms_fwdk, "fwd_kernel_tflops": fl_fwd / ms_fwdk / 1e9,
        "bwd_ms": ms_bwd, "bwd_tflops": fl_bwd / ms_bwd / 1e9,
        "decode_ms": ms_dec,
        "decode_gbps": (6 * B * H * (T + 1) * d * 2 + 12 * B * H * (T + 1)) / ms_dec / 1e6,
        "tokens_per_s_prefill": B * T / (ms_fwd * 1e-3),
        "tokens_per_s_train": B * T / ((ms_fwd + ms_bwd) * 1e-3),
    }

    def roof_mfma(flops, ms, kernel):
        a = flops / ms / 1e9
        return {"kernel": kernel, "bound": "mfma", "achieved": a, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": a / PEAK_BF16_TFLOPS, "traffic": None}

    rooflines = {
        "C2_fwd": roof_mfma(fl_fwd, ms_fwdk, "fwd_bf16_kernel"),
        "C2_bwd": roof_mfma(fl_bwd, ms_bwd, "bwd_main_kernel + bwd_dq_kernel (+prep/finish/reduce in the events)"),
    }
    workloads = {}

    # ------------------------------------------------------------------ larger workloads
    if not args.quick:
        del Kc, Vc, Gc
        # C3: long prefill
        inp3, c3 = si.config_inputs("C3", device=dev)
        B3, H3, T3 = c3["B"], c3["H"], c3["Tq"]
        G3 = torch.zeros((B3, H3, T3, 3), device=dev)
        O3 = torch.empty_like(inp3["Q"])
        L3 = torch.empty((B3, H3, T3), device=dev)
        mka.mka_route(inp3["Q"], inp3["W_r"], inp3["b_r"], G=G3, want_idx=False)
        from paper_2603_20586_amd.binding import MKA_OP_FWD
        shp3 = _shape(inp3["Q"], T3, None, True, inp3["scale"])
        # the library recommends the materialised route here (Kf, Vf once to the workspace, then
        # attention over that stream); the folded route (fusion inside the attention kernel, no
        # workspace) is timed beside it
        ws3 = torch.empty(mka.mka_workspace_bytes(MKA_OP_FWD, shp3), dtype=torch.uint8, device=dev)
        assert ws3.numel() > 0
        ms3 = time_region(lambda: mka.mka_fused_attn_fwd(
            inp3["Q"], inp3["K"], inp3["V"], None, None, G=G3, causal=True, scale=inp3["scale"],
            O=O3, LSE=L3, want_idx=False, workspace=ws3), 5, 2)
        ms3f = time_region(lambda: mka.mka_fused_attn_fwd(
            inp3["Q"], inp3["K"], inp3["V"], None, None, G=G3, causal=True, scale=inp3["scale"],
            O=O3, LSE=L3, want_idx=False, materialise=False), 5, 2)
        fl3 = 4 * d * attn_pairs(T3, T3) * B3 * H3
        Kf3 = torch.empty_like(inp3["K"][0])
        Vf3 = torch.empty_like(inp3["V"][0])
        msk = time_region(lambda: mka.mka_fuse_kv(inp3["K"], inp3["V"], G3, Kf=Kf3, Vf=Vf3), 5, 2)
        del Kf3, Vf3, ws3
        workloads["C3_prefill_fwd"] = {
            "route": "materialised", "ms": ms3, "tflops": fl3 / ms3 / 1e9,
            "tokens_per_s": B3 * T3 / (ms3 * 1e-3), "prefuse_ms": msk,
            "prefuse_gbps": (8 * B3 * H3 * T3 * d * 2 + 12 * B3 * H3 * T3) / msk / 1e6}
        workloads["C3_prefill_fwd_folded"] = {"route": "folded", "ms": ms3f,
                                              "tflops": fl3 / ms3f / 1e9}
        rooflines["C3_fwd"] = roof_mfma(fl3, ms3, "prefuse_kernel + mix_bf16_kernel (both in the events)")
        rooflines["C3_fwd_folded"] = roof_mfma(fl3, ms3f, "fwd_bf16_kernel")
        # the same shape through the per-query gated mixture over the three memories (3x the
        # pairs) and through plain attention over one memory
        msm = time_region(lambda: mka.mka_mixture_attn_fwd(
            inp3["Q"], inp3["K"], inp3["V"], G3, causal=True, scale=inp3["scale"], O=O3, LSE=L3), 5, 2)
        msp = time_region(lambda: mka.mka_mixture_attn_fwd(
            inp3["Q"], [inp3["K"][0], None, None], [inp3["V"][0], None, None], None, causal=True,
            scale=inp3["scale"], O=O3, LSE=L3), 5, 2)
        # symbolic (full) MKA of Alg. 1 on the same memories: three attentions + a combine pass
        from paper_2603_20586_amd.binding import MKA_OP_FULL_MKA
        wsf = torch.empty(mka.mka_workspace_bytes(MKA_OP_FULL_MKA, shp3), dtype=torch.uint8, device=dev)
        msfull = time_region(lambda: mka.mka_full_attn_fwd(
            inp3["Q"], inp3["K"], inp3["V"], G3, causal=True, scale=inp3["scale"], O=O3,
            workspace=wsf), 5, 2)
        del wsf
        workloads["C3_full_mka_fwd"] = {"ms": msfull, "tflops": 3 * fl3 / msfull / 1e9,
                                        "vs_route_fused": msfull / ms3}
        workloads["C3_gated_mixture_fwd"] = {"ms": msm, "tflops": 3 * fl3 / msm / 1e9}
        workloads["C3_plain_attention_fwd"] = {"ms": msp, "tflops": fl3 / msp / 1e9}
        rooflines["C3_mixture"] = roof_mfma(3 * fl3, msm, "mix_bf16_kernel")
        del inp3, G3, O3, L3

        # C5: training forward + backward
        inp5, c5 = si.config_inputs("C5", device=dev)
        B5, H5, T5 = c5["B"], c5["H"], c5["Tq"]
        G5 = torch.zeros((B5, H5, T5, 3), device=dev)
        O5 = torch.empty_like(inp5["Q"])
        L5 = torch.empty((B5, H5, T5), device=dev)
        shp5 = _shape(inp5["Q"], T5, None, True, inp5["scale"])
        ws5 = torch.empty(mka.mka_workspace_bytes(MKA_OP_BWD, shp5), dtype=torch.uint8, device=dev)
        ws5f = torch.empty(max(256, mka.mka_workspace_bytes(MKA_OP_FWD, shp5)), dtype=torch.uint8,
                           device=dev)

        def f5():
            mka.mka_fused_attn_fwd(inp5["Q"], inp5["K"], inp5["V"], inp5["W_r"], inp5["b_r"], G=G5,
                                   causal=True, scale=inp5["scale"], O=O5, LSE=L5, want_idx=False,
                                   workspace=ws5f)

        grads5 = {}

        def b5():
            grads5["g"] = mka.mka_fused_attn_bwd(inp5["dO"], inp5["Q"], inp5["K"], inp5["V"], G5,
                                                 O5, L5, inp5["W_r"], causal=True,
                                                 scale=inp5["scale"], workspace=ws5)

        msf5 = time_region(f5, 3, 1)
        msb5 = time_region(b5, 3, 1)
        p5 = attn_pairs(T5, T5) * B5 * H5
        workloads["C5_train"] = {
            "fwd_ms": msf5, "bwd_ms": msb5, "fwd_tflops": 4 * d * p5 / msf5 / 1e9,
            "bwd_tflops": 10 * d * p5 / msb5 / 1e9,
            "fwd_bwd_tflops": 14 * d * p5 / (msf5 + msb5) / 1e9,
            "tokens_per_s": B5 * T5 / ((msf5 + msb5) * 1e-3)}
        rooflines["C5_bwd"] = roof_mfma(10 * d * p5, msb5,
                                        "bwd_main_kernel + bwd_dq_kernel (+prep/finish/reduce in the events)")
        del inp5, G5, O5, L5, ws5, ws5f, grads5
        torch.cuda.empty_cache()

        # C4: bandwidth-bound decode, 64 steps with an appended L1 entry per step
        c4 = si.CONFIGS["C4"]
        B4, H4, S0, nst = c4["B"], c4["H"], c4["S0"], c4["steps"]
        cc = si.decode_caches(B4, H4, d, S0, cap_extra=nst, device=dev, seed=c4["seed"])
        q4, k4, v4 = si.decode_step_inputs(B4, H4, d, 0, device=dev, seed=c4["seed"])
        shp4 = _shape(q4, S0 + nst, None, False, cc["scale"])
        ws4 = torch.empty(mka.mka_workspace_bytes(MKA_OP_DECODE, shp4), dtype=torch.uint8,
                          device=dev)
        O4 = torch.empty_like(q4)
        ln4 = list(cc["len"])

        def run64():
            ln4[:] = [S0, S0, S0]
            for _ in range(nst):
                mka.mka_fused_attn_decode(q4, [k4, None, None], [v4, None, None], cc["Kc"],
                                          cc["Vc"], cc["Gc"], ln4, cc["W_r"], cc["b_r"],
                                          scale=cc["scale"], workspace=ws4, O=O4, want_lse=False,
                                          want_idx=False)

        ms64 = time_region(run64, 2, 1)
        ms4 = ms64 / nst
        s_avg = S0 + (nst + 1) / 2
        bytes4 = 6 * B4 * H4 * s_avg * d * 2 + 12 * B4 * H4 * s_avg
        gbps = bytes4 / ms4 / 1e6
        workloads["C4_decode"] = {"ms_per_step": ms4, "gbps": gbps,
                                  "tokens_per_s": B4 / (ms4 * 1e-3), "steps": nst}
        rooflines["C4_decode"] = {"kernel": "decode_split_kernel (+append/combine in the events)",
                                  "bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS,
                                  "unit": "GB/s", "frac": gbps / PEAK_HBM_GBPS, "traffic": None}
        # the same caches with hard top-1 gates (one level per slot): the kernel loads only the
        # selected level's rows, a third of the K / V bytes
        sel = torch.randint(0, 3, (B4, H4, S0), device=dev)
        cc["Gc"].zero_()
        cc["Gc"][:, :, :S0] = torch.nn.functional.one_hot(sel, 3).to(torch.float32)
        del sel

        def run64_top1():
            ln4[:] = [S0, S0, S0]
            for _ in range(nst):
                mka.mka_fused_attn_decode(q4, [k4, None, None], [v4, None, None], cc["Kc"],
                                          cc["Vc"], cc["Gc"], ln4, cc["W_r"], cc["b_r"],
                                          scale=cc["scale"], workspace=ws4, O=O4, want_lse=False,
                                          want_idx=False, routing=3)

        ms4h = time_region(run64_top1, 2, 1) / nst
        bytes4h = 2 * B4 * H4 * s_avg * d * 2 + 12 * B4 * H4 * s_avg
        workloads["C4_decode_top1_routing"] = {"ms_per_step": ms4h, "gbps": bytes4h / ms4h / 1e6,
                                               "vs_soft_routing": ms4 / ms4h}
        del cc, ws4
        torch.cuda.empty_cache()
        # the same decode shape over the fused KV cache in pages (one K and one V stream: a third
        # of the bytes), shuffled page table, one step at S0 slots
        P4 = 128
        npg = (S0 + P4 - 1) // P4
        g4 = torch.Generator(device=dev).manual_seed(5)
        Kp4 = torch.randn((B4 * npg, H4, P4, d), generator=g4, device=dev, dtype=torch.float32).to(torch.bfloat16) \
            if B4 * npg * H4 * P4 * d < (1 << 31) else None
        if Kp4 is None:
            Kp4 = torch.empty((B4 * npg, H4, P4, d), device=dev, dtype=torch.bfloat16)
            for i in range(0, B4 * npg, 64):
                Kp4[i:i + 64] = torch.randn((min(64, B4 * npg - i), H4, P4, d), generator=g4,
                                            device=dev).to(torch.bfloat16)
        Vp4 = Kp4.flip(0).contiguous()
        tab4 = torch.randperm(B4 * npg, generator=g4, device=dev).reshape(B4, npg).to(torch.int32)
        sl4 = torch.full((B4,), S0, dtype=torch.int32, device=dev)
        wsp = torch.empty(64 * B4 * H4 * (d + 2) * 4, dtype=torch.uint8, device=dev)
        msp4 = time_region(lambda: mka.mka_paged_fused_decode(
            q4, Kp4, Vp4, tab4, sl4, scale=1.0 / math.sqrt(d), O=O4, want_lse=False, workspace=wsp), 5, 2)
        bytesp = 2 * B4 * H4 * S0 * d * 2
        workloads["C4_paged_fused_decode"] = {"ms_per_step": msp4, "gbps": bytesp / msp4 / 1e6,
                                              "page_size": P4, "vs_raw_cache_decode": ms4 / msp4}
        del Kp4, Vp4, wsp
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ measured ceilings
    # a pure MFMA loop and a streaming read, written in this library: what the part sustains,
    # to quote beside the vendor peaks (`frac_of_ceiling` in every roofline line)
    ceilings = None
    if not args.quick:
        cbuf = torch.empty(1 << 32, dtype=torch.int32, device=dev).fill_(1)  # 16 GiB
        ms_r = time_region(lambda: mka.mka_ceiling_read(cbuf), 5, 2)
        cout = torch.empty(2048 * 512, dtype=torch.float32, device=dev)
        fl = [0.0]

        def run_mfma():
            fl[0] = mka.mka_ceiling_mfma(cout, 2048, 2000)
        ms_m = time_region(run_mfma, 5, 2)
        ceilings = {"mfma_bf16_tflops": fl[0] / ms_m / 1e9,
                    "hbm_read_gbps": cbuf.numel() * 4 / ms_r / 1e6,
                    "how": "mka_ceiling_mfma: 2048 workgroups x 8 waves x 8000 independent "
                           "32x32x16 bf16 MFMAs; mka_ceiling_read: 16 GiB, 16-byte non-temporal loads, 8 per lane in "
                           "flight (a plain loop: a tuned kernel can sit a few % above it)"}
        for r in rooflines.values():
            top = ceilings["mfma_bf16_tflops"] if r["bound"] == "mfma" else ceilings["hbm_read_gbps"]
            r["frac_of_ceiling"] = r["achieved"] / top
        del cout, cbuf
        torch.cuda.empty_cache()

    if args.calibrate_copy:
        # plain copy of known size: reads 1 GiB, writes 1 GiB (scales rocprofv3 FETCH/WRITE_SIZE)
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # HBM traffic per launch measured offline with rocprofv3 --pmc (see profiles/); filled in
    # from the committed summary when present
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            traffic = json.load(f)
        for key, r in rooflines.items():
            t = traffic.get(key)
            if t is not None:
                r["traffic"] = t
    except (OSError, ValueError):
        pass

    # dominant kernel of the step = the one with the largest share of the step time
    dom = "C2_bwd" if ms_bwd >= ms_fwd else "C2_fwd"
    roofline = dict(rooflines[dom])

    # ------------------------------------------------------------------ CPU baseline (oracle)
    cpu_baseline = None
    if not args.no_cpu:
        import oracle

        # the whole forward + backward of the step (all B*H heads; the oracle runs one head per
        # thread): a few seconds of wall time, some tens of core-seconds
        nh = B * H
        cq = inp["Q"].cpu()
        ck = [k.cpu() for k in inp["K"]]
        cv = [v.cpu() for v in inp["V"]]
        cdo = inp["dO"].cpu()
        w, b = inp["W_r"].cpu(), inp["b_r"].cpu()
        t0 = time.perf_counter()
        Oc, Lc, Gcpu, _ = oracle.fwd_routed(cq, ck, cv, w, b, causal=True, tau=inp["scale"])
        oracle.bwd(cdo, cq, ck, cv, Gcpu, w, causal=True, tau=inp["scale"])
        dt = time.perf_counter() - t0
        fl = 14 * d * attn_pairs(T, T) * nh
        cpu_baseline = {"value": fl / dt / 1e12, "unit": "TFLOP/s",
                        "cores": min(oracle.num_threads(), nh), "kind": "oracle", "seconds": dt,
                        "sample": f"forward+backward of all {nh} (batch, head) pairs of the C2 "
                                  f"workload (the decode leg of the step is not included), fp64, "
                                  f"OpenMP over heads"}

    out = {
        "metric": "FastMKA attn TFLOP/s (fwd/bwd) + decode HBM GB/s, %roofline, 1 MI355X",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C2 prefill shape B=4 H=16 d=128 T=2048 causal bf16: "
                               "fwd + bwd + one decode step per step"},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "ceilings": ceilings, "phases": phases,
        "rooflines": rooflines, "workloads": workloads,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
