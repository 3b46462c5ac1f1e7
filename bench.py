#!/usr/bin/env python3
"""Benchmark of the FastMKA route-fused attention hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input at the largest
single-GPU configurations of the benchmark:
    training forward   config C5 (B=8 H=16 d=128 T=4096 causal bf16)   mka_fused_attn_fwd
                       router + route-fusion + attention
    training backward  config C5: dQ, dK_l, dV_l, dW_r, db_r           mka_fused_attn_bwd
    decode             config C4 (B=16 H=32 d=128, three raw caches of 32768 slots): append one
                       token, attend over the caches                   mka_fused_attn_decode
`value` = algorithmic attention flops of the step / step time, inputs resident in HBM.  The
roofline objects are measured live with HIP events on the launch stream.  The other
configurations (C2 prefill, C3 long prefill, the 64-step C4 run, the paged fused cache up to 128K
slots, the widened rows) are timed beside it and reported under "workloads" / "rooflines".

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only LIST] [--no-cpu]
prints ONE JSON line.  --only takes a comma-separated subset of
step,C2,C3,C3mix,C3full,C4,C5,paged,paged128K,refs (default: all) so that a profiler run can cover one workload.
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
GROUPS = ("step", "C2", "C3", "C3mix", "C3full", "C4", "C5", "paged", "paged128K", "refs")


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
    ap.add_argument("--only", default=",".join(GROUPS),
                    help="comma-separated subset of " + ",".join(GROUPS))
    ap.add_argument("--quick", action="store_true", help="the step only (same as --only step)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB elementwise copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not provided "
              "(every (batch, head) is independent: the path would shard over batch x heads)",
              file=sys.stderr)
        sys.exit(2)
    only = {"step"} if args.quick else {g.strip() for g in args.only.split(",") if g.strip()}
    bad = only - set(GROUPS)
    if bad:
        print(f"bench.py: unknown --only entries {sorted(bad)}", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2603_20586_amd as mka  # raises if libmka.so is not built: no fallback
    import synth_inputs as si
    from paper_2603_20586_amd.binding import (MKA_OP_BWD, MKA_OP_BWD_RECOMPUTE, MKA_OP_DECODE,
                                              MKA_OP_FULL_MKA, MKA_OP_FWD, _shape)

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

    def ws(nbytes):
        return torch.empty(max(256, nbytes), dtype=torch.uint8, device=dev)

    def roof_mfma(flops, ms, kernel):
        a = flops / ms / 1e9
        return {"kernel": kernel, "bound": "mfma", "achieved": a, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": a / PEAK_BF16_TFLOPS, "traffic": None}

    def roof_hbm(nbytes, ms, kernel):
        a = nbytes / ms / 1e6
        return {"kernel": kernel, "bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBPS,
                "unit": "GB/s", "frac": a / PEAK_HBM_GBPS, "traffic": None}

    d = 128
    rooflines, workloads, phases = {}, {}, {}
    value = ms_step = None
    roofline = None
    cpu_baseline = None

    # ------------------------------------------------------------ C5 (training) and C4 (decode)
    need5 = bool(only & {"step", "C5"})
    need4 = bool(only & {"step", "C4"})
    if need5:
        inp5, c5 = si.config_inputs("C5", device=dev)
        B5, H5, T5 = c5["B"], c5["H"], c5["Tq"]
        G5 = torch.zeros((B5, H5, T5, 3), device=dev)
        O5 = torch.empty_like(inp5["Q"])
        L5 = torch.empty((B5, H5, T5), device=dev)
        shp5 = _shape(inp5["Q"], T5, None, True, inp5["scale"])
        ws5b = ws(mka.mka_workspace_bytes(MKA_OP_BWD, shp5))
        ws5f = ws(mka.mka_workspace_bytes(MKA_OP_FWD, shp5))   # the library's recommended route
        p5 = attn_pairs(T5, T5) * B5 * H5
        fl5f, fl5b = 4 * d * p5, 10 * d * p5

        def f5():
            mka.mka_fused_attn_fwd(inp5["Q"], inp5["K"], inp5["V"], inp5["W_r"], inp5["b_r"], G=G5,
                                   causal=True, scale=inp5["scale"], O=O5, LSE=L5, want_idx=False,
                                   workspace=ws5f)

        def f5_folded():
            mka.mka_fused_attn_fwd(inp5["Q"], inp5["K"], inp5["V"], inp5["W_r"], inp5["b_r"], G=G5,
                                   causal=True, scale=inp5["scale"], O=O5, LSE=L5, want_idx=False,
                                   materialise=False)

        def b5():
            mka.mka_fused_attn_bwd(inp5["dO"], inp5["Q"], inp5["K"], inp5["V"], G5, O5, L5,
                                   inp5["W_r"], causal=True, scale=inp5["scale"], workspace=ws5b)

    if need4:
        c4 = si.CONFIGS["C4"]
        B4, H4, S0, nst = c4["B"], c4["H"], c4["S0"], c4["steps"]
        cc = si.decode_caches(B4, H4, d, S0, cap_extra=nst, device=dev, seed=c4["seed"])
        q4, k4, v4 = si.decode_step_inputs(B4, H4, d, 0, device=dev, seed=c4["seed"])
        shp4 = _shape(q4, S0 + nst, None, False, cc["scale"])
        ws4 = ws(mka.mka_workspace_bytes(MKA_OP_DECODE, shp4))
        O4 = torch.empty_like(q4)
        ln4 = list(cc["len"])

        def dec4(routing=0):
            mka.mka_fused_attn_decode(q4, [k4, None, None], [v4, None, None], cc["Kc"], cc["Vc"],
                                      cc["Gc"], ln4, cc["W_r"], cc["b_r"], scale=cc["scale"],
                                      workspace=ws4, O=O4, want_lse=False, want_idx=False,
                                      routing=routing)

        def dec4_first():   # the step's decode leg: always the token after the S0 cached ones
            ln4[:] = [S0, S0, S0]
            dec4()

        bytes4_first = 6 * B4 * H4 * (S0 + 1) * d * 2 + 12 * B4 * H4 * (S0 + 1)
        fl4_first = 4 * d * (S0 + 1) * B4 * H4

    if "step" in only:
        def step():
            f5()
            b5()
            dec4_first()

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
        value = (fl5f + fl5b + fl4_first) / (ms_step * 1e-3) / 1e12
        # the legs of the step, each between HIP events on the launch stream
        ms_f = time_region(f5, args.steps, 2)
        ms_b = time_region(b5, args.steps, 2)
        ms_d = time_region(dec4_first, args.steps, 2)
        phases = {
            "C5_fwd_ms": ms_f, "C5_fwd_tflops": fl5f / ms_f / 1e9,
            "C5_bwd_ms": ms_b, "C5_bwd_tflops": fl5b / ms_b / 1e9,
            "C5_fwd_bwd_tflops": (fl5f + fl5b) / (ms_f + ms_b) / 1e9,
            "C5_tokens_per_s_train": B5 * T5 / ((ms_f + ms_b) * 1e-3),
            "C4_decode_ms": ms_d, "C4_decode_gbps": bytes4_first / ms_d / 1e6,
            "C4_tokens_per_s_decode": B4 / (ms_d * 1e-3),
        }
        rooflines["C5_fwd"] = roof_mfma(fl5f, ms_f, "route_kernel + prefuse_kernel + mix_bf16_kernel "
                                                    "(all in the events)")
        rooflines["C5_bwd"] = roof_mfma(fl5b, ms_b, "bwd_main_kernel + bwd_dqg_kernel "
                                                    "(+prep/wpart/reduce in the events)")
        rooflines["C4_decode_step"] = roof_hbm(bytes4_first, ms_d,
                                               "decode_split_kernel (+append/combine in the events)")
        # dominant kernel of the step = the launch with the largest share of the step time
        legs = {"C5_fwd": ms_f, "C5_bwd": ms_b, "C4_decode_step": ms_d}
        dom = max(legs, key=legs.get)

    if "C5" in only:
        msf5 = time_region(f5, 5, 2)
        msf5f = time_region(f5_folded, 5, 2)
        msb5 = time_region(b5, 5, 2)
        ws5r = ws(mka.mka_workspace_bytes(MKA_OP_BWD_RECOMPUTE, shp5))
        msb5r = time_region(lambda: mka.mka_fused_attn_bwd(
            inp5["dO"], inp5["Q"], inp5["K"], inp5["V"], G5, O5, L5, inp5["W_r"], causal=True,
            scale=inp5["scale"], workspace=ws5r), 5, 2)
        del ws5r
        workloads["C5_train"] = {
            "fwd_ms": msf5, "fwd_folded_ms": msf5f, "bwd_ms": msb5,
            "bwd_recompute_route_ms": msb5r, "bwd_recompute_route_tflops": fl5b / msb5r / 1e9,
            "fwd_tflops": fl5f / msf5 / 1e9, "fwd_folded_tflops": fl5f / msf5f / 1e9,
            "bwd_tflops": fl5b / msb5 / 1e9,
            "fwd_bwd_tflops": (fl5f + fl5b) / (msf5 + msb5) / 1e9,
            "tokens_per_s": B5 * T5 / ((msf5 + msb5) * 1e-3)}
        rooflines.setdefault("C5_fwd", roof_mfma(fl5f, msf5, "route_kernel + prefuse_kernel + "
                                                             "mix_bf16_kernel (all in the events)"))
        rooflines["C5_fwd_folded"] = roof_mfma(fl5f, msf5f, "route_kernel + fwd_bf16_kernel")
        rooflines.setdefault("C5_bwd", roof_mfma(fl5b, msb5, "bwd_main_kernel + bwd_dqg_kernel "
                                                             "(+prep/wpart/reduce in the events)"))
        rooflines["C5_bwd_recompute"] = roof_mfma(fl5b, msb5r, "bwd_main_kernel + bwd_dq_kernel "
                                                               "(+prep/wpart/reduce in the events)")

    if "C4" in only:
        # the configured run: 64 decode steps with an appended L1 entry per step
        def run64(routing=0):
            ln4[:] = [S0, S0, S0]
            for _ in range(nst):
                dec4(routing)

        ms4 = time_region(run64, 2, 1) / nst
        s_avg = S0 + (nst + 1) / 2
        bytes4 = 6 * B4 * H4 * s_avg * d * 2 + 12 * B4 * H4 * s_avg
        workloads["C4_decode"] = {"ms_per_step": ms4, "gbps": bytes4 / ms4 / 1e6,
                                  "tokens_per_s": B4 / (ms4 * 1e-3), "steps": nst}
        rooflines["C4_decode"] = roof_hbm(bytes4, ms4, "decode_split_kernel (+append/combine in the events)")
        # the same caches with hard top-1 gates (one level per slot): the kernel loads only the
        # selected level's rows, a third of the K / V bytes
        Gsave = cc["Gc"].clone()
        sel = torch.randint(0, 3, (B4, H4, S0), device=dev)
        cc["Gc"].zero_()
        cc["Gc"][:, :, :S0] = torch.nn.functional.one_hot(sel, 3).to(torch.float32)
        del sel
        ms4h = time_region(lambda: run64(3), 2, 1) / nst
        bytes4h = 2 * B4 * H4 * s_avg * d * 2 + 12 * B4 * H4 * s_avg
        workloads["C4_decode_top1_routing"] = {"ms_per_step": ms4h, "gbps": bytes4h / ms4h / 1e6,
                                               "vs_soft_routing": ms4 / ms4h}
        cc["Gc"].copy_(Gsave)
        del Gsave

    # ------------------------------------------------------------ CPU baseline (oracle)
    # Taken while the step's inputs are still resident: the oracle, as it stands, on a bounded
    # sample of the step's own workload.
    if "step" in only and not args.no_cpu:
        import oracle

        nh5 = H5                       # batch entry 0 of C5: 16 of the 128 (batch, head) pairs
        s0 = slice(0, 1)
        cq, cdo = inp5["Q"][s0].cpu(), inp5["dO"][s0].cpu()
        ck = [k[s0].cpu() for k in inp5["K"]]
        cv = [v[s0].cpu() for v in inp5["V"]]
        w5, b5r = inp5["W_r"].cpu(), inp5["b_r"].cpu()
        t0 = time.perf_counter()
        _, _, Gcpu, _ = oracle.fwd_routed(cq, ck, cv, w5, b5r, causal=True, tau=inp5["scale"])
        oracle.bwd(cdo, cq, ck, cv, Gcpu, w5, causal=True, tau=inp5["scale"])
        dt5 = time.perf_counter() - t0
        fl_s5 = 14 * d * attn_pairs(T5, T5) * nh5
        nh4 = 8                        # heads (0, 0..7) of the C4 decode step
        pick = lambda x: x[0:1, 0:nh4]  # noqa: E731
        f64 = lambda x: x.float().cpu().double().numpy().copy()  # noqa: E731
        Kc_o = [f64(pick(x)) for x in cc["Kc"]]
        Vc_o = [f64(pick(x)) for x in cc["Vc"]]
        Gc_o = f64(pick(cc["Gc"]))
        t0 = time.perf_counter()
        oracle.decode(pick(q4).cpu(), [pick(k4).cpu(), None, None], [pick(v4).cpu(), None, None],
                      Kc_o, Vc_o, Gc_o, [S0, S0, S0], cc["W_r"].cpu(), cc["b_r"].cpu(),
                      tau=cc["scale"])
        dt4 = time.perf_counter() - t0
        fl_s4 = 4 * d * (S0 + 1) * nh4
        del Kc_o, Vc_o, Gc_o
        cpu_baseline = {
            "value": (fl_s5 + fl_s4) / (dt5 + dt4) / 1e12, "unit": "TFLOP/s",
            "cores": min(oracle.num_threads(), nh5), "kind": "oracle", "seconds": dt5 + dt4,
            "sample": f"forward+backward of the {nh5} heads of batch entry 0 of C5 ({dt5:.1f} s; the "
                      f"other 7 entries are the same work) plus the decode step of {nh4} of the 512 "
                      f"(batch, head) pairs of C4 ({dt4:.2f} s); fp64, OpenMP over heads; the same "
                      f"flop count as `value` (attention flops of the sample / wall time)",
            "C5_fwd_bwd_tflops": fl_s5 / dt5 / 1e12,
            "C4_decode_gbps_bf16_equivalent": (6 * nh4 * (S0 + 1) * d * 2) / dt4 / 1e9}

    if need5:
        del inp5, G5, O5, L5, ws5b, ws5f
    if need4:
        del cc, ws4
    torch.cuda.empty_cache()

    # ------------------------------------------------------------ C2: short prefill shape
    if "C2" in only:
        inp, cfg = si.config_inputs("C2", device=dev)
        B, H, T = cfg["B"], cfg["H"], cfg["Tq"]
        inp["dO"] = torch.randn((B, H, T, d), device=dev,
                                generator=torch.Generator(dev).manual_seed(101)).bfloat16()
        G = torch.zeros((B, H, T, 3), device=dev)
        O = torch.empty_like(inp["Q"])
        LSE = torch.empty((B, H, T), device=dev)
        shp = _shape(inp["Q"], T, None, True, inp["scale"])
        ws_bwd = ws(mka.mka_workspace_bytes(MKA_OP_BWD, shp))
        ws_mat = ws(mka.mka_workspace_bytes(4, shp))
        mka.mka_route(inp["Q"], inp["W_r"], inp["b_r"], G=G, want_idx=False)

        def fwd2(**kw):  # gates given: the attention launch(es) only
            mka.mka_fused_attn_fwd(inp["Q"], inp["K"], inp["V"], None, None, G=G, causal=True,
                                   scale=inp["scale"], O=O, LSE=LSE, want_idx=False, **kw)

        def bwd2():
            mka.mka_fused_attn_bwd(inp["dO"], inp["Q"], inp["K"], inp["V"], G, O, LSE, inp["W_r"],
                                   causal=True, scale=inp["scale"], workspace=ws_bwd)

        ms_ff = time_region(lambda: fwd2(materialise=False), 20, 3)
        ms_fm = time_region(lambda: fwd2(workspace=ws_mat), 20, 3)
        ms_fd = time_region(lambda: mka.mka_fused_attn_fwd(
            inp["Q"], inp["K"], inp["V"], inp["W_r"], inp["b_r"], G=G, causal=True,
            scale=inp["scale"], O=O, LSE=LSE, want_idx=False), 20, 3)
        ms_b = time_region(bwd2, 20, 3)
        fl2 = 4 * d * attn_pairs(T, T) * B * H
        workloads["C2_prefill"] = {
            "fwd_default_ms": ms_fd, "fwd_default_tflops": fl2 / ms_fd / 1e9,
            "fwd_folded_kernel_ms": ms_ff, "fwd_folded_kernel_tflops": fl2 / ms_ff / 1e9,
            "fwd_materialised_ms": ms_fm, "fwd_materialised_tflops": fl2 / ms_fm / 1e9,
            "bwd_ms": ms_b, "bwd_tflops": 2.5 * fl2 / ms_b / 1e9,
            "tokens_per_s_prefill": B * T / (ms_fd * 1e-3)}
        rooflines["C2_fwd"] = roof_mfma(fl2, ms_ff, "fwd_bf16_kernel")
        rooflines["C2_fwd_materialised"] = roof_mfma(fl2, ms_fm, "prefuse_kernel + mix_bf16_kernel")
        rooflines["C2_bwd"] = roof_mfma(2.5 * fl2, ms_b, "bwd_main_kernel + bwd_dqg_kernel "
                                                         "(+prep/wpart/reduce in the events)")
        del inp, G, O, LSE, ws_bwd, ws_mat
        torch.cuda.empty_cache()

    # ------------------------------------------------------------ C3: long prefill
    if "C3" in only:
        inp3, c3 = si.config_inputs("C3", device=dev)
        B3, H3, T3 = c3["B"], c3["H"], c3["Tq"]
        G3 = torch.zeros((B3, H3, T3, 3), device=dev)
        O3 = torch.empty_like(inp3["Q"])
        L3 = torch.empty((B3, H3, T3), device=dev)
        mka.mka_route(inp3["Q"], inp3["W_r"], inp3["b_r"], G=G3, want_idx=False)
        shp3 = _shape(inp3["Q"], T3, None, True, inp3["scale"])
        # the library recommends the materialised route here (Kf, Vf once to the workspace, then
        # attention over that stream); the folded route is timed beside it
        ws3 = ws(mka.mka_workspace_bytes(MKA_OP_FWD, shp3))
        assert ws3.numel() > 256
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
        msp = time_region(lambda: mka.mka_mixture_attn_fwd(
            inp3["Q"], [Kf3, None, None], [Vf3, None, None], None, causal=True,
            scale=inp3["scale"], O=O3, LSE=L3), 5, 2)
        del Kf3, Vf3, ws3
        workloads["C3_prefill_fwd"] = {
            "route": "materialised", "ms": ms3, "tflops": fl3 / ms3 / 1e9,
            "tokens_per_s": B3 * T3 / (ms3 * 1e-3), "prefuse_ms": msk,
            "prefuse_gbps": (8 * B3 * H3 * T3 * d * 2 + 12 * B3 * H3 * T3) / msk / 1e6}
        workloads["C3_prefill_fwd_folded"] = {"route": "folded", "ms": ms3f,
                                              "tflops": fl3 / ms3f / 1e9}
        workloads["C3_plain_attention_fwd"] = {"ms": msp, "tflops": fl3 / msp / 1e9}
        rooflines["C3_fwd"] = roof_mfma(fl3, ms3, "prefuse_kernel + mix_bf16_kernel (both in the events)")
        rooflines["C3_fwd_folded"] = roof_mfma(fl3, ms3f, "fwd_bf16_kernel")
        rooflines["C3_attention_core"] = roof_mfma(fl3, msp, "mix_bf16_kernel (one memory)")
        del inp3, G3, O3, L3
        torch.cuda.empty_cache()

    # the C3 shape through the per-query gated mixture over the three memories (3x the pairs) and
    # through symbolic (full) MKA: three attentions + a combine pass
    if only & {"C3mix", "C3full"}:
        inp3, c3 = si.config_inputs("C3", device=dev)
        B3, H3, T3 = c3["B"], c3["H"], c3["Tq"]
        G3 = torch.zeros((B3, H3, T3, 3), device=dev)
        O3 = torch.empty_like(inp3["Q"])
        L3 = torch.empty((B3, H3, T3), device=dev)
        mka.mka_route(inp3["Q"], inp3["W_r"], inp3["b_r"], G=G3, want_idx=False)
        shp3 = _shape(inp3["Q"], T3, None, True, inp3["scale"])
        fl3 = 4 * d * attn_pairs(T3, T3) * B3 * H3
        if "C3mix" in only:
            msm = time_region(lambda: mka.mka_mixture_attn_fwd(
                inp3["Q"], inp3["K"], inp3["V"], G3, causal=True, scale=inp3["scale"], O=O3, LSE=L3), 5, 2)
            workloads["C3_gated_mixture_fwd"] = {"ms": msm, "tflops": 3 * fl3 / msm / 1e9}
            rooflines["C3_mixture"] = roof_mfma(3 * fl3, msm, "mix_bf16_kernel (three memories)")
        if "C3full" in only:
            wsf = ws(mka.mka_workspace_bytes(MKA_OP_FULL_MKA, shp3))
            msfull = time_region(lambda: mka.mka_full_attn_fwd(
                inp3["Q"], inp3["K"], inp3["V"], G3, causal=True, scale=inp3["scale"], O=O3,
                workspace=wsf), 5, 2)
            del wsf
            workloads["C3_full_mka_fwd"] = {"ms": msfull, "tflops": 3 * fl3 / msfull / 1e9}
            if "C3_prefill_fwd" in workloads:
                workloads["C3_full_mka_fwd"]["vs_route_fused"] = msfull / workloads["C3_prefill_fwd"]["ms"]
        del inp3, G3, O3, L3
        torch.cuda.empty_cache()

    # ------------------------------------------------------------ paged fused-KV cache decode
    if only & {"paged", "paged128K"}:
        # the decode shape of C4 over the fused cache (one K and one V stream: a third of the raw
        # bytes) in pages of 128 slots behind a shuffled page table, at 32K slots and at the
        # context length the paper pages for (128K)
        B4, H4, P4 = 16, 32, 128
        g4 = torch.Generator(device=dev).manual_seed(5)
        q4p = torch.randn((B4, H4, 1, d), generator=g4, device=dev).to(torch.bfloat16)
        O4p = torch.empty_like(q4p)
        wsp = ws(64 * B4 * H4 * (d + 2) * 4)
        for Sp in [x for g, x in (("paged", 32768), ("paged128K", 131072)) if g in only]:
            npg = Sp // P4
            Kp4 = torch.empty((B4 * npg, H4, P4, d), device=dev, dtype=torch.bfloat16)
            for i in range(0, B4 * npg, 256):
                Kp4[i:i + 256] = torch.randn((min(256, B4 * npg - i), H4, P4, d), generator=g4,
                                             device=dev).to(torch.bfloat16)
            Vp4 = Kp4.flip(0).contiguous()
            tab4 = torch.randperm(B4 * npg, generator=g4, device=dev).reshape(B4, npg).to(torch.int32)
            sl4 = torch.full((B4,), Sp, dtype=torch.int32, device=dev)
            msp4 = time_region(lambda: mka.mka_paged_fused_decode(
                q4p, Kp4, Vp4, tab4, sl4, scale=1.0 / math.sqrt(d), O=O4p, want_lse=False,
                workspace=wsp), 5, 2)
            bytesp = 2 * B4 * H4 * Sp * d * 2
            key = f"paged_fused_decode_{Sp // 1024}K"
            workloads[key] = {"ms_per_step": msp4, "gbps": bytesp / msp4 / 1e6, "page_size": P4,
                              "slots": Sp, "tokens_per_s": B4 / (msp4 * 1e-3)}
            rooflines[key] = roof_hbm(bytesp, msp4, "paged_split_kernel (+combine in the events)")
            del Kp4, Vp4, tab4, sl4
            torch.cuda.empty_cache()
        if "C4_decode" in workloads and "paged_fused_decode_32K" in workloads:
            workloads["paged_fused_decode_32K"]["vs_raw_cache_decode"] = \
                workloads["C4_decode"]["ms_per_step"] / workloads["paged_fused_decode_32K"]["ms_per_step"]
        del wsp

    # ------------------------------------------------------------ reference micro-benchmarks
    # a pure MFMA loop and a streaming read (libmka_measure.so, not the product library): what the
    # part sustains in this run, to quote beside the vendor peaks (`frac_of_reference`)
    references = None
    if "refs" in only:
        from paper_2603_20586_amd import measure

        cbuf = torch.empty(6 << 30, dtype=torch.int32, device=dev).fill_(1)  # 24 GiB
        rd = [0]

        def run_read():
            rd[0] = measure.stream_read(cbuf)
        ms_r = time_region(run_read, 5, 2)
        cout = torch.empty(2048 * 512, dtype=torch.float32, device=dev)
        fl = [0.0]

        def run_mfma():
            fl[0] = measure.mfma_loop(cout, 2048, 2000)
        ms_m = time_region(run_mfma, 5, 2)
        # the same loop on operands drawn like the workloads' (N(0,1) in bf16): the clock under
        # matrix load is set by the board's power management, and the power of an MFMA depends on
        # its operand bits, so this - not the loop on small integers - is what the matrix pipe
        # alone sustains on such data; 20 launches before the timed ones let the clock settle
        gen = torch.Generator(device=dev).manual_seed(11)
        frags = torch.randn(measure.FRAG_BYTES // 2, device=dev, generator=gen).to(torch.bfloat16)
        fld = [0.0]

        def run_mfma_data():
            fld[0] = measure.mfma_loop_data(cout, frags, 2048, 250)
        ms_d = time_region(run_mfma_data, 20, 20)
        references = {"mfma_loop_bf16_tflops": fl[0] / ms_m / 1e9,
                      "mfma_loop_bf16_normal_data_tflops": fld[0] / ms_d / 1e9,
                      "stream_read_gbps": rd[0] / ms_r / 1e6,
                      "how": "mka_measure_mfma_loop: 2048 workgroups x 8 waves x 8000 independent "
                             "32x32x16 bf16 MFMAs on small-integer operands; mka_measure_mfma_loop_data: "
                             "the same number of MFMAs on eight A and eight B fragments per lane drawn "
                             "N(0,1) (power-limited clock); mka_measure_stream_read: 24 GiB as six interleaved "
                             "streams, 16-byte non-temporal loads, 24 per lane in flight (references, "
                             "not bounds: a kernel can sit a few % above the read loop)"}
        for r in rooflines.values():
            if r["bound"] == "mfma":
                r["frac_of_reference"] = r["achieved"] / references["mfma_loop_bf16_tflops"]
                r["frac_of_normal_data_reference"] = r["achieved"] / references["mfma_loop_bf16_normal_data_tflops"]
            else:
                r["frac_of_reference"] = r["achieved"] / references["stream_read_gbps"]
        del cout, cbuf, frags
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

    if "step" in only:
        roofline = dict(rooflines[dom])

    out = {
        "metric": "FastMKA attn TFLOP/s (fwd/bwd) + decode HBM GB/s, %roofline, 1 MI355X",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C5 training forward + backward (B=8 H=16 d=128 T=4096 causal bf16) "
                               "plus one C4 decode step (B=16 H=32 d=128, append one token and attend "
                               "over three raw caches of 32768 slots) per step",
                   "only": sorted(only)},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "references": references,
        "phases": phases, "rooflines": rooflines, "workloads": workloads,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
