"""What the board's power management does to the MFMA kernels: throughput and board power of
the reference MFMA loops and of the attention core, on operands that are zero and on operands
drawn like the workloads' (N(0,1) in bf16), each in a steady loop of back-to-back launches.

    python -m paper_2603_20586_amd.measure.power_probe [--core-only]

Prints one line per case (--core-only: just the attention core, e.g. for a library built with one
of the MKA_ELIM / MKA_DOUBLE measurement flags).  Power is the hwmon `power1_input` figure of the card (read from sysfs
while the launches are queued), so it is the sensor's own average, not an integral.  A
measurement helper: nothing in the product path imports it.
"""
from __future__ import annotations

import glob
import math
import sys


def _power_reader():
    for h in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
        for name in ("power1_input", "power1_average"):
            path = f"{h}/{name}"
            try:
                int(open(path).read())
            except (OSError, ValueError):
                continue
            cap = None
            try:
                cap = int(open(f"{h}/power1_cap").read()) / 1e6
            except (OSError, ValueError):
                pass
            return (lambda: int(open(path).read()) / 1e6), cap
    return (lambda: float("nan")), None


def main() -> int:
    import torch

    import paper_2603_20586_amd as mka
    import synth_inputs as si
    from paper_2603_20586_amd import measure

    if not torch.cuda.is_available():
        print("power_probe needs the GPU", file=sys.stderr)
        return 1
    power, cap = _power_reader()
    print(f"# board power cap {cap} W, idle {power():.0f} W")

    def steady(fn, flops, label, launches):
        for _ in range(max(20, launches // 10)):
            fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        ps = []
        e0.record()
        for i in range(launches):
            fn()
            if i % (launches // 10) == launches // 10 - 1:
                ps.append(power())
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / launches
        p = sum(ps[3:]) / len(ps[3:])
        print(f"{label:58s} {ms:8.4f} ms  {flops / ms / 1e9:7.0f} TFLOP/s  {p:6.0f} W")

    dev = torch.device("cuda:0")
    if "--core-only" not in sys.argv[1:]:
        out = torch.empty(2048 * 512, dtype=torch.float32, device=dev)
        fl = [0.0]

        def ints():
            fl[0] = measure.mfma_loop(out, 2048, 2000)
        ints()
        steady(ints, fl[0], "MFMA loop, small-integer operands (no memory traffic)", 1000)
        gen = torch.Generator(device=dev).manual_seed(11)
        for label, frags in (
                ("MFMA loop, operands all zero", torch.zeros(measure.FRAG_BYTES // 2, device=dev)),
                ("MFMA loop, operands N(0,1)", torch.randn(measure.FRAG_BYTES // 2, device=dev, generator=gen))):
            fb = frags.to(torch.bfloat16)

            def data():
                fl[0] = measure.mfma_loop_data(out, fb, 2048, 250)
            data()
            steady(data, fl[0], label, 1000)

    inp, cfg = si.config_inputs("C3", device="cuda")
    B, H, T, d = cfg["B"], cfg["H"], cfg["Tq"], cfg["d"]
    O = torch.empty_like(inp["Q"])
    flops = 4.0 * d * (T * (T + 1) / 2) * B * H
    for label, (Q, K, V) in (
            ("attention core, C3 shape, Q = K = V = 0", tuple(torch.zeros_like(inp["Q"]) for _ in range(3))),
            ("attention core, C3 shape, N(0,1) inputs (the benchmark's)", (inp["Q"], inp["K"][0], inp["V"][0]))):
        def core():
            mka.mka_mixture_attn_fwd(Q, [K, None, None], [V, None, None], None, causal=True,
                                     scale=1.0 / math.sqrt(d), O=O, want_lse=False)
        steady(core, flops, label, 2500)
    return 0


if __name__ == "__main__":
    sys.exit(main())
