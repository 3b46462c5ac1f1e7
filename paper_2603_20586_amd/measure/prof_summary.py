"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2603_20586_amd.measure.prof_summary stats  <kernel_stats.csv>  <out.txt>  "<command>"
    python -m paper_2603_20586_amd.measure.prof_summary trace  <kernel_trace.csv>  <out.txt>  "<command>"
    python -m paper_2603_20586_amd.measure.prof_summary pmc    <counter_collection.csv> <out.txt> "<command>"
    python -m paper_2603_20586_amd.measure.prof_summary traffic <profiles dir> <traffic.json>

`traffic`: scaled FETCH_SIZE + WRITE_SIZE of the kernels behind each roofline line of `bench.py`
(picked by the run's workload group, kernel name and workgroup count; one profiler run per
workload: `bench.py --only <group>`) -> HBM bytes per launch, as JSON.
`stats`: per-kernel calls / average / total time.  `trace`: the same from the kernel trace, one
line per (kernel, workgroup count), i.e. per launch shape: one kernel runs at several workloads in
one bench.py run, and the roofline lines are per workload.  `pmc`: per-kernel average of every counter in
the file; for FETCH_SIZE / WRITE_SIZE (KiB per dispatch) it also prints the value scaled by what
the same counter reads for the 1 GiB calibration copy that `bench.py --calibrate-copy` runs
(factor = 2^20 KiB / measured KiB of that copy), i.e. an estimate of true HBM bytes.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def _template_args(mangled: str) -> str:
    """'IDF16bLi128ELi4ELb1EE...' -> '<bf16,128,4,true>' (the argument kinds this library uses)."""
    if not mangled.startswith("I"):
        return ""
    i, args = 1, []
    while i < len(mangled) and mangled[i] != "E":
        if mangled.startswith("DF16b", i):
            args.append("bf16")
            i += 5
        elif mangled[i] == "f":
            args.append("f32")
            i += 1
        elif mangled[i] == "L":                       # literal: L <type letter> <value> E
            j = mangled.index("E", i)
            kind, val = mangled[i + 1], mangled[i + 2:j]
            args.append(("true" if val == "1" else "false") if kind == "b" else val)
            i = j + 1
        else:
            return ""                                 # something else: leave the name bare
    return "<" + ",".join(args) + ">"


def short(name: str) -> str:
    """Readable kernel name (c++filt does not know every mangling of the bf16 type)."""
    m = re.match(r"_ZN3mka(?:12_GLOBAL__N_1)?(\d+)", name)
    if m:
        n = int(m.group(1))
        start = m.end()
        return "mka::" + name[start:start + n] + _template_args(name[start + n:])
    name = name.replace("(anonymous namespace)::", "")
    return name.split("(")[0].replace("void ", "")[:80]


def stats(src, dst, cmd):
    rows = list(csv.DictReader(open(src)))
    out = [f"# rocprofv3 kernel-trace summary", f"# command: {cmd}",
           "# kernel | calls | avg_us | total_ms | pct", ""]
    for r in rows[:14]:
        out.append(f"{short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                   f"{float(r['TotalDurationNs']) / 1e6:.2f} | {float(r['Percentage']):.2f}")
    open(dst, "w").write("\n".join(out) + "\n")


def trace(src, dst, cmd):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(src)):
        wgs = 1
        for ax in "XYZ":
            wgs *= max(1, int(r["Grid_Size_" + ax]) // max(1, int(r["Workgroup_Size_" + ax])))
        acc[(short(r["Kernel_Name"]), wgs)].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    total = sum(sum(v) for v in acc.values())
    out = ["# rocprofv3 kernel-trace summary, per kernel and launch shape", f"# command: {cmd}",
           "# kernel | workgroups | calls | avg_us | total_ms | pct", ""]
    for (k, wgs), v in sorted(acc.items(), key=lambda kv: -sum(kv[1])):
        if "mka::" not in k:
            continue
        out.append(f"{k} | {wgs} | {len(v)} | {sum(v) / len(v) / 1e3:.1f} | {sum(v) / 1e6:.2f} | "
                   f"{100.0 * sum(v) / total:.2f}")
    open(dst, "w").write("\n".join(out) + "\n")


def pmc(src, dst, cmd):
    rows = list(csv.DictReader(open(src)))
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in rows:
        key = (short(r["Kernel_Name"]), int(r["Grid_Size"]) // int(r["Workgroup_Size"]))
        acc[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    copy_kib = {}
    for (k, wgs), v in acc.items():
        if "CUDAFunctorOnSelf_add" in k:  # the 1 GiB calibration copy of bench.py
            for c, xs in v.items():
                copy_kib[c] = sum(xs) / len(xs)
    out = ["# rocprofv3 --pmc summary (average per dispatch, grouped by kernel and grid)",
           f"# command: {cmd}"]
    for c, x in copy_kib.items():
        out.append(f"# calibration copy (reads 1 GiB, writes 1 GiB): {c} = {x:.0f} KiB "
                   f"-> factor {1048576.0 / x:.4f}")
    out += ["# kernel | workgroups | counter | dispatches | avg_KiB | scaled_MB", ""]
    for (k, wgs), v in sorted(acc.items()):
        if "mka::" not in k:
            continue
        for c, xs in sorted(v.items()):
            avg = sum(xs) / len(xs)
            scaled = ""
            if c in copy_kib and c in ("FETCH_SIZE", "WRITE_SIZE"):
                scaled = f"{avg * (1048576.0 / copy_kib[c]) * 1024 / 1e6:.1f}"
            out.append(f"{k} | {wgs} | {c} | {len(xs)} | {avg:.5g} | {scaled}")
    open(dst, "w").write("\n".join(out) + "\n")


# roofline key of bench.py -> (profile group = the `--only` value of the run, [(kernel, workgroups of
# its launch at that workload), ...]): the kernels that carry the line's algorithmic work; their
# traffic is summed.  Causal launches: one workgroup per PAIR of tiles.
TRAFFIC_KEYS = {
    "C5_fwd": ("step", [("mka::route_kernel<bf16,128>", 4096), ("mka::prefuse_kernel<128>", 16384),
                        ("mka::mix_bf16_kernel<128,1>", 1024)]),      # 128 heads x 16/2 query tiles
    "C5_bwd": ("step", [("mka::bwd_main_kernel<128>", 2048),          # 128 heads x 32/2 key tiles
                        ("mka::bwd_dqg_kernel<128>", 1024)]),
    "C4_decode_step": ("step", [("mka::decode_split_kernel<bf16,128,4,false>", 2048)]),  # 4 splits x 512
    "C2_fwd": ("C2", [("mka::fwd_bf16_kernel<128>", 256)]),           # 64 heads x 8/2 query tiles
    "C2_fwd_materialised": ("C2", [("mka::prefuse_kernel<128>", 4096), ("mka::mix_bf16_kernel<128,1>", 256)]),
    "C2_bwd": ("C2", [("mka::bwd_main_kernel<128>", 512), ("mka::bwd_dqg_kernel<128>", 256)]),
    "C3_fwd": ("C3", [("mka::prefuse_kernel<128>", 8192), ("mka::mix_bf16_kernel<128,1>", 512)]),
    "C3_attention_core": ("C3", [("mka::mix_bf16_kernel<128,1>", 512)]),  # 32 heads x 32/2 query tiles
    "C3_fwd_folded": ("C3", [("mka::fwd_bf16_kernel<128>", 512)]),
    "C3_mixture": ("C3mix", [("mka::mix_bf16_kernel<128,1>", 512)]),
    "paged_fused_decode_32K": ("paged", [("mka::paged_split_kernel<128>", 2048)]),
    "paged_fused_decode_128K": ("paged128K", [("mka::paged_split_kernel<128>", 2048)]),
}


def traffic(profiles_dir, dst):
    """<profiles_dir>/<group>_fetch_size.txt and <group>_write_size.txt -> HBM bytes per launch of
    every roofline key whose kernels appear in its group's summaries."""
    import json
    import os

    def scaled(path):
        out = {}
        if not os.path.exists(path):
            return out
        for line in open(path):
            f = [x.strip() for x in line.split("|")]
            if len(f) == 6 and f[5] and not line.startswith("#"):
                out[(f[0], int(f[1]))] = float(f[5]) * 1e6  # scaled_MB -> bytes
        return out

    res = {}
    for key, (group, ks) in TRAFFIC_KEYS.items():
        rd = scaled(os.path.join(profiles_dir, f"{group}_fetch_size.txt"))
        wr = scaled(os.path.join(profiles_dir, f"{group}_write_size.txt"))
        if all(k in rd and k in wr for k in ks):
            res[key] = int(sum(rd[k] + wr[k] for k in ks))
    json.dump(res, open(dst, "w"), indent=1, sort_keys=True)
    print(json.dumps(res, indent=1, sort_keys=True))


if __name__ == "__main__":
    if sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3])
    else:
        mode, src, dst, cmd = sys.argv[1], sys.argv[2], sys.argv[3], sys.argv[4]
        {"stats": stats, "trace": trace, "pmc": pmc}[mode](src, dst, cmd)
        print(open(dst).read())
