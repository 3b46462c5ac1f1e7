"""Shared helpers of the GPU parity tests: error metrics and oracle plumbing."""
import sys

import numpy as np
import torch

BF16_ATOL = 2e-2   # max-abs error bound of the bf16 path (contract of the build)
F32_RTOL = 1e-5    # max|x-r| / max|r| bound of the f32 path
GATE_ATOL = 1e-6


def announce(msg):
    """Name the case before touching the GPU, flushed, so a lost box still tells what ran."""
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def to_np(x):
    return None if x is None else x.detach().float().cpu().double().numpy() \
        if x.dtype != torch.int32 else x.cpu().numpy()


def max_abs(x, ref):
    return float(np.max(np.abs(to_np(x) - ref))) if ref.size else 0.0


def rel_err(x, ref):
    den = float(np.max(np.abs(ref))) if ref.size else 1.0
    return max_abs(x, ref) / max(den, 1e-300)


def cpu_list(ts):
    return [None if t is None else t.cpu() for t in ts]
