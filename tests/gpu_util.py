"""Helpers for the GPU parity tests: move seeded inputs to the device, fetch results as float64."""
import numpy as np

# Tolerances of the benchmark spec: max-abs error against the fp64 oracle.
TOL = {"f32": 1e-5, "bf16": 1e-2}


def to_device(x, w, name):
    """The workload's tensor `name` as a device tensor of the workload dtype (bit-exact)."""
    import torch
    if w.dtype == "bf16":
        return torch.from_numpy(x[name + "_bits"].view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(x[name]).cuda()


def f32_device(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def max_abs(a, b):
    return float(np.max(np.abs(a - b))) if a.size else 0.0


def bf16_round_f64(x):
    """fp64 reference rounded to bf16 (via fp32), to separate kernel error from output rounding."""
    from paper_2501_06480_amd import synth
    return synth.bf16_round(x.astype(np.float32))[0].astype(np.float64)
