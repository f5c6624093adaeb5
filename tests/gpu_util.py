"""Helpers for the GPU parity tests: move seeded inputs to the device, fetch results as float64."""
import numpy as np

# Tolerances of the benchmark spec: max-abs error against the fp64 oracle.
TOL = {"f32": 1e-5, "bf16": 1e-2, "f16": 1e-2}


def to_device(x, w, name):
    """The workload's tensor `name` as a device tensor of the workload dtype (bit-exact)."""
    import torch
    if w.dtype == "bf16":
        return torch.from_numpy(x[name + "_bits"].view(np.int16)).view(torch.bfloat16).cuda()
    if w.dtype == "f16":  # the drawn values are already rounded to half: the cast is exact
        return torch.from_numpy(x[name]).cuda().half()
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


def check_bf16_output(got, want, what):
    """The benchmark's bf16 bound: max-abs 1e-2 against the un-rounded fp64 oracle.  A bf16 output of
    magnitude >= 4 cannot meet it whatever the kernel does (half an ulp is 0.0156 on [4, 8)), so
    such elements -- counted and reported -- are held to half a bf16 ulp of the reference plus the
    2e-3 allowed to the kernel's internal error, and all others to 1e-2.  Returns the largest
    error among the elements below 4."""
    err = np.abs(got - want)
    big = np.abs(want) >= 4.0
    small_err = float(err[~big].max()) if (~big).any() else 0.0
    assert small_err <= TOL["bf16"], (what, small_err)
    if big.any():
        half_ulp = 2.0 ** (np.floor(np.log2(np.abs(want[big]))) - 8)
        excess = float((err[big] - half_ulp).max())
        print(f"{what}: {int(big.sum())} elements with |ref| >= 4 (max {np.abs(want).max():.2f}), "
              f"error beyond half a bf16 ulp {excess:.2e}", flush=True)
        assert excess <= 2e-3, (what, excess)
    return small_err


def check_forward_arithmetic_bound(got, want, spread, what):
    """The bf16 forward on shapes where the flat 1e-2 of the benchmark workloads cannot hold for every
    element (few keys per row and |V| up to 4-5).  Every element is held to the flat 1e-2 unless the
    bound derived from the arithmetic is larger for THAT element, and then to that bound: the output is
    rounded once (half a bf16 ulp of the result) and the un-normalised probabilities enter the matrix
    core rounded to bf16 (unit roundoff 2^-8; the largest one, exp(0) = 1, exactly), so the error of an
    element is at most half_ulp(|o|) + 2^-8 * sum_j p_ij |v_j| plus fp32 rounding noise.  `spread` is
    that sum: the oracle's forward on |V|.  Prints how many elements needed more than the flat figure."""
    err = np.abs(got - want)
    half_ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.maximum(np.abs(want), np.abs(got)), 2.0 ** -20))) - 8)
    bound = np.maximum(half_ulp + 2.0 ** -8 * spread + 1e-4, TOL["bf16"])
    worst = float((err - bound).max())
    assert worst <= 0.0, (what, worst, float(err.max()))
    beyond = int((err > TOL["bf16"]).sum())
    if beyond:
        print(f"{what}: {beyond} of {err.size} elements beyond the flat 1e-2 (max {err.max():.3e}), "
              f"each within its own arithmetic bound", flush=True)
    return float(err.max())
