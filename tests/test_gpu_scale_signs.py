"""The softmax scale is any float: zero and negative scales against the fp64 oracle.

Without bias and mask the bf16 kernels fold the scale into the exponent and pad the columns beyond L
with an infinity whose sign follows the scale's; a zero scale must not turn that pad into NaN (the
result is then the per-window mean of V, paper eq. 3 with all scores equal), and a negative scale
takes the row minimum of the raw products as the stabiliser.  Window lengths that are not multiples
of 16 (padding present) and one that is, small and large windows, narrow and wide heads.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu

SCALES = [0.0, -0.0, -0.25, -1.0 / np.sqrt(32.0)]
SHAPES = [(49, 96, 3, 40), (17, 64, 2, 30), (32, 32, 1, 12), (144, 64, 2, 6), (100, 32, 1, 5), (49, 128, 2, 9)]


@pytest.mark.parametrize("L,C,heads,N", SHAPES)
@pytest.mark.parametrize("scale", SCALES)
@pytest.mark.parametrize("use_bias", [False, True])
def test_forward_and_backward_with_zero_and_negative_scales(oracle, L, C, heads, N, scale, use_bias):
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload(f"scale_L{L}_C{C}", N, L, C, heads, "bf16", 8800 + L + C, 0, backward=True)
    x = synth.draw(w)
    bias = synth.normal((heads, L, L), 8900 + L, 0.5) if use_bias else None
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    print(f"L={L} C={C} heads={heads} N={N} scale={scale} bias={use_bias}", flush=True)
    o = fwa.fwa_forward(q, k, v, heads, float(scale), f32_device(bias))
    dq, dk, dv, _ = fwa.fwa_backward(q, k, v, g, heads, float(scale), f32_device(bias))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], heads, float(scale), bias)
    got = to_f64(o)
    assert np.isfinite(got).all()
    assert max_abs(got, want) <= TOL["bf16"]
    if scale == 0.0 and not use_bias:
        # all scores equal: every output row is the mean of the window's V rows
        mean = x["v"].astype(np.float64).reshape(N, L, C).mean(axis=1, keepdims=True)
        assert max_abs(got, np.broadcast_to(mean, got.shape)) <= TOL["bf16"]
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], heads, float(scale), bias, want_dbias=False)
    for name, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        a = to_f64(a)
        assert np.isfinite(a).all(), name
        check_bf16_output(a, b, f"scale {scale} L={L} {name}")
    if scale == 0.0:
        assert not to_f64(dq).any() and not to_f64(dk).any()


@pytest.mark.parametrize("scale", [0.0, -0.2])
def test_fp32_with_zero_and_negative_scales(oracle, scale):
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload("scale_f32", 10, 49, 64, 2, "f32", 8990, 7, backward=True)
    x = synth.draw(w)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    o = fwa.fwa_forward(q, k, v, 2, scale)
    dq, dk, dv, _ = fwa.fwa_backward(q, k, v, g, 2, scale)
    torch.cuda.synchronize()
    assert max_abs(to_f64(o), oracle.forward(x["q"], x["k"], x["v"], 2, scale)) <= TOL["f32"]
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], 2, scale, want_dbias=False)
    for a, b in zip((dq, dk, dv), ref[:3]):
        assert max_abs(to_f64(a), b) <= TOL["f32"]
