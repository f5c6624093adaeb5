"""IEEE half data (FWA_F16) through the wide-head kernels: the head widths and window length of the
paper's kernel benchmarks (Section 3.1: L = 64, 4 heads, width per head 64 to 256) in the precision
its Section 3.3 comparison runs in.  Inputs are drawn in fp32, rounded once to half, and go to the
oracle as those exact values; outputs are half, compared with the un-rounded fp64 oracle at the
bound of the 16-bit paths, 1e-2 max-abs (half an ulp of a half result below 8 is at most 2e-3).
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu


def bias_and_mask(heads, L, seed, periods=3):
    bias = synth.normal((heads, L, L), seed, 0.5)
    mask = np.where(synth.rng(seed + 1).random((periods, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    return bias, mask


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("L", [64, 49, 33, 16, 7])
@pytest.mark.parametrize("use_bm", [False, True])
def test_forward_half(oracle, d, L, use_bm):
    import torch
    import paper_2501_06480_amd as fwa
    heads, N = 4, 12
    w = synth.Workload(f"f16_d{d}_L{L}", N, L, d * heads, heads, "f16", 8300 + d + L, 0)
    x = synth.draw(w)
    bias, mask = bias_and_mask(heads, L, 8400 + L + d) if use_bm else (None, None)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    assert q.dtype == torch.float16
    o = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), f32_device(mask))
    torch.cuda.synchronize()
    assert o.dtype == torch.float16
    want = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias, mask)
    got = to_f64(o)
    assert np.isfinite(got).all()
    err = max_abs(got, want)
    print(f"half fwd d={d} L={L} bm={use_bm}: max|ref|={np.abs(want).max():.2f} err={err:.3e}", flush=True)
    assert err <= TOL["f16"]


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("L", [64, 49, 33, 7])
@pytest.mark.parametrize("use_bm", [False, True])
def test_backward_half(oracle, d, L, use_bm):
    import torch
    import paper_2501_06480_amd as fwa
    heads, N = 4, 9
    w = synth.Workload(f"f16_bwd_d{d}_L{L}", N, L, d * heads, heads, "f16", 8500 + d + L, 0, backward=True)
    x = synth.draw(w)
    bias, mask = bias_and_mask(heads, L, 8600 + L + d) if use_bm else (None, None)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    dq, dk, dv, db = fwa.fwa_backward(q, k, v, g, heads, w.scale, f32_device(bias), f32_device(mask), want_dbias=use_bm)
    torch.cuda.synchronize()
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], heads, w.scale, bias, mask)
    errs = {}
    for name, got, want in (("dq", dq, ref[0]), ("dk", dk, ref[1]), ("dv", dv, ref[2])):
        assert got.dtype == torch.float16
        got = to_f64(got)
        assert np.isfinite(got).all(), name
        errs[name] = max_abs(got, want)
        assert errs[name] <= TOL["f16"], (name, errs[name], float(np.abs(want).max()))
    if use_bm:
        errs["dbias"] = max_abs(to_f64(db), ref[3])
        assert errs["dbias"] <= TOL["f16"]
    print(f"half bwd d={d} L={L} bm={use_bm}: " + " ".join(f"{k}={e:.2e}" for k, e in errs.items()), flush=True)


def test_half_dbias_over_many_windows_and_strided_views(oracle):
    """The paper's benchmark shape (L = 64, 4 heads x 64) with workgroups that walk several windows, q, k, v
    read in place from a fused [N, L, 3, heads, d] buffer and the gradients written into one."""
    import torch
    import paper_2501_06480_amd as fwa
    heads, d, L, N = 4, 64, 64, 300
    C = heads * d
    w = synth.Workload("f16_fused", N, L, C, heads, "f16", 8700, 0, backward=True)
    x = synth.draw(w)
    bias, mask = bias_and_mask(heads, L, 8701, periods=4)
    qkv = torch.stack([to_device(x, w, n) for n in ("q", "k", "v")], dim=2).contiguous()   # [N, L, 3, C]
    q, k, v = (qkv[:, :, t] for t in range(3))
    g = to_device(x, w, "d_o")
    o = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), f32_device(mask))
    dqkv = torch.empty_like(qkv)
    out = tuple(dqkv[:, :, t] for t in range(3))
    _, _, _, db = fwa.fwa_backward(q, k, v, g, heads, w.scale, f32_device(bias), f32_device(mask), want_dbias=True, out=out)
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias, mask)
    assert max_abs(to_f64(o), want) <= TOL["f16"]
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], heads, w.scale, bias, mask)
    for t, name in enumerate(("dq", "dk", "dv")):
        err = max_abs(to_f64(dqkv[:, :, t]), ref[t])
        assert err <= TOL["f16"], (name, err)
    err = max_abs(to_f64(db), ref[3])
    print(f"half, fused buffers, N={N}: dbias err={err:.2e} max|ref|={np.abs(ref[3]).max():.1f}", flush=True)
    assert err <= TOL["f16"]


def test_half_is_refused_at_head_width_32():
    import torch
    import paper_2501_06480_amd as fwa
    q = torch.zeros((4, 49, 96), dtype=torch.float16, device="cuda")
    with pytest.raises(fwa.FwaError) as e:
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1)
    assert e.value.code == fwa.binding.FWA_ERR_UNSUPPORTED
