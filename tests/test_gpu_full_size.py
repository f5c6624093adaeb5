"""Parity at the full sizes of the benchmark configurations, in the launch configurations bench.py times.

Every tensor is compared whole: the oracle runs over all windows (seconds for 7 x 7 windows, tens of
seconds for the 16 x 16 windows of the backward), dBias included, which is a sum over all of them.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu


FORWARD = [(w.name, w) for w in synth.config3() + synth.config4()]


@pytest.mark.parametrize("name,w", FORWARD, ids=[n for n, _ in FORWARD])
def test_forward_configs_3_and_4_full_size(oracle, name, w):
    import torch
    import paper_2501_06480_amd as fwa
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], w.k)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias64), f32_device(x["mask"]))
    torch.cuda.synchronize()
    got = to_f64(o)
    assert np.isfinite(got).all()
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, x["mask"])
    err = max_abs(got, want)
    print(f"{name} full size, all {w.N} windows: max|ref|={np.abs(want).max():.3f} max-abs err={err:.3e}", flush=True)
    assert err <= TOL["bf16"], (name, err)
    if x["labels"] is not None:  # the label form of the mask, at full size: the same bits
        o2 = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias64), labels=torch.from_numpy(x["labels"]).cuda())
        assert torch.equal(o.view(torch.int16), o2.view(torch.int16))


def test_backward_config5_stage3_full_size(oracle):
    import paper_2501_06480_amd as fwa
    w = synth.config5()[1]
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], w.k)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    got = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias64), f32_device(x["mask"]), want_dbias=True)
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias64, x["mask"])
    for name, a, b in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
        check_bf16_output(to_f64(a), b, f"config 5 stage 3 full size {name}")
    err = max_abs(to_f64(got[3]), ref[3])
    print(f"config 5 stage 3 full size dbias: err={err:.3e} max|ref|={np.abs(ref[3]).max():.2f}", flush=True)
    assert err <= TOL["bf16"]


@pytest.mark.parametrize("which", [0, 1])
def test_backward_large_windows_full_size(oracle, which):
    """The windows of config 4 (L = 144, 256 at N = 1024) through the backward, with dBias: every
    window of dQ, dK, dV and the whole of dBias against the oracle."""
    import torch
    import paper_2501_06480_amd as fwa
    base = synth.config4()[which]
    w = synth.Workload(base.name + "_bwd", base.N, base.L, base.C, base.heads, "bf16", base.seed + 50, base.k,
                       base.map_hw, True, base.k // 2, True)
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], w.k)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    dq, dk, dv, db = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias64), f32_device(x["mask"]),
                                      want_dbias=True)
    torch.cuda.synchronize()
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias64, x["mask"])
    for name, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        a = to_f64(a)
        assert np.isfinite(a).all(), name
        e = check_bf16_output(a, b, f"{w.name} full size {name}")
        print(f"{w.name} full size, all {w.N} windows, {name}: max|ref|={np.abs(b).max():.2f} max-abs err={e:.3e}", flush=True)
    # dBias, a sum over all 1024 windows, against the oracle's
    db = to_f64(db)
    assert np.isfinite(db).all()
    err = max_abs(db, ref[3])
    print(f"{w.name} full size dbias: max|ref|={np.abs(ref[3]).max():.2f} max-abs err={err:.3e}", flush=True)
    assert err <= TOL["bf16"], err
    # and the label form gives the same bits, dBias included
    lab = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias64), want_dbias=True,
                           labels=torch.from_numpy(x["labels"]).cuda())
    for a, b in zip((dq, dk, dv), lab[:3]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(lab[3].view(torch.int32), torch.from_numpy(db.astype(np.float32)).cuda().view(torch.int32))


def test_stage1_on_a_large_token_map_full_size(oracle):
    """bench.py's long-mask-period workload (stage 1 on a 224 x 224 token map: 1024 windows per image, batch 8,
    the mask as labels), forward and backward with dBias: every window and the whole of dBias against the oracle."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload("stage1_map224", 8192, 49, 96, 3, "bf16", 1400, 7, 224, True, 3, True)
    x = synth.draw(w)
    assert x["labels"].shape == (1024, 49)
    bias64 = oracle.bias_gather(x["table"], w.k)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    lab = torch.from_numpy(x["labels"]).cuda()
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias64), labels=lab)
    dq, dk, dv, db = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias64), labels=lab, want_dbias=True)
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, x["mask"])
    err = max_abs(to_f64(o), want)
    print(f"stage 1 on a 224 x 224 map, all {w.N} windows: forward err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]
    del want
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias64, x["mask"])
    for name, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        a = to_f64(a)
        assert np.isfinite(a).all(), name
        e = check_bf16_output(a, b, f"stage 1 on a 224 x 224 map {name}")
        print(f"stage 1 on a 224 x 224 map, all windows, {name}: err={e:.3e}", flush=True)
    db = to_f64(db)
    assert np.isfinite(db).all()
    err = max_abs(db, ref[3])
    print(f"stage 1 on a 224 x 224 map dbias: max|ref|={np.abs(ref[3]).max():.2f} err={err:.3e}", flush=True)
    assert err <= TOL["bf16"], err
