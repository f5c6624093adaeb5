"""Parity at the full sizes of the benchmark configurations, in the launch configurations bench.py times.

The oracle recomputes a sample of windows one by one (first and last windows plus random ones; a
sampled window n is paired with its own mask tile, n mod nW); where a result is a sum over all
windows (dBias) it is either compared whole, when the oracle finishes in seconds, or checked
through a property that holds at any size: the rows of dS sum to zero, hence so do those of dBias.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu


def sample_windows(N, seed, count=60):
    edge = [0, 1, N - 2, N - 1]
    return np.unique(np.concatenate([edge, synth.rng(seed).integers(0, N, count)])).astype(np.int64)


def mask_of_sample(mask, pick):
    """The oracle pairs window i of its batch with mask[i % nW]: give it one tile per sampled window."""
    return None if mask is None else mask[pick % mask.shape[0]]


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
    pick = sample_windows(w.N, 300 + w.L + w.heads, 40 if w.L > 64 else 100)
    want = oracle.forward(x["q"][pick], x["k"][pick], x["v"][pick], w.heads, w.scale, bias64,
                          mask_of_sample(x["mask"], pick))
    err = max_abs(got[pick], want)
    print(f"{name} full size (N={w.N}), {len(pick)} sampled windows: max-abs err={err:.3e}", flush=True)
    assert err <= TOL["bf16"], (name, err)
    # at any size: an output row is a convex combination of the rows of V
    assert (got <= x["v"].max(axis=1, keepdims=True) + 2e-2).all()
    assert (got >= x["v"].min(axis=1, keepdims=True) - 2e-2).all()
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
    """The windows of config 4 (L = 144, 256 at N = 1024) through the backward, with dBias."""
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
    pick = sample_windows(w.N, 400 + w.L, 20)
    ref = oracle.backward(x["q"][pick], x["k"][pick], x["v"][pick], x["d_o"][pick], w.heads, w.scale, bias64,
                          mask_of_sample(x["mask"], pick), want_dbias=False)
    for name, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        a = to_f64(a)
        assert np.isfinite(a).all(), name
        check_bf16_output(a[pick], b, f"{w.name} full size {name}")
    # dBias is a sum over all 1024 windows: its rows sum to zero because those of every dS do
    db = to_f64(db)
    assert np.isfinite(db).all()
    rows = np.abs(db.sum(axis=2))
    scale_of_row = np.abs(db).sum(axis=2)
    print(f"{w.name} full size dbias: max|row sum|={rows.max():.3e} against sum|row|={scale_of_row.max():.1f}", flush=True)
    assert (rows <= 1e-4 * scale_of_row + 1e-3).all()
    # and the label form gives the same bits, dBias included
    lab = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias64), want_dbias=True,
                           labels=torch.from_numpy(x["labels"]).cuda())
    for a, b in zip((dq, dk, dv), lab[:3]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(lab[3].view(torch.int32), torch.from_numpy(db.astype(np.float32)).cuda().view(torch.int32))


def test_stage1_on_a_large_token_map_full_size(oracle):
    """bench.py's long-mask-period workload (stage 1 on a 224 x 224 token map: 1024 windows per image, batch 8,
    the mask as labels), forward and backward with dBias, on sampled windows; dBias through its row sums."""
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
    pick = sample_windows(w.N, 1400, 100)
    m = mask_of_sample(x["mask"], pick)
    want = oracle.forward(x["q"][pick], x["k"][pick], x["v"][pick], w.heads, w.scale, bias64, m)
    err = max_abs(to_f64(o)[pick], want)
    print(f"stage 1 on a 224 x 224 map, {len(pick)} sampled windows: forward err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]
    ref = oracle.backward(x["q"][pick], x["k"][pick], x["v"][pick], x["d_o"][pick], w.heads, w.scale, bias64, m,
                          want_dbias=False)
    for name, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        a = to_f64(a)
        assert np.isfinite(a).all(), name
        check_bf16_output(a[pick], b, f"stage 1 on a 224 x 224 map {name}")
    db = to_f64(db)
    assert np.isfinite(db).all()
    rows, size = np.abs(db.sum(axis=2)), np.abs(db).sum(axis=2)
    assert (rows <= 1e-4 * size + 1e-3).all(), float(rows.max())
