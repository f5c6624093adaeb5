"""Seeded random combinations of everything a call can vary: window length, head count and width,
number of windows, mask period, bias (none / fp32 / bf16), mask (none / dense / labels), data type,
contiguous or fused-QKV row strides -- forward and backward against the fp64 oracle.

The other GPU tests walk one axis at a time; this one crosses them, so that a dispatch rule that is
wrong only for a combination (a workgroup shape picked for a head count it does not divide, a
persistent walk whose slot count does not fit the mask period, ...) still meets a case.  Every
shape is inside the documented limits of the entry points.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, check_forward_arithmetic_bound, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu

N_CASES = 240
ELEMENTS = 2_000_000          # cap on N*L*C per tensor: the oracle stays within a second or two per case


def draw_case(i, long_period=False):
    """The i-th combination (a pure function of i).  long_period: mask periods of 16 to 512 windows, which
    decide how many windows a persistent workgroup may walk; beyond the slot counts, labels make the
    kernels form each window's mask themselves and dense masks go to the kernels without a walk."""
    r = synth.rng(424200 + i)
    dtype = "f32" if r.random() < 0.25 else "bf16"
    wide = r.random() < 0.3
    if wide:
        d = int(r.choice([64, 128, 256]))
        L = int(r.integers(1, 65))
        heads = int(r.integers(1, 5))
    else:
        d = 32
        L = int(r.integers(1, 65)) if r.random() < 0.6 else int(r.integers(65, 257))
        heads = int(r.integers(1, 13))
    nW = int(r.choice([16, 64, 256, 512])) if long_period else int(r.choice([1, 1, 2, 3, 4, 6]))
    most = max(1, ELEMENTS // (L * heads * d * nW))
    mult = int(np.exp(r.uniform(0.4, 1.0) * np.log(most + 0.5)))   # skewed towards many windows
    N = nW * max(1, min(mult, most))
    mask_kind = str(r.choice(["dense", "labels"] if long_period else ["none", "dense", "labels"]))
    bias_kind = str(r.choice(["none", "f32", "bf16"]))
    if bias_kind == "bf16" and mask_kind == "dense":   # a bf16 bias comes with labels or with no mask
        mask_kind = "labels"
    strided = bool(r.random() < 0.35)
    want_dbias = bias_kind != "none" and dtype == "bf16" and bool(r.random() < 0.7)
    return dict(i=i, dtype=dtype, d=d, L=L, heads=heads, nW=nW, N=N, mask=mask_kind, bias=bias_kind,
                strided=strided, want_dbias=want_dbias)


def case_id(c):
    return (f"{c['i']:03d}-{c['dtype']}-L{c['L']}-h{c['heads']}-d{c['d']}-N{c['N']}-nW{c['nW']}-"
            f"b{c['bias']}-m{c['mask']}{'-strided' if c['strided'] else ''}{'-dB' if c['want_dbias'] else ''}")


CASES = [draw_case(i) for i in range(N_CASES)] + [draw_case(N_CASES + i, long_period=True) for i in range(48)]


def fused(tensors, torch):
    """The given [N, L, C] tensors as views of one [N, L, len, C] tensor (row stride len*C)."""
    N, L, C = tensors[0].shape
    buf = torch.empty((N, L, len(tensors), C), dtype=tensors[0].dtype, device="cuda")
    views = []
    for t, x in enumerate(tensors):
        buf[:, :, t].copy_(x)
        views.append(buf[:, :, t])
    return views


@pytest.mark.parametrize("c", CASES, ids=[case_id(c) for c in CASES])
def test_random_combination(oracle, c):
    import torch
    import paper_2501_06480_amd as fwa
    L, heads, d, N, nW, dtype = c["L"], c["heads"], c["d"], c["N"], c["nW"], c["dtype"]
    print("case", case_id(c), flush=True)
    backward = dtype == "bf16" or L <= 64
    w = synth.Workload(case_id(c), N, L, heads * d, heads, dtype, 515000 + c["i"], 0, backward=backward)
    x = synth.draw(w)
    r = synth.rng(616000 + c["i"])

    bias64 = bias_dev = None
    if c["bias"] != "none":
        b = synth.normal((heads, L, L), 717000 + c["i"], 0.5)
        if c["bias"] == "bf16":
            b, bits = synth.bf16_round(b)
            bias_dev = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        else:
            bias_dev = torch.from_numpy(b).cuda()
        bias64 = b.astype(np.float64)
    mask64 = mask_dev = labels_dev = None
    if c["mask"] == "dense":
        m = np.where(r.random((nW, L, L)) < 0.25, -100.0, 0.0).astype(np.float32)
        m[:, np.arange(L), np.arange(L)] = 0.0
        mask64, mask_dev = m.astype(np.float64), torch.from_numpy(m).cuda()
    elif c["mask"] == "labels":
        lab = r.integers(0, 3, (nW, L)).astype(np.int32)
        mask64 = oracle.mask_from_labels(lab, -100.0)
        labels_dev = torch.from_numpy(lab).cuda()

    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    if c["strided"]:
        q, k, v = fused([q, k, v], torch)

    # ---- forward
    o = fwa.fwa_forward(q, k, v, heads, w.scale, bias_dev, mask_dev, labels=labels_dev)
    torch.cuda.synchronize()
    got = to_f64(o)
    assert np.isfinite(got).all()
    want = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias64, mask64)
    if dtype == "f32":
        err = max_abs(got, want)
        assert err <= TOL["f32"], ("forward", err)
    else:
        spread = oracle.forward(x["q"], x["k"], np.abs(x["v"]), heads, w.scale, bias64, mask64)
        err = check_forward_arithmetic_bound(got, want, spread, "forward")
        assert err <= 2e-2, ("forward", err)
    print(f"  forward err={err:.3e}", flush=True)
    if not backward:
        return

    # ---- backward
    g = to_device(x, w, "d_o")
    want_dbias = c["want_dbias"]
    dq, dk, dv, db = fwa.fwa_backward(q, k, v, g, heads, w.scale, bias_dev, mask_dev, want_dbias=want_dbias,
                                      labels=labels_dev)
    torch.cuda.synchronize()
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], heads, w.scale, bias64, mask64, want_dbias=want_dbias)
    errs = {}
    for name, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        a = to_f64(a)
        assert np.isfinite(a).all(), name
        if dtype == "f32":
            errs[name] = max_abs(a, b)
            assert errs[name] <= TOL["f32"], (name, errs[name])
        else:
            errs[name] = check_bf16_output(a, b, f"  {name}")
    if want_dbias:
        a = to_f64(db)
        assert np.isfinite(a).all()
        errs["dbias"] = max_abs(a, ref[3])
        assert errs["dbias"] <= TOL["bf16"], ("dbias", errs["dbias"], float(np.abs(ref[3]).max()))
    else:
        assert db is None
    print("  backward " + " ".join(f"{n}={e:.2e}" for n, e in errs.items()), flush=True)
