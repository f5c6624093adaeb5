"""Tensors larger than 4 GiB: every kernel family addresses windows with 64-bit offsets.

A window is reached as base + w * L * ld * e bytes; the tests above never leave the first few hundred
MB, where a 32-bit product would still be right.  Here each of Q, K, V (dO, dQ, dK, dV) is just over
4 GiB.  The inputs are a seeded block of B windows, drawn on the host, repeated down the tensor with a
sign and a power of two that change from repetition to repetition (exact in bf16 and fp32, so the
host knows every window without holding the tensor): an offset that wrapped at 2^31 or 2^32 bytes
would land inside a window of a different repetition and give different numbers.  The oracle
recomputes the windows on both sides of the 2 GiB and 4 GiB marks, the first and last ones and a few
random ones; over all windows the outputs are held to properties (an output row is a convex
combination of the rows of V; the rows of dV sum to the rows of dO).
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, max_abs, to_f64

pytestmark = pytest.mark.gpu

SIGNS = np.array([1.0, -1.0, 0.5, -0.5], dtype=np.float32)


def rep_scale(r, t):
    """Multiplier of repetition r of tensor number t (q, k, v, d_o = 0..3): +-1 or +-1/2."""
    return SIGNS[(np.asarray(r) * (2 * t + 3) + t) % 4]


# name, L, heads, d, dtype, bias, mask ("none" / "dense" / "labels"), nW, strided, want_dbias
CASES = [
    ("stage1_plain", 49, 3, 32, "bf16", False, "none", 1, False, False),
    ("stage1_bias_labels", 49, 3, 32, "bf16", True, "labels", 64, False, True),
    ("stage1_fused_qkv", 49, 3, 32, "bf16", True, "dense", 64, True, False),
    ("six_heads_bias_mask", 49, 6, 32, "bf16", True, "dense", 16, False, True),
    ("five_heads", 49, 5, 32, "bf16", True, "dense", 4, False, False),
    ("mask_period_512", 49, 3, 32, "bf16", True, "dense", 512, False, True),
    ("L144_bias", 144, 4, 32, "bf16", True, "labels", 16, False, True),
    ("L256_plain", 256, 2, 32, "bf16", False, "none", 1, False, False),
    ("wide64_bias_mask", 64, 4, 64, "bf16", True, "dense", 4, False, True),
    ("wide256", 49, 1, 256, "bf16", False, "none", 1, False, False),
    ("f32_width32", 49, 3, 32, "f32", True, "dense", 4, False, False),
    ("f32_width128", 64, 2, 128, "f32", False, "none", 1, False, False),
]


@pytest.mark.parametrize("name,L,heads,d,dtype,use_bias,mask_kind,nW,strided,want_dbias", CASES,
                         ids=[c[0] for c in CASES])
def test_windows_beyond_4gib(oracle, name, L, heads, d, dtype, use_bias, mask_kind, nW, strided, want_dbias):
    import torch
    import paper_2501_06480_amd as fwa
    C = heads * d
    e = 2 if dtype == "bf16" else 4
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    wb = L * C * e                                   # bytes of one window in a contiguous tensor
    B = max(nW, 1536 // nW * nW)                     # windows of the seeded block
    reps = -(-int(1.03 * 2 ** 32) // (wb * B))
    N = reps * B
    assert N * wb > 2 ** 32
    print(f"case {name}: N={N} ({reps} x {B}), {N * wb / 2 ** 30:.2f} GiB per tensor", flush=True)

    w = synth.Workload(name, B, L, C, heads, dtype, 880000 + L + heads + d, 0, backward=True)
    base = synth.draw(w)
    names = ("q", "k", "v", "d_o")
    scale_dev = [torch.from_numpy(rep_scale(np.arange(reps), t)).to(tdt).cuda().view(reps, 1, 1, 1) for t in range(4)]

    def on_device(t, out=None):
        b = torch.from_numpy(base[names[t]]).to(tdt).cuda()   # the values are already rounded to dtype: exact
        x = torch.empty((N, L, C), dtype=tdt, device="cuda") if out is None else out
        for r0 in range(0, reps, 64):                # in slices: the broadcast product needs no full-size temporary
            r1 = min(reps, r0 + 64)
            x[r0 * B:r1 * B].view(r1 - r0, B, L, C).copy_(b[None] * scale_dev[t][r0:r1])
        return x

    def on_host(t, pick):
        return base[names[t]][pick % B].astype(np.float64) * rep_scale(pick // B, t).astype(np.float64)[:, None, None]

    if strided:
        buf = torch.empty((N, L, 3, C), dtype=tdt, device="cuda")
        q, k, v = (on_device(t, out=buf[:, :, t]) for t in range(3))
        wb_in = 3 * wb
    else:
        q, k, v = (on_device(t) for t in range(3))
        wb_in = wb

    r = synth.rng(881000 + L + heads)
    bias64 = bias_dev = mask64 = mask_dev = labels_dev = None
    if use_bias:
        b32 = synth.normal((heads, L, L), 882000 + L, 0.5)
        bias64, bias_dev = b32.astype(np.float64), torch.from_numpy(b32).cuda()
    if mask_kind == "dense":
        m = np.where(r.random((nW, L, L)) < 0.25, -100.0, 0.0).astype(np.float32)
        m[:, np.arange(L), np.arange(L)] = 0.0
        mask64, mask_dev = m.astype(np.float64), torch.from_numpy(m).cuda()
    elif mask_kind == "labels":
        lab = r.integers(0, 3, (nW, L)).astype(np.int32)
        mask64, labels_dev = oracle.mask_from_labels(lab, -100.0), torch.from_numpy(lab).cuda()

    marks = [m // b for m in (2 ** 31, 2 ** 32) for b in {wb, wb_in}]
    pick = np.unique(np.clip(np.concatenate([[0, 1, N - 2, N - 1], *[[m - 1, m, m + 1] for m in marks],
                                             r.integers(0, N, 10)]), 0, N - 1)).astype(np.int64)
    hq, hk, hv, hg = (on_host(t, pick) for t in range(4))
    mask_pick = None if mask64 is None else mask64[pick % nW]

    # ---- forward
    print("  forward", flush=True)
    o = fwa.fwa_forward(q, k, v, heads, w.scale, bias_dev, mask_dev, labels=labels_dev)
    torch.cuda.synchronize()
    want = oracle.forward(hq, hk, hv, heads, w.scale, bias64, mask_pick)
    got = to_f64(o[torch.from_numpy(pick).cuda()])
    if dtype == "f32":
        err = max_abs(got, want)
        assert err <= TOL["f32"], err
    else:
        err = check_bf16_output(got, want, "  o")
    # all windows: finite, and inside the range of the window's V per channel
    slack = 2e-2 if dtype == "bf16" else 1e-5
    assert bool(torch.isfinite(o).all())
    assert bool((o.amax(dim=1) <= v.amax(dim=1) + slack).all()) and bool((o.amin(dim=1) >= v.amin(dim=1) - slack).all())
    print(f"  forward err={err:.3e} over {len(pick)} windows", flush=True)
    del o

    # ---- backward
    print("  backward", flush=True)
    g = on_device(3)
    dq, dk, dv, db = fwa.fwa_backward(q, k, v, g, heads, w.scale, bias_dev, mask_dev, want_dbias=want_dbias,
                                      labels=labels_dev)
    torch.cuda.synchronize()
    ref = oracle.backward(hq, hk, hv, hg, heads, w.scale, bias64, mask_pick, want_dbias=False)
    sel = torch.from_numpy(pick).cuda()
    errs = {}
    for nme, a, b in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        assert bool(torch.isfinite(a).all()), nme
        a = to_f64(a[sel])
        if dtype == "f32":
            errs[nme] = max_abs(a, b)
            assert errs[nme] <= TOL["f32"], (nme, errs[nme])
        else:
            errs[nme] = check_bf16_output(a, b, f"  {nme}")
    # all windows: the probabilities of a row sum to one, so the rows of dV sum to the rows of dO
    # (dV is rounded once per element: half an ulp of its largest entry per term)
    col_dv, col_g = dv.sum(dim=1, dtype=torch.float32), g.sum(dim=1, dtype=torch.float32)
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -20
    bound = L * ulp * dv.abs().amax(dim=1).float() + 1e-3
    assert bool(((col_dv - col_g).abs() <= bound).all())
    if want_dbias:
        db = to_f64(db)
        assert np.isfinite(db).all()
        rows, size = np.abs(db.sum(axis=2)), np.abs(db).sum(axis=2)
        assert (rows <= 1e-4 * size + 1e-2).all(), float(rows.max())   # rows of dS, hence of dBias, sum to zero
    print("  backward " + " ".join(f"{n}={x:.2e}" for n, x in errs.items()), flush=True)
    del q, k, v, g, dq, dk, dv
    torch.cuda.empty_cache()
