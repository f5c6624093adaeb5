"""GPU test of fwa_backward_noalloc, the backward for callers that cannot allocate.

It runs the kernels of fwa_backward with the library's static scratch array as workspace, so its
outputs must equal those of fwa_backward bit for bit (both are bit-reproducible), which in turn are
held to the fp64 oracle here as everywhere else.  Two calls in a row share the array: the second, on
a smaller input, must not see anything the first one left behind.
"""
import ctypes

import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu


def raw_noalloc(lib, q, k, v, g, dq, dk, dv, db, N, L, C, heads, scale, bias, mask, nW, stream):
    """The call through the C ABI itself: plain pointers and sizes."""
    ptr = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    return lib.fwa_backward_noalloc(ptr(q), ptr(k), ptr(v), ptr(g), ptr(dq), ptr(dk), ptr(dv), ptr(db), N, L, C, heads,
                                    scale, ptr(bias), ptr(mask), nW, 1, ctypes.c_void_p(stream))


def one_case(oracle, w, label):
    import torch
    import paper_2501_06480_amd as fwa
    lib = fwa.load_library()
    x = synth.draw(w)
    bias_np = oracle.bias_gather(x["table"], w.k).astype(np.float32)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    bias, mask = f32_device(bias_np), f32_device(x["mask"])
    nW = 0 if mask is None else int(mask.shape[0])
    want = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, bias, mask, want_dbias=True)
    torch.cuda.synchronize()
    # outputs pre-filled with a pattern the kernels must overwrite completely
    dq, dk, dv = (torch.full_like(q, 7.0) for _ in range(3))
    db = torch.full((w.heads, w.L, w.L), 7.0, dtype=torch.float32, device=q.device)
    torch.cuda.synchronize()
    print(f"{label}: fwa_backward_noalloc N={w.N} L={w.L} C={w.C} heads={w.heads} nW={nW}", flush=True)
    rc = raw_noalloc(lib, q, k, v, g, dq, dk, dv, db, w.N, w.L, w.C, w.heads, w.scale, bias, mask, nW,
                     torch.cuda.current_stream().cuda_stream)
    assert rc == 0, fwa.fwa_status_string(rc)
    torch.cuda.synchronize()
    for name, got, ref in (("dq", dq, want[0]), ("dk", dk, want[1]), ("dv", dv, want[2])):
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), (label, name)
    assert torch.equal(db.view(torch.int32), want[3].view(torch.int32)), (label, "dbias")
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias_np, x["mask"])
    for name, got, r in (("dq", dq, ref[0]), ("dk", dk, ref[1]), ("dv", dv, ref[2])):
        check_bf16_output(to_f64(got), r, f"{label} {name}")
    err = max_abs(to_f64(db), ref[3])
    assert err <= TOL["bf16"], (label, "dbias", err)
    print(f"{label}: bit-equal to fwa_backward; dbias err vs oracle {err:.2e}", flush=True)


def test_two_calls_in_a_row_the_second_smaller(oracle):
    big = synth.swin_t_stage(1, shifted=True, backward=True).with_N(512)      # 3 heads, L = 49, nW = 64
    small = synth.swin_t_stage(3, shifted=True, backward=True).with_N(8)      # 12 heads, L = 49, nW = 4
    one_case(oracle, big, "first call")
    one_case(oracle, small, "second call")
    # and a third with another window length, whose partial sums have another layout
    w = synth.Workload("noalloc_L25", 12, 25, 64, 2, "bf16", 7301, 5, use_bias=True, backward=True)
    one_case(oracle, w, "third call")


def test_without_dbias_no_scratch_is_touched(oracle):
    import torch
    import paper_2501_06480_amd as fwa
    lib = fwa.load_library()
    w = synth.swin_t_stage(2, shifted=False, backward=True).with_N(32)
    x = synth.draw(w)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    want = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, want_dbias=False)
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    rc = raw_noalloc(lib, q, k, v, g, dq, dk, dv, None, w.N, w.L, w.C, w.heads, w.scale, None, None, 0,
                     torch.cuda.current_stream().cuda_stream)
    assert rc == 0, fwa.fwa_status_string(rc)
    torch.cuda.synchronize()
    for got, ref in zip((dq, dk, dv), want[:3]):
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
