"""Row-strided inputs (q, k, v read in place out of a fused [N, L, 3, heads, d] tensor, gradients
written into a fused gradient tensor) and the autograd wrappers, on the GPU through the C ABI."""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu

# (L, heads, d, N, bias+mask?): one case per kernel family
CASES = [(49, 3, 32, 40, True), (49, 3, 32, 40, False), (49, 5, 32, 12, True), (49, 12, 32, 16, True),
         (33, 2, 32, 6, False), (100, 4, 32, 24, True), (144, 4, 32, 40, False), (144, 3, 32, 6, True),
         (64, 4, 64, 8, True), (49, 2, 128, 6, False)]


def fused_views(x, w, names, torch):
    """q, k, v (or three zero gradients) as views of one [N, L, 3, heads, d] tensor."""
    d = w.C // w.heads
    buf = torch.empty((w.N, w.L, 3, w.heads, d), dtype=torch.bfloat16, device="cuda")
    views = [buf[:, :, t].reshape(w.N, w.L, w.C) for t in range(3)]
    for t, (view, nme) in enumerate(zip(views, names)):
        if nme is not None:
            view.copy_(to_device(x, w, nme))
        assert view.data_ptr() == buf.data_ptr() + t * w.C * 2   # a view, not a copy
    return buf, views


@pytest.mark.parametrize("L,heads,d,N,use_bm", CASES)
def test_strided_calls_match_contiguous_calls_bit_for_bit(L, heads, d, N, use_bm):
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload(f"strided_L{L}_h{heads}_d{d}", N, L, heads * d, heads, "bf16", 9100 + L + heads + d, 0, backward=True)
    x = synth.draw(w)
    bias = mask = None
    if use_bm:
        bias = f32_device(synth.normal((heads, L, L), 61 + L, 0.5))
        m = np.where(synth.rng(67 + L).random((2, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        m[:, np.arange(L), np.arange(L)] = 0.0
        mask = f32_device(m)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    _, (qs, ks, vs) = fused_views(x, w, ("q", "k", "v"), torch)
    o_ref = fwa.fwa_forward(q, k, v, heads, w.scale, bias, mask)
    o_str = fwa.fwa_forward(qs, ks, vs, heads, w.scale, bias, mask)
    assert torch.equal(o_ref, o_str)
    # output into a strided tensor too
    obuf = torch.full((N, L, 2, heads * d), 7.0, dtype=torch.bfloat16, device="cuda")
    fwa.fwa_forward(qs, ks, vs, heads, w.scale, bias, mask, out=obuf[:, :, 1])
    assert torch.equal(obuf[:, :, 1], o_ref) and bool((obuf[:, :, 0] == 7.0).all())
    ref = fwa.fwa_backward(q, k, v, g, heads, w.scale, bias, mask)
    dbuf, dviews = fused_views(x, w, (None, None, None), torch)
    dbuf.fill_(3.0)
    fwa.fwa_backward(qs, ks, vs, g, heads, w.scale, bias, mask, out=tuple(dviews))
    torch.cuda.synchronize()
    for a, b, nme in zip(ref[:3], dviews, ("dq", "dk", "dv")):
        assert torch.equal(a, b), nme


def test_strided_dbias_and_stride_checks():
    import torch
    import paper_2501_06480_amd as fwa
    from paper_2501_06480_amd import binding
    w = synth.swin_t_stage(2, shifted=True, backward=True).with_N(64)
    x = synth.draw(w)
    bias = fwa.fwa_bias_gather(f32_device(x["table"]), w.k)
    mask = f32_device(x["mask"])
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    _, (qs, ks, vs) = fused_views(x, w, ("q", "k", "v"), torch)
    ref = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, bias, mask, want_dbias=True)
    got = fwa.fwa_backward(qs, ks, vs, g, w.heads, w.scale, bias, mask, want_dbias=True)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    with pytest.raises(ValueError):     # channels not contiguous
        fwa.fwa_forward(q.transpose(1, 2).contiguous().transpose(1, 2), k, v, w.heads, w.scale)
    lib = binding.load_library()
    args = (q.data_ptr(), k.data_ptr(), v.data_ptr(), torch.empty_like(q).data_ptr(), w.N, w.L, w.C, w.heads, 0.1)
    tail = (None, None, 0, binding.FWA_BF16, None)
    assert lib.fwa_forward_strided(*args, w.C - 8, w.C, *tail) == binding.FWA_ERR_SHAPE      # rows overlap
    assert lib.fwa_forward_strided(*args, w.C + 4, w.C, *tail) == binding.FWA_ERR_ALIGN      # rows not 16-byte aligned


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("as_labels", [False, True])
def test_autograd_wrappers_against_the_oracle(oracle, fused, as_labels):
    import torch
    from paper_2501_06480_amd import autograd
    w = synth.swin_t_stage(1, shifted=True, backward=True).with_N(128)
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], w.k)
    bias = f32_device(bias64).requires_grad_(True)
    mask = None if as_labels else f32_device(x["mask"])
    mask_args = {"labels": torch.from_numpy(x["labels"]).cuda()} if as_labels else {}
    g = to_device(x, w, "d_o")
    if fused:
        buf, _ = fused_views(x, w, ("q", "k", "v"), torch)
        buf.requires_grad_(True)
        o = autograd.window_attention_qkv(buf, w.scale, bias, mask, **mask_args)
        o.backward(g)
        d = w.C // w.heads
        grads = [buf.grad[:, :, t].reshape(w.N, w.L, w.C) for t in range(3)]
    else:
        q, k, v = (to_device(x, w, n).requires_grad_(True) for n in ("q", "k", "v"))
        o = autograd.window_attention(q, k, v, w.heads, w.scale, bias, mask, **mask_args)
        o.backward(g)
        grads = [q.grad, k.grad, v.grad]
    torch.cuda.synchronize()
    want_o = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, x["mask"])
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias64, x["mask"])
    check_bf16_output(to_f64(o), want_o, "o")
    for got, want, nme in zip(grads, ref[:3], ("dq", "dk", "dv")):
        check_bf16_output(to_f64(got), want, nme)
    assert max_abs(to_f64(bias.grad), ref[3]) <= TOL["bf16"]
