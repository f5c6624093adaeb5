"""Pins for the fp64 oracle's backward (paper Algorithm 2).

The gradients are checked against what the *forward* implies (central
differences, the adjoint identity), against closed forms, and against
properties of the softmax Jacobian -- never against a retyped copy of the
backward formulas.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth


def loss(oracle, q, k, v, g, heads, scale, bias, mask):
    return float((oracle.forward(q, k, v, heads, scale, bias, mask) * g).sum())


@pytest.mark.parametrize("N,L,d,heads,nW,use_bias", [
    (1, 3, 2, 1, 0, False), (2, 4, 3, 2, 2, True), (3, 5, 4, 2, 3, True), (2, 2, 1, 1, 1, False),
    (4, 3, 2, 3, 2, True),
])
def test_central_differences(oracle, N, L, d, heads, nW, use_bias):
    r = synth.rng(100 + N + 10 * L)
    C = heads * d
    q, k, v, g = (r.standard_normal((N, L, C)) for _ in range(4))
    bias = r.standard_normal((heads, L, L)) if use_bias else None
    mask = r.standard_normal((nW, L, L)) if nW else None
    scale = 0.45
    dq, dk, dv, db = oracle.backward(q, k, v, g, heads, scale, bias, mask, want_dbias=True)
    eps = 1e-6

    def fd(arr, which):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            lp = loss(oracle, q, k, v, g, heads, scale, bias, mask)
            arr[idx] = old - eps
            lm = loss(oracle, q, k, v, g, heads, scale, bias, mask)
            arr[idx] = old
            out[idx] = (lp - lm) / (2 * eps)
        return out

    np.testing.assert_allclose(dq, fd(q, "q"), atol=2e-8)
    np.testing.assert_allclose(dk, fd(k, "k"), atol=2e-8)
    np.testing.assert_allclose(dv, fd(v, "v"), atol=2e-8)
    if use_bias:
        np.testing.assert_allclose(db, fd(bias, "b"), atol=2e-8)
    else:
        # dB is still defined (gradient w.r.t. an all-zero bias)
        zb = np.zeros((heads, L, L))
        bias = zb
        np.testing.assert_allclose(db, fd(zb, "b"), atol=2e-8)


@pytest.mark.parametrize("wl", ["s1", "s3", "L144"])
def test_adjoint_identity_at_real_shapes(oracle, wl):
    """<dO, J dx> == <J^T dO, dx> with J dx from a central difference of the forward."""
    w = {"s1": synth.swin_t_stage(1, shifted=True, backward=True).with_N(64),
         "s3": synth.swin_t_stage(3, shifted=True, backward=True).with_N(8),
         "L144": synth.config4()[0].with_N(16)}[wl]
    w.backward = True
    x = synth.draw(w)
    q, k, v, g = (x[n].astype(np.float64) for n in ("q", "k", "v", "d_o"))
    bias = oracle.bias_gather(x["table"], w.k)
    mask = x["mask"]
    dq, dk, dv, db = oracle.backward(q, k, v, g, w.heads, w.scale, bias, mask)
    r = synth.rng(55)
    tq, tk, tv = (r.standard_normal(q.shape) for _ in range(3))
    tb = r.standard_normal(bias.shape)
    eps = 1e-5
    fp = oracle.forward(q + eps * tq, k + eps * tk, v + eps * tv, w.heads, w.scale, bias + eps * tb, mask)
    fm = oracle.forward(q - eps * tq, k - eps * tk, v - eps * tv, w.heads, w.scale, bias - eps * tb, mask)
    lhs = float((g * (fp - fm)).sum() / (2 * eps))
    rhs = float((dq * tq).sum() + (dk * tk).sum() + (dv * tv).sum() + (db * tb).sum())
    assert abs(lhs - rhs) <= 1e-6 * max(1.0, abs(lhs)), (lhs, rhs)
    # and one tensor at a time, so that errors cannot cancel between them
    for name, t, grad in (("q", tq, dq), ("k", tk, dk), ("v", tv, dv)):
        args = {"q": q, "k": k, "v": v}
        ap = dict(args); am = dict(args)
        ap[name] = args[name] + eps * t
        am[name] = args[name] - eps * t
        fp = oracle.forward(ap["q"], ap["k"], ap["v"], w.heads, w.scale, bias, mask)
        fm = oracle.forward(am["q"], am["k"], am["v"], w.heads, w.scale, bias, mask)
        lhs = float((g * (fp - fm)).sum() / (2 * eps))
        rhs = float((grad * t).sum())
        assert abs(lhs - rhs) <= 1e-6 * max(1.0, abs(lhs)), (name, lhs, rhs)


def test_L1_closed_form(oracle):
    r = synth.rng(21)
    q, k, v, g = (r.standard_normal((5, 1, 8)) for _ in range(4))
    dq, dk, dv, db = oracle.backward(q, k, v, g, 2, 0.5)
    np.testing.assert_array_equal(dv, g)
    np.testing.assert_array_equal(dq, np.zeros_like(q))
    np.testing.assert_array_equal(dk, np.zeros_like(q))
    np.testing.assert_array_equal(db, np.zeros((2, 1, 1)))


def test_dv_is_independent_of_v_and_linear_in_do(oracle):
    r = synth.rng(22)
    N, L, C, heads = 3, 9, 8, 2
    q, k, v1, v2, g1, g2 = (r.standard_normal((N, L, C)) for _ in range(6))
    a = oracle.backward(q, k, v1, g1, heads, 0.6)
    b = oracle.backward(q, k, v2, g1, heads, 0.6)
    np.testing.assert_allclose(a[2], b[2], atol=1e-14)
    c = oracle.backward(q, k, v1, g1 + 2.5 * g2, heads, 0.6)
    d = oracle.backward(q, k, v1, g2, heads, 0.6)
    for x, y, z in zip(c, a, d):
        np.testing.assert_allclose(x, y + 2.5 * z, atol=1e-12)


def test_dv_equals_p_transpose_do(oracle):
    r = synth.rng(23)
    N, L, C, heads = 3, 9, 8, 2
    q, k, v, g = (r.standard_normal((N, L, C)) for _ in range(4))
    _, p = oracle.forward(q, k, v, heads, 0.6, return_p=True)
    dv = oracle.backward(q, k, v, g, heads, 0.6)[2]
    d = C // heads
    for h in range(heads):
        want = np.einsum("nij,nic->njc", p[:, h], g[..., h * d:(h + 1) * d])
        np.testing.assert_allclose(dv[..., h * d:(h + 1) * d], want, atol=1e-14)


def test_dbias_rows_sum_to_zero(oracle):
    """Rows of dS sum to zero (softmax Jacobian annihilates constants)."""
    w = synth.swin_t_stage(3, shifted=True, backward=True).with_N(8)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k)
    db = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias, x["mask"])[3]
    np.testing.assert_allclose(db.sum(axis=-1), 0.0, atol=1e-11)
    assert np.abs(db).max() > 0.1


def test_scale_zero_kills_dq_dk(oracle):
    r = synth.rng(24)
    q, k, v, g = (r.standard_normal((2, 6, 8)) for _ in range(4))
    dq, dk, dv, db = oracle.backward(q, k, v, g, 2, 0.0)
    assert np.abs(dq).max() == 0 and np.abs(dk).max() == 0
    # uniform P: dV_j = mean over queries of dO
    np.testing.assert_allclose(dv, np.broadcast_to(g.mean(axis=1, keepdims=True), g.shape), atol=1e-14)


def test_dq_dk_scale_with_scale_only_through_chain_rule(oracle):
    """Folding the scale into Q must give the same dK and scale*dQ_folded == dQ."""
    r = synth.rng(25)
    q, k, v, g = (r.standard_normal((2, 7, 8)) for _ in range(4))
    s = 0.3
    dq, dk, dv, _ = oracle.backward(q, k, v, g, 2, s)
    dq2, dk2, dv2, _ = oracle.backward(q * s, k, v, g, 2, 1.0)
    np.testing.assert_allclose(dq, s * dq2, atol=1e-14)
    np.testing.assert_allclose(dk, dk2, atol=1e-14)
    np.testing.assert_allclose(dv, dv2, atol=1e-14)


def test_dbias_sums_over_windows_and_is_thread_count_independent(oracle):
    r = synth.rng(26)
    N, L, C, heads = 12, 5, 6, 3
    q, k, v, g = (r.standard_normal((N, L, C)) for _ in range(4))
    db = oracle.backward(q, k, v, g, heads, 0.5)[3]
    per = sum(oracle.backward(q[n:n + 1], k[n:n + 1], v[n:n + 1], g[n:n + 1], heads, 0.5)[3] for n in range(N))
    np.testing.assert_allclose(db, per, atol=1e-13)
    db1 = oracle.backward(q, k, v, g, heads, 0.5, threads=1)[3]
    db3 = oracle.backward(q, k, v, g, heads, 0.5, threads=3)[3]
    np.testing.assert_allclose(db1, db3, atol=1e-13)
    oracle.backward(q, k, v, g, heads, 0.5, threads=0)


def test_autograd_float64_third_opinion(oracle):
    import torch
    w = synth.swin_t_stage(2, shifted=True, backward=True).with_N(32)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k)
    got = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias, x["mask"])
    d = w.C // w.heads
    tq, tk, tv = (torch.from_numpy(x[n].astype(np.float64)).requires_grad_() for n in ("q", "k", "v"))
    tb = torch.from_numpy(bias).requires_grad_()
    hq, hk, hv = (t.view(w.N, w.L, w.heads, d).permute(0, 2, 1, 3) for t in (tq, tk, tv))
    s = torch.matmul(hq, hk.transpose(-1, -2)) * w.scale + tb[None]
    m = torch.from_numpy(x["mask"].astype(np.float64))
    s = (s.view(w.N // w.nW, w.nW, w.heads, w.L, w.L) + m[None, :, None]).view(w.N, w.heads, w.L, w.L)
    o = torch.matmul(torch.softmax(s, dim=-1), hv).permute(0, 2, 1, 3).reshape(w.N, w.L, w.C)
    o.backward(torch.from_numpy(x["d_o"].astype(np.float64)))
    for a, b in zip(got, (tq.grad, tk.grad, tv.grad, tb.grad)):
        np.testing.assert_allclose(a, b.numpy(), rtol=0, atol=1e-12)


def test_empty_batch(oracle):
    x = np.zeros((0, 5, 4))
    dq, dk, dv, db = oracle.backward(x, x, x, x, 2, 1.0)
    assert dq.shape == (0, 5, 4) and np.abs(db).max() == 0
