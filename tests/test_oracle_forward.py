"""Pins for the fp64 oracle's forward: brute force, closed forms, invariants.

None of these retypes the oracle's own loop nest: the brute force works
token by token in pure Python with un-shifted exponentials, the rest are
closed forms or properties that the definition (paper eq. 2-4) implies.
"""
import itertools
import math

import numpy as np
import pytest

from paper_2501_06480_amd import synth


def brute_forward(q, k, v, heads, scale, bias=None, mask=None):
    """Scalar Python loops, weights exp(s) without max subtraction."""
    N, L, C = q.shape
    d = C // heads
    o = np.zeros((N, L, C))
    for n, h, i in itertools.product(range(N), range(heads), range(L)):
        w = []
        for j in range(L):
            s = 0.0
            for c in range(d):
                s += float(q[n, i, h * d + c]) * float(k[n, j, h * d + c])
            s *= scale
            if bias is not None:
                s += float(bias[h, i, j])
            if mask is not None:
                s += float(mask[n % mask.shape[0], i, j])
            w.append(math.exp(s))
        z = math.fsum(w)
        for c in range(d):
            o[n, i, h * d + c] = math.fsum(w[j] * float(v[n, j, h * d + c]) for j in range(L)) / z
    return o


@pytest.mark.parametrize("N,L,d,heads,nW", [
    (1, 1, 1, 1, 0), (1, 2, 1, 1, 0), (3, 3, 2, 2, 0), (1, 5, 4, 1, 0), (3, 5, 4, 2, 3),
    (4, 3, 2, 2, 2), (6, 4, 3, 3, 3), (2, 7, 1, 2, 1),
])
@pytest.mark.parametrize("use_bias", [False, True])
def test_brute_force_tiny(oracle, N, L, d, heads, nW, use_bias):
    r = synth.rng(7 + N * 100 + L * 10 + d)
    C = heads * d
    q, k, v = (r.standard_normal((N, L, C)) for _ in range(3))
    bias = r.standard_normal((heads, L, L)) if use_bias else None
    mask = r.standard_normal((nW, L, L)) * 2 if nW else None
    scale = 0.37
    got = oracle.forward(q, k, v, heads, scale, bias, mask)
    want = brute_forward(q, k, v, heads, scale, bias, mask)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_L1_output_is_v(oracle):
    r = synth.rng(1)
    q, k, v = (r.standard_normal((5, 1, 8)) for _ in range(3))
    bias = r.standard_normal((2, 1, 1))
    np.testing.assert_array_equal(oracle.forward(q, k, v, 2, 0.5, bias), v)


def test_L2_is_logistic(oracle):
    r = synth.rng(2)
    q, k, v = (r.standard_normal((4, 2, 6)) for _ in range(3))
    scale = 0.7
    o = oracle.forward(q, k, v, 1, scale)
    for n in range(4):
        for i in range(2):
            s = scale * (k[n] @ q[n, i])
            p0 = 1.0 / (1.0 + math.exp(s[1] - s[0]))
            want = p0 * v[n, 0] + (1 - p0) * v[n, 1]
            np.testing.assert_allclose(o[n, i], want, atol=1e-14)


def test_equal_keys_give_uniform_weights(oracle):
    r = synth.rng(3)
    N, L, C = 3, 9, 8
    q, v = r.standard_normal((N, L, C)), r.standard_normal((N, L, C))
    k = np.broadcast_to(r.standard_normal((N, 1, C)), (N, L, C)).copy()
    o, p = oracle.forward(q, k, v, 2, 1.3, return_p=True)
    np.testing.assert_allclose(p, 1.0 / L, atol=1e-15)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), o.shape), atol=1e-14)


def test_rows_of_p_sum_to_one_and_are_positive(oracle):
    w = synth.swin_t_stage(3, shifted=True).with_N(8)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k)
    _, p = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias, x["mask"], return_p=True)
    np.testing.assert_allclose(p.sum(axis=-1), 1.0, atol=1e-14)
    assert (p >= 0).all() and (p <= 1).all()


def test_zero_query_gives_mean_of_values(oracle):
    r = synth.rng(4)
    N, L, C, heads = 4, 49, 96, 3
    k, v = r.standard_normal((N, L, C)), r.standard_normal((N, L, C))
    o = oracle.forward(np.zeros((N, L, C)), k, v, heads, 32 ** -0.5)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), o.shape), atol=1e-14)


def test_joint_key_value_permutation_leaves_output_unchanged(oracle):
    r = synth.rng(5)
    N, L, C, heads, nW = 4, 13, 8, 2, 2
    q, k, v = (r.standard_normal((N, L, C)) for _ in range(3))
    bias, mask = r.standard_normal((heads, L, L)), r.standard_normal((nW, L, L))
    perm = r.permutation(L)
    o1 = oracle.forward(q, k, v, heads, 0.4, bias, mask)
    o2 = oracle.forward(q, k[:, perm], v[:, perm], heads, 0.4, bias[:, :, perm], mask[:, :, perm])
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    # permuting the queries (and the rows of B, M) permutes the output rows
    o3 = oracle.forward(q[:, perm], k, v, heads, 0.4, bias[:, perm, :], mask[:, perm, :])
    np.testing.assert_allclose(o3, o1[:, perm], atol=1e-14)


def test_constant_added_to_a_score_row_has_no_effect(oracle):
    r = synth.rng(6)
    N, L, C, heads = 3, 11, 12, 3
    q, k, v = (r.standard_normal((N, L, C)) for _ in range(3))
    bias = r.standard_normal((heads, L, L))
    shift = r.standard_normal((heads, L, 1)) * 30.0
    o1 = oracle.forward(q, k, v, heads, 0.5, bias)
    o2 = oracle.forward(q, k, v, heads, 0.5, bias + shift)
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    # and exp never overflows thanks to the row-max subtraction
    o3 = oracle.forward(q, k, v, heads, 0.5, bias + 5000.0)
    np.testing.assert_allclose(o1, o3, atol=1e-9)


def test_output_is_linear_in_v(oracle):
    r = synth.rng(8)
    N, L, C, heads = 2, 10, 8, 2
    q, k, v1, v2 = (r.standard_normal((N, L, C)) for _ in range(4))
    a = 1.75
    lhs = oracle.forward(q, k, v1 + a * v2, heads, 0.6)
    rhs = oracle.forward(q, k, v1, heads, 0.6) + a * oracle.forward(q, k, v2, heads, 0.6)
    np.testing.assert_allclose(lhs, rhs, atol=1e-13)


def test_heads_are_independent_channel_slices(oracle):
    r = synth.rng(9)
    N, L, heads, d = 3, 7, 3, 4
    q, k, v = (r.standard_normal((N, L, heads * d)) for _ in range(3))
    bias = r.standard_normal((heads, L, L))
    o = oracle.forward(q, k, v, heads, 0.5, bias)
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        oh = oracle.forward(q[..., sl], k[..., sl], v[..., sl], 1, 0.5, bias[h:h + 1])
        np.testing.assert_array_equal(o[..., sl], oh)


def test_feature_chunk_identity(oracle):
    """Paper eq. 5-6: S is the sum of per-chunk products, O_i = P V_i.

    The oracle does not expose S, but log P equals S up to a per-row
    constant, so row-centred log P must be additive over feature chunks.
    """
    r = synth.rng(10)
    N, L, d = 2, 12, 32
    q, k, v = (r.standard_normal((N, L, d)) for _ in range(3))
    scale = d ** -0.5

    def centred_log_p(qc, kc):
        _, p = oracle.forward(qc, kc, np.zeros_like(qc), 1, scale, return_p=True)
        lp = np.log(p)
        return lp - lp.mean(axis=-1, keepdims=True)

    full = centred_log_p(q, k)
    o, p = oracle.forward(q, k, v, 1, scale, return_p=True)
    for rchunks in (2, 4, 32):
        w = d // rchunks
        acc = sum(centred_log_p(q[..., i * w:(i + 1) * w], k[..., i * w:(i + 1) * w]) for i in range(rchunks))
        np.testing.assert_allclose(acc, full, atol=1e-12)
        for i in range(rchunks):
            np.testing.assert_allclose(o[..., i * w:(i + 1) * w], p[:, 0] @ v[..., i * w:(i + 1) * w], atol=1e-13)


def test_block_mask_limit_equals_separate_attention(oracle):
    r = synth.rng(11)
    N, L, C, heads = 4, 10, 8, 2
    q, k, v = (r.standard_normal((N, L, C)) for _ in range(3))
    groups = [np.array([0, 3, 4, 9]), np.array([1, 2]), np.array([5, 6, 7, 8])]
    lab = np.empty(L, dtype=int)
    for g, idx in enumerate(groups):
        lab[idx] = g
    mask = np.where(lab[:, None] == lab[None, :], 0.0, -1e9)[None]
    o = oracle.forward(q, k, v, heads, 0.8, None, mask)
    for idx in groups:
        sub = oracle.forward(q[:, idx], k[:, idx], v[:, idx], heads, 0.8)
        np.testing.assert_allclose(o[:, idx], sub, atol=1e-14)


def test_mask_is_indexed_by_window_modulo(oracle):
    r = synth.rng(12)
    N, L, C, nW = 6, 5, 4, 3
    q, k, v = (r.standard_normal((N, L, C)) for _ in range(3))
    mask = r.standard_normal((nW, L, L)) * 3
    o = oracle.forward(q, k, v, 1, 0.5, None, mask)
    for n in range(N):
        on = oracle.forward(q[n:n + 1], k[n:n + 1], v[n:n + 1], 1, 0.5, None, mask[n % nW][None])
        np.testing.assert_array_equal(o[n:n + 1], on)


@pytest.mark.parametrize("wl", ["c1", "s1_shift", "s4", "L144"])
def test_library_float64_expression_third_opinion(oracle, wl):
    """With real shapes: a torch float64 softmax/matmul expression agrees."""
    import torch
    w = {"c1": synth.config1(), "s1_shift": synth.swin_t_stage(1, shifted=True).with_N(128),
         "s4": synth.swin_t_stage(4).with_N(4), "L144": synth.config4()[0].with_N(16)}[wl]
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k) if w.use_bias else None
    got = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias, x["mask"])
    d = w.C // w.heads
    tq, tk, tv = (torch.from_numpy(x[n].astype(np.float64)).view(w.N, w.L, w.heads, d).permute(0, 2, 1, 3)
                  for n in ("q", "k", "v"))
    s = torch.matmul(tq, tk.transpose(-1, -2)) * w.scale
    if bias is not None:
        s = s + torch.from_numpy(bias)[None]
    if x["mask"] is not None:
        m = torch.from_numpy(x["mask"].astype(np.float64))
        s = (s.view(w.N // w.nW, w.nW, w.heads, w.L, w.L) + m[None, :, None]).view(w.N, w.heads, w.L, w.L)
    want = torch.matmul(torch.softmax(s, dim=-1), tv).permute(0, 2, 1, 3).reshape(w.N, w.L, w.C).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_bad_arguments_raise(oracle):
    x = np.zeros((4, 3, 6))
    with pytest.raises(ValueError):
        oracle.forward(x, x, x, 4, 1.0)             # C % heads != 0
    with pytest.raises(ValueError):
        oracle.forward(x, x, x, 2, 1.0, None, np.zeros((3, 3, 3)))   # N % nW != 0
    with pytest.raises(ValueError):
        oracle.forward(x, x, x, 2, 1.0, np.zeros((2, 3, 4)))         # bias shape


def test_empty_batch(oracle):
    x = np.zeros((0, 5, 4))
    assert oracle.forward(x, x, x, 2, 1.0).shape == (0, 5, 4)
