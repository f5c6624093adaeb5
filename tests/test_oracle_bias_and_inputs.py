"""Pins for the relative-position gather/scatter of the oracle and for the input generators."""
import numpy as np
import pytest

from paper_2501_06480_amd import synth


def test_gather_k2_written_out_by_hand(oracle):
    # k = 2: tokens 0..3 at (0,0) (0,1) (1,0) (1,1); table is 3x3, entry (dy+1)*3 + (dx+1).
    table = np.arange(9, dtype=np.float64)[None] * 10
    want = np.array([[40, 30, 10, 0],
                     [50, 40, 20, 10],
                     [70, 60, 40, 30],
                     [80, 70, 50, 40]], dtype=np.float64)
    np.testing.assert_array_equal(oracle.bias_gather(table, 2)[0], want)


@pytest.mark.parametrize("k", [1, 3, 7, 12, 16])
def test_gather_depends_only_on_relative_offset(oracle, k):
    heads = 2
    table = synth.bias_table(heads, k, 5).astype(np.float64)
    b = oracle.bias_gather(table, k)
    L = k * k
    ys, xs = np.divmod(np.arange(L), k)
    centre = (k - 1) * (2 * k - 1) + (k - 1)
    for h in range(heads):
        np.testing.assert_array_equal(np.diag(b[h]), np.full(L, table[h, centre]))
    seen = {}
    for i in range(L):
        for j in range(L):
            key = (ys[i] - ys[j], xs[i] - xs[j])
            val = b[1, i, j]
            assert seen.setdefault(key, val) == val
    assert len(seen) == (2 * k - 1) ** 2
    # every table entry is used, and the corner pairs hit the table corners
    assert set(np.unique(b[1])) == set(np.unique(table[1]))
    assert b[0, 0, L - 1] == table[0, 0]                 # dy = dx = -(k-1)
    assert b[0, L - 1, 0] == table[0, -1]                # dy = dx = +(k-1)
    if k > 1:
        assert b[0, 0, k - 1] == table[0, (k - 1) * (2 * k - 1)]   # same row, dx = -(k-1)


@pytest.mark.parametrize("k", [2, 7])
def test_scatter_is_the_adjoint_of_gather(oracle, k):
    r = synth.rng(31)
    heads, L = 3, k * k
    t = r.standard_normal((heads, (2 * k - 1) ** 2))
    g = r.standard_normal((heads, L, L))
    lhs = float((oracle.bias_gather(t, k) * g).sum())
    rhs = float((t * oracle.bias_scatter(g, k)).sum())
    assert abs(lhs - rhs) < 1e-10
    # counts: scattering all-ones counts how often each offset occurs: (k-|dy|)(k-|dx|)
    cnt = oracle.bias_scatter(np.ones((1, L, L)), k)[0].reshape(2 * k - 1, 2 * k - 1)
    dy = np.abs(np.arange(2 * k - 1) - (k - 1))
    np.testing.assert_array_equal(cnt, np.outer(k - dy, k - dy))


def test_bf16_round_matches_torch_and_is_idempotent():
    import torch
    x = synth.normal((4096,), 3) * 7
    x[:8] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38, -1e-40, 65504.0]
    vals, bits = synth.bf16_round(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(vals, t.to(torch.float32).numpy())
    np.testing.assert_array_equal(bits.view(np.int16), t.view(torch.int16).numpy())
    np.testing.assert_array_equal(synth.bf16_round(vals)[0], vals)
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(bits), vals)


def test_draw_is_seeded_and_distinct():
    w = synth.swin_t_stage(3, shifted=True, backward=True).with_N(8)
    a, b = synth.draw(w), synth.draw(w)
    for n in ("q", "k", "v", "d_o", "table", "mask"):
        np.testing.assert_array_equal(a[n], b[n])
    assert not np.array_equal(a["q"], a["k"])
    assert abs(a["q"].std() - 1.0) < 0.02 and abs(a["q"].mean()) < 0.02
    assert abs(a["table"].std() - 0.02) < 0.004


def test_shift_mask_structure():
    m = synth.shift_mask(56, 56, 7, 3)
    assert m.shape == (64, 49, 49) and m.dtype == np.float32
    assert set(np.unique(m)) == {-100.0, 0.0}
    np.testing.assert_array_equal(m, m.transpose(0, 2, 1))
    assert (np.diagonal(m, axis1=1, axis2=2) == 0).all()
    nonzero = [w for w in range(64) if m[w].any()]
    # only the last window row and column see more than one region: 8 + 8 - 1 windows
    assert nonzero == sorted(set(range(56, 64)) | set(range(7, 64, 8)))
    # last window: 4 regions of 4x4, 4x3, 3x4, 3x3 tokens -> allowed pairs
    assert (m[63] == 0).sum() == 16 ** 2 + 12 ** 2 + 12 ** 2 + 9 ** 2
    # a window in the last column (not the corner): two regions of 7x4 and 7x3 tokens
    assert (m[7] == 0).sum() == 28 ** 2 + 21 ** 2


def test_shift_mask_single_window_map():
    m = synth.shift_mask(7, 7, 7, 3)
    assert m.shape == (1, 49, 49)
    assert (m[0] == 0).sum() == 16 ** 2 + 12 ** 2 + 12 ** 2 + 9 ** 2


def test_mask_from_labels_written_out_by_hand(oracle):
    # two windows of 4 tokens; the second has three regions
    lab = np.array([[5, 5, 5, 5], [0, 1, 0, 2]], dtype=np.int32)
    m = oracle.mask_from_labels(lab, -7.5)
    x = -7.5
    want1 = np.array([[0, x, 0, x],
                      [x, 0, x, x],
                      [0, x, 0, x],
                      [x, x, x, 0]], dtype=np.float64)
    np.testing.assert_array_equal(m[0], np.zeros((4, 4)))
    np.testing.assert_array_equal(m[1], want1)


def test_mask_from_labels_properties(oracle):
    g = np.random.default_rng(11)
    lab = g.integers(0, 4, size=(5, 13)).astype(np.int32)
    m = oracle.mask_from_labels(lab, -100.0)
    assert m.shape == (5, 13, 13)
    np.testing.assert_array_equal(m, m.transpose(0, 2, 1))            # an equivalence relation: symmetric,
    assert (np.diagonal(m, axis1=1, axis2=2) == 0).all()               # reflexive,
    for w in range(5):                                                 # and its classes are the label classes
        for i in range(13):
            np.testing.assert_array_equal(np.flatnonzero(m[w, i] == 0), np.flatnonzero(lab[w] == lab[w, i]))
    # relabelling the regions changes nothing; a window only sees its own labels
    np.testing.assert_array_equal(oracle.mask_from_labels(17 - 3 * lab, -100.0), m)
    np.testing.assert_array_equal(oracle.mask_from_labels(lab[2:3], -100.0)[0], m[2])
    # the value is taken as given (the oracle does not hard-wire -100)
    np.testing.assert_array_equal(oracle.mask_from_labels(lab, 2.5), m * (2.5 / -100.0))


@pytest.mark.parametrize("H,k,shift", [(56, 7, 3), (28, 7, 3), (7, 7, 3), (24, 12, 6)])
def test_mask_from_labels_reproduces_the_shift_mask(oracle, H, k, shift):
    # third opinion: the generator's dense mask, built by broadcasting, against the oracle's loops
    lab = synth.shift_labels(H, H, k, shift)
    assert lab.shape == ((H // k) ** 2, k * k) and lab.dtype == np.int32
    np.testing.assert_array_equal(oracle.mask_from_labels(lab, -100.0), synth.shift_mask(H, H, k, shift))


def test_masked_attention_is_attention_inside_each_region(oracle):
    # With a large negative value, a token attends only inside its region: the output equals
    # plain attention over the region's tokens alone (the block-diagonal limit, per label class).
    g = np.random.default_rng(3)
    L, C, heads = 9, 8, 2
    q, k, v = (g.standard_normal((2, L, C)) for _ in range(3))
    lab = np.array([[0, 0, 1, 0, 1, 1, 2, 0, 2], [3, 3, 3, 3, 3, 3, 3, 3, 3]], dtype=np.int32)
    o = oracle.forward(q, k, v, heads, 0.5, mask=oracle.mask_from_labels(lab, -1e4))
    for w in range(2):
        for c in np.unique(lab[w]):
            idx = np.flatnonzero(lab[w] == c)
            sub = oracle.forward(q[w:w + 1, idx], k[w:w + 1, idx], v[w:w + 1, idx], heads, 0.5)
            np.testing.assert_allclose(o[w, idx], sub[0], rtol=0, atol=1e-12)


def test_workload_shapes_match_the_configs():
    assert (synth.config1().N, synth.config1().dtype) == (64, "f32")
    c2 = synth.config2()
    assert (c2.N, c2.L, c2.C, c2.heads) == (8192, 49, 96, 3) and abs(c2.scale - 32 ** -0.5) < 1e-12
    shapes = [(w.N, w.C, w.heads, w.nW, w.shift) for w in synth.config3()]
    assert shapes == [(8192, 96, 3, 64, 0), (8192, 96, 3, 64, 3), (2048, 192, 6, 16, 0), (2048, 192, 6, 16, 3),
                      (512, 384, 12, 4, 0), (512, 384, 12, 4, 3), (128, 768, 24, 1, 0), (128, 768, 24, 1, 0)]
    a, b = synth.config4()
    assert (a.N, a.L, a.C, a.heads, b.N, b.L) == (1024, 144, 128, 4, 1024, 256)
    s1, s3 = synth.config5()
    assert s1.backward and (s1.N, s3.N, s3.C, s3.heads, s3.nW) == (8192, 512, 384, 12, 4)
