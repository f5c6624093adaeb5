"""GPU parity of fwa_forward against the fp64 oracle, element by element.

Every call goes through the C ABI (ctypes binding).  Tolerances are the ones
the task fixes: 1e-5 max-abs for fp32, 1e-2 for bf16 data with fp32
accumulation.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, bf16_round_f64, check_forward_arithmetic_bound, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu


def run_forward(w, x, bias_np=None):
    import paper_2501_06480_amd as fwa
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    bias = None
    if w.use_bias:
        bias = fwa.fwa_bias_gather(f32_device(x["table"]), w.k) if bias_np is None else f32_device(bias_np)
    mask = f32_device(x["mask"])
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, bias, mask)
    return o, bias


def check_forward(oracle, w, label=""):
    import torch
    x = synth.draw(w)
    o, bias = run_forward(w, x)
    torch.cuda.synchronize()
    bias64 = None
    if w.use_bias:
        bias64 = oracle.bias_gather(x["table"], w.k)
        # the gather is index work: bit-exact
        np.testing.assert_array_equal(to_f64(bias), bias64)
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, x["mask"])
    got = to_f64(o)
    assert np.isfinite(got).all()
    err = max_abs(got, want)
    print(f"{label or w.name}: max|ref|={np.abs(want).max():.3f} max-abs err={err:.3e}", flush=True)
    assert err <= TOL[w.dtype], (w.name, err)
    if w.dtype == "bf16":
        # against the oracle rounded to bf16 the results differ by at most one bf16 ulp (2^-7 relative)
        err_r = max_abs(got, bf16_round_f64(want))
        assert err_r <= 2.0 ** -7 * max(1.0, np.abs(want).max()), err_r
    return err


def test_config1_single_head_fp32(oracle):
    check_forward(oracle, synth.config1())


def test_swin_t_stage1_small_bf16(oracle):
    check_forward(oracle, synth.config2().with_N(70))   # 70 windows: ragged last workgroup


@pytest.mark.parametrize("stage", [1, 2, 3, 4])
@pytest.mark.parametrize("shifted", [False, True])
def test_swin_t_stages_bias_and_mask_bf16(oracle, stage, shifted):
    w = synth.swin_t_stage(stage, shifted=shifted)
    n_small = max(w.nW, 1) * (2 if stage < 4 else 8)
    check_forward(oracle, w.with_N(n_small))


@pytest.mark.parametrize("stage,N", [(1, 2560), (2, 1008), (3, 1028)])
@pytest.mark.parametrize("which", ["bias+mask", "bias", "mask"])
def test_many_windows_per_workgroup_with_bias_and_mask(oracle, stage, N, which):
    """Enough windows that each workgroup walks several of them with its bias/mask term held
    on chip (the window count is not a multiple of the workgroup count: uneven walks)."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.swin_t_stage(stage, shifted=True).with_N(N)
    assert N % w.nW == 0
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], w.k) if "bias" in which else None
    mask = x["mask"] if "mask" in which else None
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias64), f32_device(mask))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, mask)
    err = max_abs(to_f64(o), want)
    print(f"{w.name} {which}: err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]


@pytest.mark.parametrize("L", [9, 16, 25, 32, 36, 48, 64])
@pytest.mark.parametrize("heads", [2, 3, 4])
def test_all_heads_of_a_window_in_one_workgroup(oracle, L, heads):
    """2 to 4 heads with bias and mask and enough windows for the persistent walk: one wave per head
    and 16-query block, every key-block count from 1 to 4, an odd number of windows per workgroup."""
    import torch
    import paper_2501_06480_amd as fwa
    nW, N = 4, 4 * 73
    w = synth.Workload(f"allheads_L{L}_h{heads}", N, L, 32 * heads, heads, "bf16", 7800 + L + heads, 0)
    x = synth.draw(w)
    bias = synth.normal((heads, L, L), 7900 + L, 0.5)
    mask = np.where(synth.rng(7950 + L).random((nW, L, L)) < 0.3, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), f32_device(mask))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias, mask)
    # few keys per row and |V| up to 4-5: held to the bound derived from the arithmetic, element by element
    spread = oracle.forward(x["q"], x["k"], np.abs(x["v"]), heads, w.scale, bias, mask)
    err = check_forward_arithmetic_bound(to_f64(o), want, spread, w.name)
    print(f"{w.name}: err={err:.3e}", flush=True)
    assert err <= 1.5e-2


@pytest.mark.parametrize("L,k,hw,heads,N", [(144, 12, 48, 4, 176), (256, 16, 64, 4, 80), (196, 14, 56, 3, 48),
                                            (81, 9, 18, 2, 300)])
@pytest.mark.parametrize("which", ["bias+mask", "bias", "mask"])
def test_large_windows_many_windows_per_workgroup(oracle, L, k, hw, heads, N, which):
    """Large windows with bias / mask: each wave keeps the additive term of its 16 query rows on
    chip and walks several windows (one or two workgroups per head, uneven walks)."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload(f"L{L}_h{heads}", N, L, 32 * heads, heads, "bf16", 7000 + L, k, hw, True, k // 2)
    assert N % w.nW == 0
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], w.k) if "bias" in which else None
    mask = x["mask"] if "mask" in which else None
    q, kk, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, kk, v, w.heads, w.scale, f32_device(bias64), f32_device(mask))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, mask)
    err = max_abs(to_f64(o), want)
    print(f"{w.name} N={N} {which}: err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("L", [64, 49, 33, 16, 7])
@pytest.mark.parametrize("use_bm", [False, True])
def test_wide_heads(oracle, d, L, use_bm, dtype):
    """Head widths of the paper's kernel benchmark (L = 64, 4 heads, width per head swept): the
    score product runs over the feature dimension in chunks, the output in 16-channel blocks."""
    import torch
    import paper_2501_06480_amd as fwa
    heads, N = 4, 12
    w = synth.Workload(f"wide_d{d}_L{L}", N, L, d * heads, heads, dtype, 8000 + d + L, 0)
    assert abs(w.scale - d ** -0.5) < 1e-12
    x = synth.draw(w)
    bias = mask = None
    if use_bm:
        bias = synth.normal((heads, L, L), 41 + L, 0.5)
        mask = np.where(synth.rng(43 + L + d).random((3, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), f32_device(mask))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias, mask)
    err = max_abs(to_f64(o), want)
    print(f"{dtype} d={d} L={L} bm={use_bm}: max|ref|={np.abs(want).max():.2f} err={err:.3e}", flush=True)
    assert err <= TOL[dtype]


@pytest.mark.parametrize("N", [1365, 1366])
@pytest.mark.parametrize("which", ["none", "bias+own_mask"])
def test_both_sides_of_the_few_tiles_threshold(oracle, N, which):
    """Up to 4096 window-heads a wave takes one query block (4 waves per head), above that a wave
    walks all query blocks of its head: 1365 x 3 = 4095 and 1366 x 3 = 4098 window-heads.  A mask
    with one tile per window (period N) keeps the call off the kernel that walks windows."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload(f"few_tiles_N{N}", N, 49, 96, 3, "bf16", 7700 + N, 7, 0, True)
    x = synth.draw(w)
    bias64 = mask = None
    if which != "none":
        bias64 = oracle.bias_gather(x["table"], w.k)
        mask = np.where(synth.rng(7800 + N).random((N, 49, 49)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(49), np.arange(49)] = 0.0
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias64), f32_device(mask))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias64, mask)
    err = max_abs(to_f64(o), want)
    print(f"N={N} {which}: err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]


def test_stage4_single_window_map_with_mask(oracle):
    """A 7x7 map is one window; the shift mask then has 4 regions inside it."""
    w = synth.Workload("s4_masked", 8, 49, 768, 24, "bf16", 1234, 7, 7, True, 3)
    assert w.nW == 1
    check_forward(oracle, w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,k", [(1, 1), (4, 2), (9, 3), (16, 4), (25, 5), (36, 6), (49, 7), (64, 8), (81, 9),
                                 (100, 10), (144, 12), (169, 13), (196, 14), (225, 15), (256, 16)])
def test_every_key_block_count(oracle, dtype, L, k):
    """k*k windows for k = 1..16 hit every on-chip block count, full and ragged."""
    hw = 2 * k
    w = synth.Workload(f"L{L}_{dtype}", 4 * 3, L, 64, 2, dtype, 2000 + L, k, hw, True, k // 2)
    if k == 1:
        w.shift = 0
    check_forward(oracle, w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L", [2, 3, 15, 17, 31, 33, 47, 50, 63, 65, 127, 129, 143, 145, 250, 255])
def test_window_lengths_that_are_not_squares(oracle, dtype, L):
    """L need not be a square: bias and mask are passed as plain [.,L,L] tensors."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload(f"L{L}_{dtype}", 5, L, 96, 3, dtype, 3000 + L, 0)
    x = synth.draw(w)
    bias = synth.normal((3, L, L), 77 + L, 0.5)
    mask = np.where(synth.rng(5 + L).random((5, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, 3, w.scale, f32_device(bias), f32_device(mask))
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], 3, w.scale, bias, mask)
    err = max_abs(to_f64(o), want)
    print(f"L={L} {dtype}: err={err:.3e}", flush=True)
    assert err <= TOL[dtype]


@pytest.mark.parametrize("L", [49, 100])
@pytest.mark.parametrize("heads", [1, 2, 3, 4, 5, 6, 7, 8, 9, 12])
def test_head_counts_reach_every_kernel_variant(oracle, heads, L):
    """Odd/even head counts select different workgroup shapes (and, for L <= 64 with an odd
    count above 4, the kernel that reads head slices directly)."""
    import torch
    import paper_2501_06480_amd as fwa
    N = 6
    w = synth.Workload(f"heads{heads}_L{L}", N, L, 32 * heads, heads, "bf16", 6000 + heads + L, 0)
    x = synth.draw(w)
    bias = synth.normal((heads, L, L), 13 + heads, 0.5)
    mask = np.where(synth.rng(17 + heads).random((3, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    for use_bm in (False, True):
        o = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias) if use_bm else None,
                            f32_device(mask) if use_bm else None)
        torch.cuda.synchronize()
        want = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias if use_bm else None,
                              mask if use_bm else None)
        err = max_abs(to_f64(o), want)
        assert err <= TOL["bf16"], (heads, L, use_bm, err)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bias_only_mask_only_and_neither(oracle, dtype):
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload("combo", 8, 49, 96, 3, dtype, 4000, 7, 14, True, 3)
    x = synth.draw(w)
    bias64 = oracle.bias_gather(x["table"], 7)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    for use_b, use_m in ((False, False), (True, False), (False, True), (True, True)):
        o = fwa.fwa_forward(q, k, v, 3, w.scale, f32_device(bias64) if use_b else None,
                            f32_device(x["mask"]) if use_m else None)
        torch.cuda.synchronize()
        want = oracle.forward(x["q"], x["k"], x["v"], 3, w.scale, bias64 if use_b else None,
                              x["mask"] if use_m else None)
        assert max_abs(to_f64(o), want) <= TOL[dtype], (use_b, use_m)


def test_large_score_offsets_do_not_overflow(oracle):
    """Scores shifted by +-80 per row (through the bias) must give the same output."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload("shifted_scores", 6, 49, 64, 2, "f32", 4100, 7)
    x = synth.draw(w)
    bias = (synth.normal((2, 49, 1), 9, 40.0) + np.zeros((2, 49, 49), dtype=np.float32)).astype(np.float32)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, 2, w.scale, f32_device(bias), None)
    torch.cuda.synchronize()
    want = oracle.forward(x["q"], x["k"], x["v"], 2, w.scale, bias, None)
    assert max_abs(to_f64(o), want) <= 1e-5


def test_forward_is_bit_reproducible_and_leaves_inputs_alone():
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.swin_t_stage(2, shifted=True).with_N(64)
    x = synth.draw(w)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    q0, k0, v0 = q.clone(), k.clone(), v.clone()
    bias = fwa.fwa_bias_gather(f32_device(x["table"]), 7)
    mask = f32_device(x["mask"])
    a = fwa.fwa_forward(q, k, v, w.heads, w.scale, bias, mask)
    b = fwa.fwa_forward(q, k, v, w.heads, w.scale, bias, mask)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(q, q0) and torch.equal(k, k0) and torch.equal(v, v0)


def test_output_buffer_is_not_touched_outside_its_extent():
    """Guard bands around O keep their fill pattern (ragged last rows are not over-written)."""
    import torch
    import paper_2501_06480_amd as fwa
    N, L, C = 3, 49, 96
    w = synth.Workload("guard", N, L, C, 3, "bf16", 4200, 7)
    x = synth.draw(w)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    pad = 4096
    buf = torch.full((pad + N * L * C + pad,), 7.0, dtype=torch.bfloat16, device="cuda")
    out = buf[pad:pad + N * L * C].view(N, L, C)
    fwa.fwa_forward(q, k, v, 3, w.scale, out=out)
    torch.cuda.synchronize()
    assert (buf[:pad] == 7.0).all() and (buf[-pad:] == 7.0).all()


def test_empty_batch_is_a_no_op():
    import torch
    import paper_2501_06480_amd as fwa
    q = torch.empty((0, 49, 96), dtype=torch.bfloat16, device="cuda")
    assert fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1).shape == (0, 49, 96)


def test_full_size_stage1_every_window(oracle):
    """Config 2 at its full size, in the launch configuration the benchmark times: every window of
    the output against the oracle."""
    import torch
    w = synth.config2()
    x = synth.draw(w)
    o, _ = run_forward(w, x)
    torch.cuda.synchronize()
    got = to_f64(o)
    assert np.isfinite(got).all()
    want = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale)
    err = max_abs(got, want)
    print(f"config 2 full size, all {w.N} windows: max|ref|={np.abs(want).max():.3f} max-abs err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]
