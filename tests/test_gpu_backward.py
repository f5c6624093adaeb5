"""GPU parity of fwa_backward (and the bias scatter) against the fp64 oracle.

dQ, dK, dV are bf16 outputs (one final rounding) and dBias is fp32; all four
are held to the benchmark's bf16 bound of 1e-2 max-abs against the oracle.
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu


def run_backward(w, x, bias_np, mask_np, want_dbias=True):
    import torch
    import paper_2501_06480_amd as fwa
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    out = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias_np), f32_device(mask_np),
                           want_dbias=want_dbias)
    torch.cuda.synchronize()
    return out


def check_backward(oracle, w, bias_np, mask_np, label, want_dbias=True):
    x = synth.draw(w)
    dq, dk, dv, db = run_backward(w, x, bias_np, mask_np, want_dbias)
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias_np, mask_np)
    errs = {}
    for name, got, want in (("dq", dq, ref[0]), ("dk", dk, ref[1]), ("dv", dv, ref[2])):
        got = to_f64(got)
        assert np.isfinite(got).all(), name
        errs[name] = (check_bf16_output(got, want, f"{label} {name}"), float(np.abs(want).max()))
    if want_dbias:
        got = to_f64(db)
        assert np.isfinite(got).all()
        errs["dbias"] = (max_abs(got, ref[3]), float(np.abs(ref[3]).max()))
        assert errs["dbias"][0] <= TOL["bf16"], (label, "dbias", errs["dbias"][0])
    else:
        assert db is None
    print(label, " ".join(f"{k}: err={e:.2e} (max|ref|={m:.2f})" for k, (e, m) in errs.items()), flush=True)


@pytest.mark.parametrize("stage,n_small", [(1, 128), (3, 16)])
def test_config5_shapes_small(oracle, stage, n_small):
    w = synth.swin_t_stage(stage, shifted=True, backward=True).with_N(n_small)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k).astype(np.float32)
    check_backward(oracle, w, bias, x["mask"], w.name)


@pytest.mark.parametrize("stage", [2, 4])
def test_other_stages_small(oracle, stage):
    w = synth.swin_t_stage(stage, shifted=True, backward=True)
    w = w.with_N(max(w.nW, 1) * 2)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k).astype(np.float32)
    check_backward(oracle, w, bias, x["mask"], w.name)


@pytest.mark.parametrize("L", [1, 2, 5, 15, 16, 17, 31, 32, 33, 47, 48, 49, 50, 63, 64])
@pytest.mark.parametrize("use_bm", [False, True])
def test_window_lengths_up_to_64(oracle, L, use_bm):
    w = synth.Workload(f"bwd_L{L}", 7, L, 96, 3, "bf16", 5000 + L, 0, backward=True)
    bias = synth.normal((3, L, L), 11 + L, 0.5) if use_bm else None
    mask = None
    if use_bm:
        w = w.with_N(6)
        mask = np.where(synth.rng(3 + L).random((3, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, f"L={L} bm={use_bm}")


def test_without_dbias_and_many_windows_per_wave(oracle):
    """More windows than resident waves: every wave loops over several windows."""
    w = synth.Workload("bwd_loop", 3000, 49, 32, 1, "bf16", 5100, 7, backward=True)
    check_backward(oracle, w, None, None, "N=3000 heads=1", want_dbias=False)
    w = synth.Workload("bwd_loop_db", 1500, 49, 64, 2, "bf16", 5101, 7, backward=True)
    check_backward(oracle, w, None, None, "N=1500 heads=2 dbias", want_dbias=True)


@pytest.mark.parametrize("heads", [1, 2, 3, 4, 5, 6, 7, 9, 12])
def test_head_counts_reach_every_workgroup_shape(oracle, heads):
    """Up to 3 heads share one workgroup (whole rows); above that every head has its own
    workgroup and the head groups of a window are spread over neighbouring workgroups."""
    L, N = 49, 6
    w = synth.Workload(f"bwd_heads{heads}", N, L, 32 * heads, heads, "bf16", 7000 + heads, 0, backward=True)
    bias = synth.normal((heads, L, L), 23 + heads, 0.5)
    mask = np.where(synth.rng(29 + heads).random((3, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, f"heads={heads}")


def test_mask_period_too_long_for_the_cooperative_kernel(oracle):
    """nW larger than the number of workgroups the cooperative kernel walks in parallel:
    the single-wave kernel, which reads the mask tile per window, takes over."""
    L, heads, nW = 33, 3, 300
    w = synth.Workload("bwd_long_period", 2 * nW, L, 32 * heads, heads, "bf16", 7100, 0, backward=True)
    bias = synth.normal((heads, L, L), 31, 0.5)
    mask = np.where(synth.rng(37).random((nW, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, "nW=300")


@pytest.mark.parametrize("L", [65, 80, 81, 100, 127, 128, 129, 144, 145, 176, 177, 200, 225, 240, 250, 256])
@pytest.mark.parametrize("use_bm", [False, True])
def test_window_lengths_above_64(oracle, L, use_bm):
    """Every block count 5..16 of the two-pass kernel, ragged and full last blocks; three heads,
    more windows than the mask period."""
    w = synth.Workload(f"bwd_L{L}", 6, L, 96, 3, "bf16", 5200 + L, 0, backward=True)
    bias = synth.normal((3, L, L), 13 + L, 0.5) if use_bm else None
    mask = None
    if use_bm:
        mask = np.where(synth.rng(7 + L).random((3, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, f"L={L} bm={use_bm}", want_dbias=False)


@pytest.mark.parametrize("L,k,hw,heads,N", [(144, 12, 48, 4, 160), (256, 16, 64, 4, 144), (196, 14, 56, 3, 208)])
def test_large_windows_many_windows_per_workgroup(oracle, L, k, hw, heads, N):
    """Config-4 shapes with bias and the shift mask, more windows than resident workgroups."""
    w = synth.Workload(f"bwd_L{L}_h{heads}", N, L, 32 * heads, heads, "bf16", 5300 + L, k, hw, True, k // 2, True)
    assert N % w.nW == 0
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k).astype(np.float32)
    check_backward(oracle, w, bias, x["mask"], w.name, want_dbias=True)


@pytest.mark.parametrize("L", [65, 100, 144, 145, 177, 256])
@pytest.mark.parametrize("use_bm", [False, True])
def test_dbias_for_window_lengths_above_64(oracle, L, use_bm):
    """dBias of large windows comes from a kernel of its own (row statistics handed over through
    the workspace); 37 windows over at most 2 x 85 slots of partial sums, three heads."""
    w = synth.Workload(f"bwd_db_L{L}", 36, L, 96, 3, "bf16", 5400 + L, 0, backward=True)
    bias = synth.normal((3, L, L), 17 + L, 0.5) if use_bm else None
    mask = None
    if use_bm:
        mask = np.where(synth.rng(19 + L).random((4, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, f"L={L} bm={use_bm} dbias", want_dbias=True)


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("L", [64, 49, 33, 16, 7])
@pytest.mark.parametrize("use_bm", [False, True])
def test_wide_heads(oracle, d, L, use_bm):
    """Head widths of the paper's forward-backward kernel benchmark (L = 64, 4 heads)."""
    heads = 4
    w = synth.Workload(f"bwd_wide_d{d}_L{L}", 9, L, d * heads, heads, "bf16", 8100 + d + L, 0, backward=True)
    bias = mask = None
    if use_bm:
        bias = synth.normal((heads, L, L), 47 + L, 0.5)
        mask = np.where(synth.rng(53 + L + d).random((3, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, f"d={d} L={L} bm={use_bm}", want_dbias=False)


@pytest.mark.parametrize("d,L,N", [(64, 64, 300), (128, 49, 200), (256, 33, 140)])
def test_wide_heads_dbias_over_many_windows(oracle, d, L, N):
    """dBias for wide heads: workgroups walk several windows (N exceeds the slot count of 128)."""
    heads = 4
    w = synth.Workload(f"bwd_wide_db_d{d}_L{L}", N, L, d * heads, heads, "bf16", 8200 + d + L, 0, backward=True)
    bias = synth.normal((heads, L, L), 59 + L, 0.5)
    mask = np.where(synth.rng(71 + L + d).random((4, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    mask[:, np.arange(L), np.arange(L)] = 0.0
    check_backward(oracle, w, bias, mask, f"d={d} L={L} N={N} dbias", want_dbias=True)


@pytest.mark.parametrize("d", [32, 64, 128, 256])
@pytest.mark.parametrize("L", [64, 49, 17, 5])
@pytest.mark.parametrize("use_bm", [False, True])
def test_fp32_backward(oracle, d, L, use_bm):
    """fp32 data, fp32 arithmetic: the precision of the paper's own kernel benchmark; 1e-5 max-abs."""
    import torch
    import paper_2501_06480_amd as fwa
    heads = 2
    w = synth.Workload(f"bwd_f32_d{d}_L{L}", 5, L, d * heads, heads, "f32", 8300 + d + L, 0, backward=True)
    x = synth.draw(w)
    bias = mask = None
    if use_bm:
        bias = synth.normal((heads, L, L), 83 + L, 0.5)
        mask = np.where(synth.rng(89 + L + d).random((5, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    dq, dk, dv, _ = fwa.fwa_backward(q, k, v, g, heads, w.scale, f32_device(bias), f32_device(mask))
    torch.cuda.synchronize()
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], heads, w.scale, bias, mask)
    errs = {nme: max_abs(to_f64(got), want) for nme, got, want in (("dq", dq, ref[0]), ("dk", dk, ref[1]), ("dv", dv, ref[2]))}
    print(f"f32 d={d} L={L} bm={use_bm}: " + " ".join(f"{a}={b:.2e}" for a, b in errs.items()), flush=True)
    for nme, e in errs.items():
        assert e <= TOL["f32"], (nme, e)


def test_backward_is_bit_reproducible():
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.swin_t_stage(2, shifted=True, backward=True).with_N(256)
    x = synth.draw(w)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    bias = fwa.fwa_bias_gather(f32_device(x["table"]), 7)
    mask = f32_device(x["mask"])
    a = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, bias, mask, want_dbias=True)
    b = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, bias, mask, want_dbias=True)
    torch.cuda.synchronize()
    for s, t in zip(a[:3], b[:3]):
        assert torch.equal(s.view(torch.int16), t.view(torch.int16))
    assert torch.equal(a[3], b[3])


def test_guard_bands_around_outputs_stay_untouched():
    import torch
    from paper_2501_06480_amd import binding
    lib = binding.load_library()
    N, L, C, heads = 5, 49, 96, 3
    w = synth.Workload("guard", N, L, C, heads, "bf16", 5200, 7, backward=True)
    x = synth.draw(w)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    pad, n = 2048, N * L * C
    bufs = [torch.full((pad + n + pad,), 3.0, dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    outs = [b[pad:pad + n] for b in bufs]
    rc = lib.fwa_backward(q.data_ptr(), k.data_ptr(), v.data_ptr(), g.data_ptr(), outs[0].data_ptr(),
                          outs[1].data_ptr(), outs[2].data_ptr(), None, N, L, C, heads, w.scale, None, None, 0,
                          binding.FWA_BF16, None, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == 0
    for b in bufs:
        assert (b[:pad] == 3.0).all() and (b[-pad:] == 3.0).all()
        assert not (b[pad:pad + n] == 3.0).all()


def test_unsupported_backward_cases_are_rejected():
    import torch
    import paper_2501_06480_amd as fwa
    from paper_2501_06480_amd import binding
    q = torch.zeros((2, 144, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fwa.FwaError) as e:   # wide heads only for windows of up to 64 tokens
        fwa.fwa_backward(q, q.clone(), q.clone(), q.clone(), 4, 0.1)
    assert e.value.code == binding.FWA_ERR_UNSUPPORTED
    q = torch.zeros((2, 49, 96), dtype=torch.float32, device="cuda")
    with pytest.raises(fwa.FwaError) as e:   # no dBias in fp32
        fwa.fwa_backward(q, q.clone(), q.clone(), q.clone(), 3, 0.1, want_dbias=True)
    assert e.value.code == binding.FWA_ERR_UNSUPPORTED
    q = torch.zeros((2, 100, 96), dtype=torch.float32, device="cuda")
    with pytest.raises(fwa.FwaError) as e:   # fp32 backward only for windows of up to 64 tokens
        fwa.fwa_backward(q, q.clone(), q.clone(), q.clone(), 3, 0.1)
    assert e.value.code == binding.FWA_ERR_UNSUPPORTED


def test_empty_batch_zeroes_dbias():
    import torch
    import paper_2501_06480_amd as fwa
    q = torch.empty((0, 49, 96), dtype=torch.bfloat16, device="cuda")
    dq, dk, dv, db = fwa.fwa_backward(q, q.clone(), q.clone(), q.clone(), 3, 0.1, want_dbias=True)
    torch.cuda.synchronize()
    assert dq.shape == (0, 49, 96) and db.shape == (3, 49, 49) and (db == 0).all()


@pytest.mark.parametrize("k", [1, 2, 7, 12, 16])
def test_bias_scatter_matches_oracle(oracle, k):
    import torch
    import paper_2501_06480_amd as fwa
    heads, L = 3, k * k
    g = synth.normal((heads, L, L), 60 + k)
    got = fwa.fwa_bias_scatter(f32_device(g), k)
    again = fwa.fwa_bias_scatter(f32_device(g), k)
    torch.cuda.synchronize()
    want = oracle.bias_scatter(g, k)
    assert max_abs(to_f64(got), want) <= 1e-4 * max(1.0, np.abs(want).max())
    assert torch.equal(got, again)


def test_full_size_config5_stage1(oracle):
    """Config 5 stage 1 at full size (N = 8192) against the whole oracle backward."""
    w = synth.swin_t_stage(1, shifted=True, backward=True)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k).astype(np.float32)
    dq, dk, dv, db = run_backward(w, x, bias, x["mask"])
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias, x["mask"])
    for name, got, want in (("dq", dq, ref[0]), ("dk", dk, ref[1]), ("dv", dv, ref[2]), ("dbias", db, ref[3])):
        err = max_abs(to_f64(got), want)
        print(f"config 5 stage 1 full size {name}: err={err:.3e} max|ref|={np.abs(want).max():.2f}", flush=True)
        assert err <= TOL["bf16"], name
