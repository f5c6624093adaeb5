"""GPU parity of the label form of the shift mask (fwa_forward_labels / fwa_backward_labels).

Two checks per case: against the fp64 oracle fed the dense mask that the ORACLE writes out from
the same labels, to the bounds of the other parity tests; and bit for bit against this library's
own dense-mask call on the mask written out on the host, since both forms add the same fp32
values to the same scores.  The labels are random (more regions than the shift creates, any
integer values) and the mask value is small enough (-3) that masked pairs still carry weight, so
a wrong label, row or column shows up in the numbers instead of vanishing in exp(-100).
"""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import TOL, check_bf16_output, check_forward_arithmetic_bound, f32_device, max_abs, to_device, to_f64

pytestmark = pytest.mark.gpu

VALUE = -3.0


def random_labels(nW, L, seed, regions=5):
    lab = synth.rng(seed).integers(0, regions, size=(nW, L)).astype(np.int32)
    return (lab * 37 - 50).astype(np.int32)  # arbitrary integers, negative ones included


def dense_of(labels, value):
    same = labels[:, :, None] == labels[:, None, :]
    return np.where(same, np.float32(0.0), np.float32(value)).astype(np.float32)


def workload(name, N, L, C, heads, dtype, seed, backward=False):
    return synth.Workload(name, N, L, C, heads, dtype, seed, 0, backward=backward)


def check_forward(oracle, w, nW, use_bias, seed, value=VALUE):
    import torch
    import paper_2501_06480_amd as fwa
    x = synth.draw(w)
    labels = random_labels(nW, w.L, seed)
    bias = synth.normal((w.heads, w.L, w.L), seed + 1, 0.5) if use_bias else None
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    lab_d = torch.from_numpy(labels).cuda()
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias), labels=lab_d, mask_value=value)
    o_dense = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias), f32_device(dense_of(labels, value)))
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16 if w.dtype == "bf16" else torch.int32),
                       o_dense.view(torch.int16 if w.dtype == "bf16" else torch.int32)), w.name
    ref = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias, oracle.mask_from_labels(labels, value))
    got = to_f64(o)
    assert np.isfinite(got).all()
    err = max_abs(got, ref)
    print(f"{w.name}: labels nW={nW} bias={use_bias} err={err:.2e}", flush=True)
    if w.dtype == "bf16" and err > TOL["bf16"] and got.size > 4_000_000:
        # among millions of outputs a few of size 2..4 (half a bf16 ulp: 0.0078) also meet an unlucky rounding
        # of their probabilities and pass the flat bound by a little: such a call is held to the element-wise
        # bound of the arithmetic, and to twice the flat one
        spread = oracle.forward(x["q"], x["k"], np.abs(x["v"]), w.heads, w.scale, bias, oracle.mask_from_labels(labels, value))
        check_forward_arithmetic_bound(got, ref, spread, w.name)
        assert err <= 2 * TOL["bf16"], (w.name, err)
        return
    assert err <= TOL[w.dtype], (w.name, err)


def check_backward(oracle, w, nW, use_bias, seed, want_dbias, value=VALUE, bitwise=True):
    import torch
    import paper_2501_06480_amd as fwa
    x = synth.draw(w)
    labels = random_labels(nW, w.L, seed)
    bias = synth.normal((w.heads, w.L, w.L), seed + 1, 0.5) if use_bias else None
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    lab_d = torch.from_numpy(labels).cuda()
    got = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias), want_dbias=want_dbias, labels=lab_d,
                           mask_value=value)
    dense = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias), f32_device(dense_of(labels, value)),
                             want_dbias=want_dbias)
    torch.cuda.synchronize()
    bits = torch.int16 if w.dtype == "bf16" else torch.int32
    for name, a, b in zip(("dq", "dk", "dv"), got[:3], dense[:3]):
        if bitwise:
            assert torch.equal(a.view(bits), b.view(bits)), (w.name, name)
        else:  # another kernel takes the dense form: the same numbers up to a rounding of the output
            assert max_abs(to_f64(a), to_f64(b)) <= 2.0 ** -7 * max(1.0, float(b.float().abs().max())), (w.name, name)
    if want_dbias:
        if bitwise:
            assert torch.equal(got[3].view(torch.int32), dense[3].view(torch.int32)), (w.name, "dbias")
        else:
            assert max_abs(to_f64(got[3]), to_f64(dense[3])) <= 1e-3 * max(1.0, float(dense[3].abs().max())), (w.name, "dbias")
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], w.heads, w.scale, bias,
                          oracle.mask_from_labels(labels, value), want_dbias=want_dbias)
    errs = {}
    for name, t, want in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
        a = to_f64(t)
        assert np.isfinite(a).all(), name
        if w.dtype == "bf16":
            errs[name] = check_bf16_output(a, want, f"{w.name} {name}")
        else:
            errs[name] = max_abs(a, want)
            assert errs[name] <= TOL["f32"], (w.name, name, errs[name])
    if want_dbias:
        errs["dbias"] = max_abs(to_f64(got[3]), ref[3])
        assert errs["dbias"] <= TOL["bf16"], (w.name, errs["dbias"])
    print(f"{w.name}: labels nW={nW} bias={use_bias} " + " ".join(f"{k}={e:.2e}" for k, e in errs.items()), flush=True)


# name, N, L, C, heads, nW: one case per forward kernel of the bf16 path with head width 32
FWD_BF16 = [
    ("persistent_s1", 256, 49, 96, 3, 64),      # walk over windows with the term in registers
    ("persistent_s2", 128, 49, 192, 6, 16),
    ("persistent_four_heads", 1280, 49, 128, 4, 16),   # all four heads in one workgroup, one wave each
    ("staged_one_window_each", 6, 49, 96, 3, 3),  # too few windows for the walk
    ("staged_four_waves_per_head", 8, 49, 768, 24, 1),
    ("direct_five_heads", 12, 49, 160, 5, 4),
    ("ragged_L37", 10, 37, 64, 2, 5),
    ("tiny_L5", 9, 5, 32, 1, 3),
    ("rowpersist_L144", 64, 144, 96, 3, 4),
    ("rowpersist_L256_two_parts", 16, 256, 64, 2, 4),
    ("rowblock_L100", 3, 100, 64, 2, 3),        # fewer windows than the walk needs
    ("rowblock_L201", 2, 201, 96, 3, 1),
]


@pytest.mark.parametrize("name,N,L,C,heads,nW", FWD_BF16, ids=[c[0] for c in FWD_BF16])
@pytest.mark.parametrize("use_bias", [True, False])
def test_forward_bf16(oracle, name, N, L, C, heads, nW, use_bias):
    check_forward(oracle, workload("lab_" + name, N, L, C, heads, "bf16", 7100 + L), nW, use_bias, 7200 + L)


FWD_OTHER = [
    ("f32_tile_L49", 12, 49, 96, 3, "f32", 4),
    ("f32_tile_L64_d64", 8, 64, 128, 2, "f32", 2),
    ("f32_L144", 4, 144, 64, 2, "f32", 2),
    ("f32_L200", 2, 200, 32, 1, "f32", 2),
    ("wide_d64", 12, 64, 256, 4, "bf16", 4),
    ("wide_d128_L49", 6, 49, 256, 2, "bf16", 3),
    ("wide_d256", 4, 64, 512, 2, "bf16", 2),
]


@pytest.mark.parametrize("name,N,L,C,heads,dtype,nW", FWD_OTHER, ids=[c[0] for c in FWD_OTHER])
def test_forward_fp32_and_wide_heads(oracle, name, N, L, C, heads, dtype, nW):
    check_forward(oracle, workload("lab_" + name, N, L, C, heads, dtype, 7300 + L), nW, True, 7400 + L)


# name, N, L, C, heads, dtype, nW, dbias
BWD = [
    ("coop_s1", 256, 49, 96, 3, "bf16", 64, True),
    ("coop_s3", 32, 49, 384, 12, "bf16", 4, True),
    ("coop_no_dbias", 128, 49, 96, 3, "bf16", 16, False),
    # a mask period too long for the cooperative kernel: labels keep it (per-window masks), the dense form
    # goes to the one-wave kernel
    ("period_beyond_the_slots", 64, 49, 768, 24, "bf16", 64, True),
    ("period_beyond_the_slots_3_heads", 1024, 49, 96, 3, "bf16", 512, True),
    ("period_beyond_the_slots_L25", 1536, 25, 64, 2, "bf16", 768, False),
    ("ragged_L23", 12, 23, 64, 2, "bf16", 4, True),
    ("large_L144", 16, 144, 96, 3, "bf16", 4, True),
    ("large_L144_no_dbias", 8, 144, 64, 2, "bf16", 2, False),
    ("large_L256", 8, 256, 64, 2, "bf16", 4, True),
    ("large_L77", 6, 77, 32, 1, "bf16", 3, True),
    ("wide_d64", 12, 64, 256, 4, "bf16", 4, True),
    ("wide_d128_L49", 6, 49, 256, 2, "bf16", 3, True),
    ("f32_L49", 12, 49, 96, 3, "f32", 4, False),
    ("f32_L64_d64", 6, 64, 128, 2, "f32", 3, False),
]


@pytest.mark.parametrize("name,N,L,C,heads,dtype,nW,dbias", BWD, ids=[c[0] for c in BWD])
@pytest.mark.parametrize("use_bias", [True, False])
def test_backward(oracle, name, N, L, C, heads, dtype, nW, dbias, use_bias):
    check_backward(oracle, workload("lab_" + name, N, L, C, heads, dtype, 7500 + L, backward=True), nW, use_bias,
                   7600 + L, dbias, bitwise=not name.startswith("period_beyond"))


def test_swin_labels_reproduce_the_shift_mask_results(oracle):
    """The labels of the shifted Swin-T stage-1 map with the usual -100, against the dense shift mask."""
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.swin_t_stage(1, shifted=True, backward=True).with_N(128)
    x = synth.draw(w)
    bias = oracle.bias_gather(x["table"], w.k).astype(np.float32)
    q, k, v, g = (to_device(x, w, n) for n in ("q", "k", "v", "d_o"))
    lab = torch.from_numpy(x["labels"]).cuda()
    o = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias), labels=lab)
    o_dense = fwa.fwa_forward(q, k, v, w.heads, w.scale, f32_device(bias), f32_device(x["mask"]))
    assert torch.equal(o.view(torch.int16), o_dense.view(torch.int16))
    ref = oracle.forward(x["q"], x["k"], x["v"], w.heads, w.scale, bias, oracle.mask_from_labels(x["labels"]))
    assert max_abs(to_f64(o), ref) <= TOL["bf16"]
    got = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias), want_dbias=True, labels=lab)
    dense = fwa.fwa_backward(q, k, v, g, w.heads, w.scale, f32_device(bias), f32_device(x["mask"]), want_dbias=True)
    for a, b in zip(got, dense):
        assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                           b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))


def test_equal_labels_are_no_mask_and_strided_views_work(oracle):
    """One region per window adds zero everywhere: the result is that of the call without a mask.
    And the label entry points take the row-strided views of a fused [N, L, 3, heads, d] tensor."""
    import torch
    import paper_2501_06480_amd as fwa
    w = workload("lab_equal", 24, 49, 96, 3, "bf16", 7700)
    x = synth.draw(w)
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    lab = torch.full((4, 49), 9, dtype=torch.int32, device="cuda")
    a = fwa.fwa_forward(q, k, v, 3, w.scale, labels=lab)
    b = fwa.fwa_forward(q, k, v, 3, w.scale)
    assert max_abs(to_f64(a), to_f64(b)) <= 2.0 ** -8 * 4  # another kernel and exponent folding: a bf16 ulp or so
    qkv = torch.stack((q, k, v), dim=2).contiguous()       # [N, L, 3, C]
    labels = torch.from_numpy(random_labels(4, 49, 7701)).cuda()
    s = fwa.fwa_forward(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], 3, w.scale, labels=labels, mask_value=VALUE)
    c = fwa.fwa_forward(q, k, v, 3, w.scale, labels=labels, mask_value=VALUE)
    assert torch.equal(s.view(torch.int16), c.view(torch.int16))


def test_label_arguments_are_checked():
    import torch
    import paper_2501_06480_amd as fwa
    q = torch.zeros((6, 49, 96), dtype=torch.bfloat16, device="cuda")
    lab = torch.zeros((4, 49), dtype=torch.int32, device="cuda")
    with pytest.raises(fwa.FwaError) as e:
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1, labels=lab)   # 6 % 4 != 0
    assert e.value.code == 2
    with pytest.raises(ValueError):
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1, labels=lab[:, :48].contiguous())
    with pytest.raises(ValueError):
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1, labels=lab.long())
    with pytest.raises(ValueError):
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1, mask=torch.zeros((3, 49, 49), device="cuda"),
                        labels=lab[:3].contiguous())


# ---------------------------------------------------------------------------------- bf16 bias
def bf16_exact(a):
    """fp32 array whose values are exactly representable in bf16, and the same as a bf16 device tensor."""
    import torch
    vals, bits = synth.bf16_round(a.astype(np.float32))
    return vals, torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


BF16_BIAS = [
    # name, N, L, C, heads, dtype, nW (0 = no mask), backward, dbias
    ("fwd_persistent_s1", 256, 49, 96, 3, "bf16", 64, False, False),
    ("fwd_one_wave_per_head_s3", 512, 49, 384, 12, "bf16", 4, False, False),
    ("fwd_staged_few_windows", 6, 49, 96, 3, "bf16", 3, False, False),
    ("fwd_direct_five_heads", 12, 49, 160, 5, "bf16", 4, False, False),
    ("fwd_odd_heads_odd_L_no_mask", 9, 37, 96, 3, "bf16", 0, False, False),
    ("fwd_rowpersist_L144", 64, 144, 96, 3, "bf16", 4, False, False),
    ("fwd_rowblock_L201", 2, 201, 96, 3, "bf16", 1, False, False),
    ("fwd_wide_d64", 12, 64, 256, 4, "bf16", 4, False, False),
    ("fwd_f32_tile_L49", 12, 49, 96, 3, "f32", 4, False, False),
    ("fwd_f32_L145", 4, 145, 96, 3, "f32", 2, False, False),
    ("bwd_coop_s1", 256, 49, 96, 3, "bf16", 64, True, True),
    ("bwd_coop_s3", 32, 49, 384, 12, "bf16", 4, True, True),
    ("bwd_large_L143_odd", 12, 143, 96, 3, "bf16", 4, True, True),
    ("bwd_large_L256", 8, 256, 64, 2, "bf16", 4, True, True),
    ("bwd_large_L81_no_mask", 6, 81, 96, 3, "bf16", 0, True, False),
    ("bwd_wide_d128_L49", 6, 49, 384, 3, "bf16", 3, True, True),
    ("bwd_f32_L49", 12, 49, 96, 3, "f32", 4, True, False),
]


@pytest.mark.parametrize("name,N,L,C,heads,dtype,nW,backward,dbias", BF16_BIAS, ids=[c[0] for c in BF16_BIAS])
def test_bf16_bias(oracle, name, N, L, C, heads, dtype, nW, backward, dbias):
    """A bf16 bias gives the bits of the fp32 call on the same values, and matches the oracle."""
    import torch
    import paper_2501_06480_amd as fwa
    w = workload("b16_" + name, N, L, C, heads, dtype, 7800 + L, backward=backward)
    x = synth.draw(w)
    bias, bias_dev = bf16_exact(synth.normal((heads, L, L), 7900 + L, 0.5))
    labels = random_labels(nW, L, 7950 + L) if nW else None
    kw = {"labels": torch.from_numpy(labels).cuda(), "mask_value": VALUE} if nW else {}
    mask64 = oracle.mask_from_labels(labels, VALUE) if nW else None
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    bits = torch.int16 if dtype == "bf16" else torch.int32
    if not backward:
        o = fwa.fwa_forward(q, k, v, heads, w.scale, bias_dev, **kw)
        o32 = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), **kw)
        torch.cuda.synchronize()
        assert torch.equal(o.view(bits), o32.view(bits)), name
        ref = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias, mask64)
        err = max_abs(to_f64(o), ref)
        print(f"{w.name}: bf16 bias, err={err:.2e}", flush=True)
        assert err <= TOL[dtype], (name, err)
        return
    g = to_device(x, w, "d_o")
    got = fwa.fwa_backward(q, k, v, g, heads, w.scale, bias_dev, want_dbias=dbias, **kw)
    got32 = fwa.fwa_backward(q, k, v, g, heads, w.scale, f32_device(bias), want_dbias=dbias, **kw)
    torch.cuda.synchronize()
    for nm, a, b in zip(("dq", "dk", "dv"), got[:3], got32[:3]):
        assert torch.equal(a.view(bits), b.view(bits)), (name, nm)
    if dbias:
        assert torch.equal(got[3].view(torch.int32), got32[3].view(torch.int32)), (name, "dbias")
    ref = oracle.backward(x["q"], x["k"], x["v"], x["d_o"], heads, w.scale, bias, mask64, want_dbias=dbias)
    for nm, t, want in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
        if dtype == "bf16":
            check_bf16_output(to_f64(t), want, f"{w.name} {nm}")
        else:
            assert max_abs(to_f64(t), want) <= TOL["f32"], (name, nm)
    if dbias:
        assert max_abs(to_f64(got[3]), ref[3]) <= TOL["bf16"]


def test_bf16_bias_argument_rules():
    import torch
    import paper_2501_06480_amd as fwa
    q = torch.zeros((4, 49, 96), dtype=torch.bfloat16, device="cuda")
    bias = torch.zeros((3, 49, 49), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):   # a dense mask goes with an fp32 bias
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1, bias, torch.zeros((2, 49, 49), device="cuda"))
    with pytest.raises(ValueError):
        fwa.fwa_forward(q, q.clone(), q.clone(), 3, 0.1, bias[:2])


# Mask periods that no workgroup stride over the windows can be a multiple of (more windows per image
# than the chip holds workgroups, as on the token maps of detection and segmentation inputs).  With
# the mask as labels the persistent kernels keep only the bias in registers and form each window's
# mask from its labels, so the arithmetic differs in rounding order from the dense-mask call, which
# takes another kernel: both are held to the oracle, not to each other bit for bit.
# name, N, L, C, heads, nW
LONG_PERIOD_FWD = [
    ("all_heads_3", 1024, 49, 96, 3, 512),       # one workgroup per window position, three heads
    ("all_heads_2_L25", 1024, 25, 64, 2, 1024),
    ("all_heads_4_L64", 768, 64, 128, 4, 384),
    ("four_heads_many_windows", 2048, 49, 128, 4, 1024),   # beyond the small calls: one wave per head, two windows in flight
    ("wave_per_head_6", 1024, 49, 192, 6, 512),  # two heads per workgroup, one wave each
    ("wave_per_head_12", 1024, 49, 384, 12, 512),
    ("ragged_L37_8_heads", 1536, 37, 256, 8, 768),
    ("rows_L144", 512, 144, 128, 4, 256),
    ("rows_L256_two_parts", 256, 256, 64, 2, 128),
    ("rows_L100_3_heads", 768, 100, 96, 3, 384),
]


@pytest.mark.parametrize("name,N,L,C,heads,nW", LONG_PERIOD_FWD, ids=[c[0] for c in LONG_PERIOD_FWD])
@pytest.mark.parametrize("use_bias", [True, False])
def test_forward_long_mask_periods(oracle, name, N, L, C, heads, nW, use_bias):
    import torch
    import paper_2501_06480_amd as fwa
    w = workload("longp_" + name, N, L, C, heads, "bf16", 7700 + L + heads)
    x = synth.draw(w)
    labels = random_labels(nW, L, 7800 + L + heads)
    bias = synth.normal((heads, L, L), 7900 + L, 0.5) if use_bias else None
    q, k, v = (to_device(x, w, n) for n in ("q", "k", "v"))
    o = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), labels=torch.from_numpy(labels).cuda(), mask_value=VALUE)
    o_dense = fwa.fwa_forward(q, k, v, heads, w.scale, f32_device(bias), f32_device(dense_of(labels, VALUE)))
    torch.cuda.synchronize()
    ref = oracle.forward(x["q"], x["k"], x["v"], heads, w.scale, bias, oracle.mask_from_labels(labels, VALUE))
    got = to_f64(o)
    assert np.isfinite(got).all()
    err, err_dense = max_abs(got, ref), max_abs(to_f64(o_dense), ref)
    # the two calls differ by a rounding of the additive term: at most one bf16 step of the output apart
    apart = max_abs(got, to_f64(o_dense))
    print(f"{w.name}: nW={nW} bias={use_bias} err={err:.2e} (dense-mask call {err_dense:.2e}, apart {apart:.2e})", flush=True)
    flat = TOL["bf16"]
    if max(err, err_dense) > flat and got.size > 4_000_000:   # see check_forward: the tail of millions of outputs
        spread = oracle.forward(x["q"], x["k"], np.abs(x["v"]), heads, w.scale, bias, oracle.mask_from_labels(labels, VALUE))
        check_forward_arithmetic_bound(got, ref, spread, w.name)
        check_forward_arithmetic_bound(to_f64(o_dense), ref, spread, w.name + " dense")
        flat *= 2
    assert err <= flat and err_dense <= flat, (w.name, err, err_dense)
    assert apart <= 2.0 ** -7 * max(1.0, np.abs(ref).max()), (w.name, apart)
