"""Host-side tests of the C ABI: the library loads, exports what the header declares,
and rejects bad arguments before touching the GPU (so these run without one)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2501_06480_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2501_06480_amd import build
        build.build(verbose=False)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fwa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fwa_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    from paper_2501_06480_amd import binding
    names = declared_functions()
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = set()
    for code in range(8):
        s = lib.fwa_status_string(code).decode()
        assert s and s != "unknown status code"
        seen.add(s)
    assert len(seen) == 8
    assert lib.fwa_status_string(99).decode() == "unknown status code"


P = 0x10000000  # a fake, 16-byte aligned, non-NULL "device pointer"; never dereferenced on error paths


def fwd(lib, q=P, k=P + 0x1000000, v=P + 0x2000000, o=P + 0x3000000, N=4, L=49, C=96, heads=3, scale=0.1, bias=None,
        mask=None, nW=0, dtype=1):
    return lib.fwa_forward(q, k, v, o, N, L, C, heads, scale, bias, mask, nW, dtype, None)


def bwd(lib, q=P, k=P + 0x1000000, v=P + 0x2000000, g=P + 0x3000000, dq=P + 0x4000000, dk=P + 0x5000000, dv=P + 0x6000000,
        dbias=None, N=4, L=49, C=96, heads=3, scale=0.1, bias=None, mask=None, nW=0, dtype=1, ws=None,
        ws_bytes=0):
    return lib.fwa_backward(q, k, v, g, dq, dk, dv, dbias, N, L, C, heads, scale, bias, mask, nW, dtype, ws,
                            ws_bytes, None)


def test_forward_rejects_bad_arguments(lib):
    from paper_2501_06480_amd import binding as b
    assert fwd(lib, N=-1) == b.FWA_ERR_SHAPE
    assert fwd(lib, L=0) == b.FWA_ERR_SHAPE
    assert fwd(lib, heads=0) == b.FWA_ERR_SHAPE
    assert fwd(lib, C=100, heads=3) == b.FWA_ERR_SHAPE
    assert fwd(lib, C=48, heads=3) == b.FWA_ERR_UNSUPPORTED       # head dim 16
    assert fwd(lib, C=288, heads=3) == b.FWA_ERR_UNSUPPORTED      # head dim 96
    assert fwd(lib, C=192, heads=3, dtype=0, L=65) == b.FWA_ERR_UNSUPPORTED   # head dim 64 beyond one tile, fp32
    assert fwd(lib, C=192, heads=3, L=65) == b.FWA_ERR_UNSUPPORTED      # head dim 64 beyond one tile
    assert fwd(lib, L=257) == b.FWA_ERR_UNSUPPORTED
    assert fwd(lib, dtype=2) == b.FWA_ERR_UNSUPPORTED            # half data at head width 32
    assert fwd(lib, dtype=3) == b.FWA_ERR_UNSUPPORTED
    assert fwd(lib, mask=P + 0x9000000, nW=0) == b.FWA_ERR_SHAPE
    assert fwd(lib, mask=P + 0x9000000, nW=3) == b.FWA_ERR_SHAPE     # 4 % 3 != 0
    assert fwd(lib, q=None) == b.FWA_ERR_NULL
    assert fwd(lib, o=None) == b.FWA_ERR_NULL
    assert fwd(lib, k=P + 8) == b.FWA_ERR_ALIGN
    assert fwd(lib, bias=P + 4) == b.FWA_ERR_ALIGN
    assert fwd(lib, o=P) == b.FWA_ERR_ALIAS
    assert fwd(lib, N=0, q=None, k=None, v=None, o=None) == b.FWA_OK   # empty batch: no-op


def test_backward_rejects_bad_arguments(lib):
    from paper_2501_06480_amd import binding as b
    assert bwd(lib, N=-1) == b.FWA_ERR_SHAPE
    assert bwd(lib, C=128, heads=2, L=65) == b.FWA_ERR_UNSUPPORTED    # head dim 64 beyond one tile
    assert bwd(lib, C=96, heads=2) == b.FWA_ERR_UNSUPPORTED      # head dim 48
    assert bwd(lib, L=300) == b.FWA_ERR_UNSUPPORTED
    assert bwd(lib, g=None) == b.FWA_ERR_NULL
    assert bwd(lib, dv=None) == b.FWA_ERR_NULL
    assert bwd(lib, dq=P + 2) == b.FWA_ERR_ALIGN
    assert bwd(lib, dq=P) == b.FWA_ERR_ALIAS
    assert bwd(lib, dk=P + 0x4000000) == b.FWA_ERR_ALIAS              # dk == dq
    assert bwd(lib, mask=P + 0x9000000, nW=8) == b.FWA_ERR_SHAPE
    need = lib.fwa_backward_workspace_bytes(4, 49, 96, 3, 1, 1)
    assert need >= 3 * 64 * 64 * 4
    assert bwd(lib, dbias=P + 0x7000000) == b.FWA_ERR_WORKSPACE
    assert bwd(lib, dbias=P + 0x7000000, ws=P + 0x8000000, ws_bytes=need - 1) == b.FWA_ERR_WORKSPACE
    assert lib.fwa_backward_workspace_bytes(4, 49, 96, 3, 1, 0) == 0
    assert lib.fwa_backward_workspace_bytes(4, 49, 100, 3, 1, 1) == 0
    assert lib.fwa_backward_workspace_bytes(0, 49, 96, 3, 1, 1) == 0
    assert bwd(lib, N=0) == b.FWA_OK


def test_bias_helpers_reject_bad_arguments(lib):
    from paper_2501_06480_amd import binding as b
    assert lib.fwa_bias_gather(P, P + 0x1000000, 0, 7, None) == b.FWA_ERR_SHAPE
    assert lib.fwa_bias_gather(P, P + 0x1000000, 3, 0, None) == b.FWA_ERR_SHAPE
    assert lib.fwa_bias_gather(P, P + 0x1000000, 3, 17, None) == b.FWA_ERR_UNSUPPORTED
    assert lib.fwa_bias_gather(None, P, 3, 7, None) == b.FWA_ERR_NULL
    assert lib.fwa_bias_gather(P, P + 4, 3, 7, None) == b.FWA_ERR_ALIGN
    assert lib.fwa_bias_gather(P, P, 3, 7, None) == b.FWA_ERR_ALIAS
    assert lib.fwa_bias_scatter(P, None, 3, 7, None) == b.FWA_ERR_NULL
    assert lib.fwa_bias_scatter(P, P + 0x1000000, 3, 20, None) == b.FWA_ERR_UNSUPPORTED


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2501_06480_amd as fwa
    q = torch.zeros((2, 49, 96), dtype=torch.bfloat16)
    with pytest.raises((TypeError, RuntimeError, AssertionError)):
        fwa.fwa_forward(q, q, q, 3, 0.1)


def test_strided_entry_points_check_their_strides(lib):
    from paper_2501_06480_amd import binding as b
    fwd = lambda ldq, ldo, dtype=1: lib.fwa_forward_strided(P, P + 0x1000000, P + 0x2000000, P + 0x3000000, 4, 49, 96, 3, 0.1,
                                                            ldq, ldo, None, None, 0, dtype, None)
    assert fwd(95, 96) == b.FWA_ERR_SHAPE            # rows would overlap
    assert fwd(288, 88) == b.FWA_ERR_SHAPE
    assert fwd(100, 96) == b.FWA_ERR_ALIGN           # bf16 rows must stay 16-byte aligned: multiples of 8
    assert fwd(98, 96, dtype=0) == b.FWA_ERR_ALIGN   # fp32: multiples of 4
    assert fwd(1 << 21, 96) == b.FWA_ERR_UNSUPPORTED
    bwd = lambda ldq, ldg, ldd: lib.fwa_backward_strided(P, P + 0x1000000, P + 0x2000000, P + 0x3000000, P + 0x4000000, P + 0x5000000,
                                                         P + 0x6000000, None, 4, 49, 96, 3, 0.1, ldq, ldg, ldd, None, None,
                                                         0, 1, None, 0, None)
    assert bwd(288, 90, 288) == b.FWA_ERR_SHAPE
    assert bwd(288, 96, 100) == b.FWA_ERR_ALIGN
    assert bwd(95, 96, 96) == b.FWA_ERR_SHAPE



def test_label_entry_points_check_their_arguments(lib):
    from paper_2501_06480_amd import binding as b
    fwd = lambda N=4, labels=P + 0x9000000, nW=2, ldq=96, bias=None, bias_dtype=0: lib.fwa_forward_labels(
        P, P + 0x1000000, P + 0x2000000, P + 0x3000000, N, 49, 96, 3, 0.1, ldq, 96, bias, bias_dtype, labels, -100.0, nW, 1, None)
    assert fwd(nW=0) == b.FWA_ERR_SHAPE
    assert fwd(nW=3) == b.FWA_ERR_SHAPE              # 4 % 3 != 0
    assert fwd(labels=P + 0x9000004) == b.FWA_ERR_ALIGN
    assert fwd(ldq=95) == b.FWA_ERR_SHAPE
    assert fwd(N=0, labels=None, nW=0) == b.FWA_OK   # empty batch, no mask: no-op
    assert fwd(bias=P + 0x7000000, bias_dtype=2) == b.FWA_ERR_UNSUPPORTED   # bias is fp32 or bf16
    assert fwd(bias=P + 0x7000002, bias_dtype=1) == b.FWA_ERR_ALIGN
    bwd = lambda labels=P + 0x9000000, nW=2, dbias=None, bias=None, bias_dtype=0, N=4, heads=3: lib.fwa_backward_labels(
        P, P + 0x1000000, P + 0x2000000, P + 0x3000000, P + 0x4000000, P + 0x5000000, P + 0x6000000, dbias, N, 49, 32 * heads, heads, 0.1,
        32 * heads, 32 * heads, 32 * heads, bias, bias_dtype, labels, -100.0, nW, 1, None, 0, None)
    assert bwd(nW=8) == b.FWA_ERR_SHAPE
    assert bwd(labels=P + 0x9000008) == b.FWA_ERR_ALIGN
    assert bwd(dbias=P + 0x7000000) == b.FWA_ERR_WORKSPACE
    assert bwd(bias=P + 0x7000000, bias_dtype=3) == b.FWA_ERR_UNSUPPORTED


def test_large_window_backward_needs_a_workspace_for_a_bf16_bias(lib):
    """Above 64 tokens the backward works on an fp32 copy of a bf16 bias, which lives in the workspace:
    the size query always leaves room for it, and a call that passes a bf16 bias without a workspace
    is turned away before anything is launched."""
    from paper_2501_06480_amd import binding as b
    L, heads = 144, 4
    room = (heads * L * L * 4 + 255) // 256 * 256
    assert lib.fwa_backward_workspace_bytes(16, L, 32 * heads, heads, 1, 0) == room
    assert lib.fwa_backward_workspace_bytes(16, L, 32 * heads, heads, 1, 1) > room
    assert lib.fwa_backward_workspace_bytes(16, 64, 32 * heads, heads, 1, 0) == 0
    bwd = lambda bias_dtype, ws=None, ws_bytes=0: lib.fwa_backward_labels(
        P, P + 0x1000000, P + 0x2000000, P + 0x3000000, P + 0x4000000, P + 0x5000000, P + 0x6000000, None, 16, L, 32 * heads, heads, 0.1,
        32 * heads, 32 * heads, 32 * heads, P + 0x7000000, bias_dtype, None, -100.0, 0, 1, ws, ws_bytes, None)
    assert bwd(1) == b.FWA_ERR_WORKSPACE
    assert bwd(1, P + 0x8000000, room - 1) == b.FWA_ERR_WORKSPACE


def test_overlapping_tensors_are_rejected_and_interleaved_views_are_not(lib):
    """An output may not share a byte with an input or another output: not only equal pointers but
    any overlap of the byte ranges is turned away, while the views of one fused [N, L, 3, heads, d]
    buffer (equal row strides, rows interleaved) pass."""
    from paper_2501_06480_amd import binding as b
    N, L, C, heads = 4, 49, 96, 3
    nbytes = N * L * C * 2
    assert fwd(lib, o=P + nbytes - 16) == b.FWA_ERR_ALIAS           # o starts inside q's last row
    assert fwd(lib, o=P + 0x1000000 - nbytes + 32) == b.FWA_ERR_ALIAS   # o's tail reaches into k
    assert bwd(lib, dq=P + 0x3000000 + 64) == b.FWA_ERR_ALIAS        # dq inside d_o
    assert bwd(lib, dv=P + 0x5000000 + nbytes - 16) == b.FWA_ERR_ALIAS   # dv starts in dk's last row
    assert bwd(lib, dbias=P + 0x4000000 + 1024, ws=P + 0x8000000, ws_bytes=1 << 30) == b.FWA_ERR_ALIAS  # dbias inside dq
    # fused buffers: q, k, v at base, base + C, base + 2C with row stride 3C, and the same for dq, dk, dv.
    # The call gets past the alias check and is stopped by the next one (dbias without a workspace).
    e = 2
    strided = lambda dq, dk, dv, ldd=3 * C: lib.fwa_backward_strided(
        P, P + C * e, P + 2 * C * e, P + 0x3000000, dq, dk, dv, P + 0x7000000, N, L, C, heads, 0.1, 3 * C, C, ldd,
        None, None, 0, 1, None, 0, None)
    G = P + 0x4000000
    assert strided(G, G + C * e, G + 2 * C * e) == b.FWA_ERR_WORKSPACE
    assert strided(G, G + C * e - 16, G + 2 * C * e) == b.FWA_ERR_ALIAS      # dk's rows start inside dq's rows
    assert strided(G, G + C * e, G + 3 * C * e - 16) == b.FWA_ERR_ALIAS      # dv's rows run into the next row of dq
    assert strided(P + 3 * C * e * 2, G + C * e, G + 2 * C * e) == b.FWA_ERR_ALIAS  # dq on top of q, two rows down
    # different strides with intersecting extents: rejected (conservative)
    assert strided(P + 16, G + C * e, G + 2 * C * e, ldd=4 * C) == b.FWA_ERR_ALIAS


def test_noalloc_backward_checks_its_arguments_and_its_limit(lib):
    from paper_2501_06480_amd import binding as b
    call = lambda N=4, L=49, C=96, heads=3, dbias=None, dq=P + 0x4000000, dtype=1: lib.fwa_backward_noalloc(
        P, P + 0x1000000, P + 0x2000000, P + 0x3000000, dq, P + 0x5000000, P + 0x6000000, dbias, N, L, C, heads, 0.1,
        None, None, 0, dtype, None)
    assert call(N=-1) == b.FWA_ERR_SHAPE
    assert call(dq=P) == b.FWA_ERR_ALIAS
    assert call(dq=P + 4) == b.FWA_ERR_ALIGN
    assert call(N=0) == b.FWA_OK
    assert call(dtype=0, dbias=P + 0x7000000) == b.FWA_ERR_UNSUPPORTED        # no dBias in fp32
    # the dBias workspace of large windows exceeds the static array: turned away, nothing launched
    assert b.FWA_NOALLOC_SCRATCH_BYTES == 16 * 1024 * 1024
    assert lib.fwa_backward_workspace_bytes(1024, 144, 128, 4, 1, 1) > b.FWA_NOALLOC_SCRATCH_BYTES
    assert call(N=64, L=144, C=128, heads=4, dbias=P + 0x7000000) == b.FWA_ERR_WORKSPACE


def test_header_and_binding_agree_on_the_scratch_limit():
    from paper_2501_06480_amd import binding as b
    text = open(os.path.join(ROOT, "include", "fwa.h")).read()
    m = re.search(r"#define FWA_NOALLOC_SCRATCH_BYTES \((\d+)u \* (\d+)u \* (\d+)u\)", text)
    assert m and int(m.group(1)) * int(m.group(2)) * int(m.group(3)) == b.FWA_NOALLOC_SCRATCH_BYTES
