"""ctypes binding of the C-ABI library declared in ``include/fwa.h``.

Argument marshalling only: every step of the attention path runs in the HIP
kernels of ``libfwa.so``.  torch supplies device memory and the stream.  There
is no CPU fallback: when the library has not been built, or a call is made
without a GPU tensor, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

FWA_F32 = 0
FWA_BF16 = 1
FWA_F16 = 2

FWA_OK = 0
FWA_ERR_NULL = 1
FWA_ERR_SHAPE = 2
FWA_ERR_UNSUPPORTED = 3
FWA_ERR_ALIGN = 4
FWA_ERR_WORKSPACE = 5
FWA_ERR_LAUNCH = 6
FWA_ERR_ALIAS = 7
FWA_NOALLOC_SCRATCH_BYTES = 16 * 1024 * 1024

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfwa.so")
_lib = None

EXPORTS = ("fwa_forward", "fwa_forward_strided", "fwa_forward_labels", "fwa_backward", "fwa_backward_strided",
           "fwa_backward_labels", "fwa_backward_noalloc",
           "fwa_backward_workspace_bytes", "fwa_bias_gather", "fwa_bias_scatter", "fwa_status_string")


class FwaError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {fwa_status_string(code)} (code {code})")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load ``libfwa.so`` (built in-tree by ``paper_2501_06480_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2501_06480_amd.build` "
            "(hipcc, gfx950). There is no fallback path.")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, ci, cf, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.fwa_forward.restype = ci
    lib.fwa_forward.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, cf, vp, vp, ci, ci, vp]
    lib.fwa_forward_strided.restype = ci
    lib.fwa_forward_strided.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, cf, i64, i64, vp, vp, ci, ci, vp]
    lib.fwa_forward_labels.restype = ci
    lib.fwa_forward_labels.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, cf, i64, i64, vp, ci, vp, cf, ci, ci, vp]
    lib.fwa_backward_labels.restype = ci
    lib.fwa_backward_labels.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, ci, ci, ci, cf, i64, i64, i64,
                                        vp, ci, vp, cf, ci, ci, vp, sz, vp]
    lib.fwa_backward.restype = ci
    lib.fwa_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, ci, ci, ci, cf, vp, vp, ci, ci,
                                 vp, sz, vp]
    lib.fwa_backward_noalloc.restype = ci
    lib.fwa_backward_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, ci, ci, ci, cf, vp, vp, ci, ci, vp]
    lib.fwa_backward_strided.restype = ci
    lib.fwa_backward_strided.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, ci, ci, ci, cf, i64, i64, i64,
                                         vp, vp, ci, ci, vp, sz, vp]
    lib.fwa_backward_workspace_bytes.restype = sz
    lib.fwa_backward_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci]
    lib.fwa_bias_gather.restype = ci
    lib.fwa_bias_gather.argtypes = [vp, vp, ci, ci, vp]
    lib.fwa_bias_scatter.restype = ci
    lib.fwa_bias_scatter.argtypes = [vp, vp, ci, ci, vp]
    lib.fwa_status_string.restype = ctypes.c_char_p
    lib.fwa_status_string.argtypes = [ci]
    _lib = lib
    return lib


def fwa_status_string(code: int) -> str:
    return load_library().fwa_status_string(int(code)).decode()


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return FWA_F32
    if t.dtype == torch.bfloat16:
        return FWA_BF16
    if t.dtype == torch.float16:
        return FWA_F16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev_ptr(t, name: str, like=None, f32: bool = False) -> Optional[int]:
    if t is None:
        return None
    if not getattr(t, "is_cuda", False):
        raise TypeError(f"{name} must be a GPU tensor (there is no CPU path)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if f32 and t.dtype != _torch().float32:
        raise TypeError(f"{name} must be float32")
    if like is not None and (t.shape != like.shape or t.dtype != like.dtype or t.device != like.device):
        raise ValueError(f"{name} must match q in shape, dtype and device")
    return t.data_ptr()


def _row_ptr(t, name: str, like=None):
    """(device pointer, row stride in elements) of an [N, L, C] tensor whose channels are
    contiguous and whose token rows are evenly spaced, e.g. a q/k/v view of a fused
    [N, L, 3, heads, d] projection output.  A contiguous tensor has row stride C."""
    if not getattr(t, "is_cuda", False):
        raise TypeError(f"{name} must be a GPU tensor (there is no CPU path)")
    if t.dim() != 3:
        raise ValueError(f"{name} must be [N, L, C]")
    if like is not None and (t.shape != like.shape or t.dtype != like.dtype or t.device != like.device):
        raise ValueError(f"{name} must match q in shape, dtype and device")
    N, L, C = t.shape
    if t.is_contiguous():
        return t.data_ptr(), C
    s0, s1, s2 = t.stride()
    if (C > 1 and s2 != 1) or (L > 1 and s1 < C) or (N > 1 and s0 != L * s1):
        raise ValueError(f"{name}: channels must be contiguous and token rows evenly spaced (stride {t.stride()})")
    return t.data_ptr(), (s1 if L > 1 else (s0 if N > 1 else C))


_torch_mod = None


def _torch():
    global _torch_mod
    if _torch_mod is None:
        import torch
        _torch_mod = torch
    return _torch_mod


def _stream_handle(stream, device) -> int:
    if stream is None:
        return _torch().cuda.current_stream(device).cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


class _alloc_on:
    """Allocate from torch's caching allocator as work of `stream`: a block handed out under
    another stream could be given to other work while the kernels enqueued on `stream` still use
    it.  `stream` = None (the current stream) needs nothing."""

    def __init__(self, stream, device):
        torch = _torch()
        if stream is None:
            self.ctx = None
        else:
            ts = stream if hasattr(stream, "cuda_stream") else torch.cuda.ExternalStream(int(stream), device=device)
            self.ctx = torch.cuda.stream(ts)

    def __enter__(self):
        if self.ctx is not None:
            self.ctx.__enter__()

    def __exit__(self, *exc):
        if self.ctx is not None:
            self.ctx.__exit__(*exc)


class _on_device:
    """Make `device` current for the duration of the call, only if it is not already."""

    def __init__(self, device):
        torch = _torch()
        self.ctx = None if device.index == torch.cuda.current_device() else torch.cuda.device(device)

    def __enter__(self):
        if self.ctx is not None:
            self.ctx.__enter__()

    def __exit__(self, *exc):
        if self.ctx is not None:
            self.ctx.__exit__(*exc)


def _bias_ptr(bias, heads: int, L: int):
    """(device pointer, dtype code) of a [heads, L, L] bias, fp32 or bf16."""
    if bias is None:
        return None, FWA_F32
    if tuple(bias.shape) != (heads, L, L):
        raise ValueError("bias must be [heads, L, L]")
    if bias.dtype == _torch().bfloat16:
        return _dev_ptr(bias, "bias"), FWA_BF16
    return _dev_ptr(bias, "bias", f32=True), FWA_F32


def _labels_ptr(labels, mask, L: int):
    """(device pointer, nW) of int32 region labels [nW, L]; they stand in for a dense mask."""
    if mask is not None:
        raise ValueError("give the mask either as a dense tensor or as labels, not both")
    if not getattr(labels, "is_cuda", False):
        raise TypeError("labels must be a GPU tensor (there is no CPU path)")
    if labels.dtype != _torch().int32 or labels.dim() != 2 or labels.shape[1] != L or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 tensor [nW, L]")
    return labels.data_ptr(), int(labels.shape[0])


def fwa_forward(q, k, v, heads: int, scale: float, bias=None, mask=None, out=None, stream=None, labels=None,
                mask_value: float = -100.0):
    """O = softmax(scale*QK^T + B + M) V (paper Algorithm 1).  Tensors are [N, L, C] on the GPU;
    q, k, v (and `out`) may be row-strided views, e.g. of a fused [N, L, 3, heads, d] tensor.
    The mask is a dense [nW, L, L] fp32 tensor, or int32 region `labels` [nW, L] from which the
    kernels form M[i][j] = 0 if labels agree else `mask_value`."""
    lib = _lib if _lib is not None else load_library()
    N, L, C = q.shape
    if out is None:
        with _alloc_on(stream, q.device):
            o = _torch().empty_like(q, memory_format=_torch().contiguous_format)
    else:
        o = out
    nW = 0 if mask is None else int(mask.shape[0])
    bp, bias_code = _bias_ptr(bias, heads, L)
    if mask is not None and tuple(mask.shape) != (nW, L, L):
        raise ValueError("mask must be [nW, L, L]")
    if bias_code == FWA_BF16 and mask is not None:
        raise ValueError("a bf16 bias goes with a mask given as labels (or with no mask), not with a dense mask")
    if labels is not None or bias_code == FWA_BF16:
        lp, nW = _labels_ptr(labels, mask, L) if labels is not None else (None, 0)
        (qp, ld), (kp, ldk), (vp, ldv), (op, ldo) = (_row_ptr(q, "q"), _row_ptr(k, "k", q), _row_ptr(v, "v", q),
                                                    _row_ptr(o, "out", q))
        if not ld == ldk == ldv:
            raise ValueError("q, k and v must share one row stride")
        with _on_device(q.device):
            rc = lib.fwa_forward_labels(qp, kp, vp, op, N, L, C, int(heads), float(scale), ld, ldo,
                                        bp, bias_code, lp, float(mask_value), nW, _dtype_code(q),
                                        _stream_handle(stream, q.device))
        if rc != FWA_OK:
            raise FwaError(rc, "fwa_forward_labels")
        return o
    tail = (bp, _dev_ptr(mask, "mask", f32=True), nW, _dtype_code(q), _stream_handle(stream, q.device))
    if q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and o.is_contiguous():
        args = (_dev_ptr(q, "q"), _dev_ptr(k, "k", q), _dev_ptr(v, "v", q), _dev_ptr(o, "out", q), N, L, C,
                int(heads), float(scale)) + tail
        fn, what = lib.fwa_forward, "fwa_forward"
    else:
        (qp, ld), (kp, ldk), (vp, ldv), (op, ldo) = (_row_ptr(q, "q"), _row_ptr(k, "k", q), _row_ptr(v, "v", q),
                                                    _row_ptr(o, "out", q))
        if not ld == ldk == ldv:
            raise ValueError("q, k and v must share one row stride")
        args = (qp, kp, vp, op, N, L, C, int(heads), float(scale), ld, ldo) + tail
        fn, what = lib.fwa_forward_strided, "fwa_forward_strided"
    with _on_device(q.device):
        rc = fn(*args)
    if rc != FWA_OK:
        raise FwaError(rc, what)
    return o


def fwa_backward_workspace_bytes(N: int, L: int, C: int, heads: int, dtype: int, want_dbias: bool) -> int:
    return int(load_library().fwa_backward_workspace_bytes(N, L, C, heads, dtype, int(bool(want_dbias))))


def fwa_backward(q, k, v, d_o, heads: int, scale: float, bias=None, mask=None, want_dbias: bool = False,
                 workspace=None, stream=None, out=None, labels=None, mask_value: float = -100.0):
    """(dQ, dK, dV, dBias) from Q, K, V, dO (paper Algorithm 2).  dBias is None unless asked for.
    q, k, v, d_o may be row-strided views; `out` = (dq, dk, dv) writes the gradients into given
    tensors, e.g. the three views of a fused [N, L, 3, heads, d] gradient buffer.  `labels` and
    `mask_value` give the mask as region labels, as in ``fwa_forward``."""
    import torch
    lib = load_library()
    N, L, C = q.shape
    with _alloc_on(stream, q.device):
        if out is None:
            dq, dk, dv = (torch.empty_like(q, memory_format=torch.contiguous_format) for _ in range(3))
        else:
            dq, dk, dv = out
        dbias = torch.empty((heads, L, L), dtype=torch.float32, device=q.device) if want_dbias else None
    nW = 0 if mask is None else int(mask.shape[0])
    bp, bias_code = _bias_ptr(bias, heads, L)
    if mask is not None and tuple(mask.shape) != (nW, L, L):
        raise ValueError("mask must be [nW, L, L]")
    if bias_code == FWA_BF16 and mask is not None:
        raise ValueError("a bf16 bias goes with a mask given as labels (or with no mask), not with a dense mask")
    need = fwa_backward_workspace_bytes(N, L, C, heads, _dtype_code(q), want_dbias)
    # needed for dBias, and above 64 tokens for the fp32 copy the library makes of a bf16 bias
    if workspace is None and need and (want_dbias or (bias_code == FWA_BF16 and L > 64)):
        with _alloc_on(stream, q.device):
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tail = (bp, _dev_ptr(mask, "mask", f32=True), nW, _dtype_code(q),
            None if workspace is None else workspace.data_ptr(), ws_bytes, _stream_handle(stream, q.device))
    tensors = (q, k, v, d_o, dq, dk, dv)
    if labels is not None or bias_code == FWA_BF16:
        lp, nW = _labels_ptr(labels, mask, L) if labels is not None else (None, 0)
        rows = [_row_ptr(t, nm, None if nm == "q" else q) for t, nm in zip(tensors, ("q", "k", "v", "d_o", "dq", "dk", "dv"))]
        if not rows[0][1] == rows[1][1] == rows[2][1]:
            raise ValueError("q, k and v must share one row stride")
        if not rows[4][1] == rows[5][1] == rows[6][1]:
            raise ValueError("dq, dk and dv must share one row stride")
        args = tuple(r[0] for r in rows) + (None if dbias is None else dbias.data_ptr(), N, L, C, int(heads),
                                            float(scale), rows[0][1], rows[3][1], rows[4][1],
                                            bp, bias_code, lp, float(mask_value), nW) + tail[3:]
        with _on_device(q.device):
            rc = lib.fwa_backward_labels(*args)
        if rc != FWA_OK:
            raise FwaError(rc, "fwa_backward_labels")
        return dq, dk, dv, dbias
    if all(t.is_contiguous() for t in tensors):
        ptrs = (_dev_ptr(q, "q"), _dev_ptr(k, "k", q), _dev_ptr(v, "v", q), _dev_ptr(d_o, "d_o", q),
                _dev_ptr(dq, "dq", q), _dev_ptr(dk, "dk", q), _dev_ptr(dv, "dv", q))
        args = ptrs + (None if dbias is None else dbias.data_ptr(), N, L, C, int(heads), float(scale)) + tail
        fn, what = lib.fwa_backward, "fwa_backward"
    else:
        rows = [_row_ptr(t, nm, None if nm == "q" else q) for t, nm in zip(tensors, ("q", "k", "v", "d_o", "dq", "dk", "dv"))]
        if not rows[0][1] == rows[1][1] == rows[2][1]:
            raise ValueError("q, k and v must share one row stride")
        if not rows[4][1] == rows[5][1] == rows[6][1]:
            raise ValueError("dq, dk and dv must share one row stride")
        args = tuple(r[0] for r in rows) + (None if dbias is None else dbias.data_ptr(), N, L, C, int(heads),
                                            float(scale), rows[0][1], rows[3][1], rows[4][1]) + tail
        fn, what = lib.fwa_backward_strided, "fwa_backward_strided"
    with _on_device(q.device):
        rc = fn(*args)
    if rc != FWA_OK:
        raise FwaError(rc, what)
    return dq, dk, dv, dbias


def fwa_backward_noalloc(q, k, v, d_o, heads: int, scale: float, out, dbias=None, bias=None, mask=None, stream=None):
    """``fwa_backward`` for callers that cannot allocate: the caller passes every output
    (`out` = (dq, dk, dv), contiguous; `dbias` = a [heads, L, L] fp32 tensor or None) and the
    library uses its own static scratch array as workspace.  Returns (dq, dk, dv, dbias)."""
    lib = load_library()
    N, L, C = q.shape
    dq, dk, dv = out
    nW = 0 if mask is None else int(mask.shape[0])
    if mask is not None and tuple(mask.shape) != (nW, L, L):
        raise ValueError("mask must be [nW, L, L]")
    if dbias is not None and tuple(dbias.shape) != (heads, L, L):
        raise ValueError("dbias must be [heads, L, L]")
    bp, bias_code = _bias_ptr(bias, heads, L)
    if bias_code != FWA_F32:
        raise TypeError("fwa_backward_noalloc takes an fp32 bias")
    args = (_dev_ptr(q, "q"), _dev_ptr(k, "k", q), _dev_ptr(v, "v", q), _dev_ptr(d_o, "d_o", q),
            _dev_ptr(dq, "dq", q), _dev_ptr(dk, "dk", q), _dev_ptr(dv, "dv", q), _dev_ptr(dbias, "dbias", f32=True),
            N, L, C, int(heads), float(scale), bp, _dev_ptr(mask, "mask", f32=True), nW, _dtype_code(q),
            _stream_handle(stream, q.device))
    with _on_device(q.device):
        rc = lib.fwa_backward_noalloc(*args)
    if rc != FWA_OK:
        raise FwaError(rc, "fwa_backward_noalloc")
    return dq, dk, dv, dbias


def fwa_bias_gather(table, k: int, stream=None):
    """[heads, (2k-1)^2] fp32 table -> [heads, k*k, k*k] fp32 bias, on the GPU."""
    import torch
    lib = load_library()
    heads = int(table.shape[0])
    if tuple(table.shape) != (heads, (2 * k - 1) ** 2):
        raise ValueError("table must be [heads, (2k-1)^2]")
    tp = _dev_ptr(table, "table", f32=True)
    bias = torch.empty((heads, k * k, k * k), dtype=torch.float32, device=table.device)
    with _on_device(table.device):
        rc = lib.fwa_bias_gather(tp, bias.data_ptr(), heads, int(k),
                                 _stream_handle(stream, table.device))
    if rc != FWA_OK:
        raise FwaError(rc, "fwa_bias_gather")
    return bias


def fwa_bias_scatter(dbias, k: int, stream=None):
    """[heads, k*k, k*k] fp32 bias gradient -> [heads, (2k-1)^2] table gradient."""
    import torch
    lib = load_library()
    heads = int(dbias.shape[0])
    if tuple(dbias.shape) != (heads, k * k, k * k):
        raise ValueError("dbias must be [heads, k*k, k*k]")
    dp = _dev_ptr(dbias, "dbias", f32=True)
    dtable = torch.empty((heads, (2 * k - 1) ** 2), dtype=torch.float32, device=dbias.device)
    with _on_device(dbias.device):
        rc = lib.fwa_bias_scatter(dp, dtable.data_ptr(), heads, int(k),
                                  _stream_handle(stream, dbias.device))
    if rc != FWA_OK:
        raise FwaError(rc, "fwa_bias_scatter")
    return dtable
