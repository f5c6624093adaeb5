"""fp64 CPU oracle for window attention -- TEST INFRASTRUCTURE, not the product.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It wraps ``fwa_oracle.c`` (plain C,
double precision, loops in the order of the paper's equations 2-4 and of
Algorithm 2) through ctypes.  It shares no code with the GPU library and
never imports it.

``build()`` compiles the C file with gcc; ``load()`` builds on demand.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fwa_oracle.c")
_LIB = os.path.join(_HERE, "libfwa_oracle.so")
_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, strict IEEE: no fast-math)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", out, src, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def _f64(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_dp)


class Oracle:
    """The oracle's entry points bound to one compiled library.

    The module-level functions use the in-tree build; the mutation test binds
    deliberately broken builds to check that the pins notice.
    """

    def __init__(self, lib_path: str):
        lib = ctypes.CDLL(lib_path)
        lib.fwa_oracle_forward.restype = ctypes.c_int
        lib.fwa_oracle_forward.argtypes = [
            _dp, _dp, _dp, _dp, _dp, ctypes.c_long, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_double, _dp, _dp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        lib.fwa_oracle_backward.restype = ctypes.c_int
        lib.fwa_oracle_backward.argtypes = [
            _dp, _dp, _dp, _dp, _dp, _dp, _dp, _dp, ctypes.c_long, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_double, _dp, _dp, ctypes.c_int, ctypes.c_int,
            ctypes.POINTER(ctypes.c_int)]
        lib.fwa_oracle_bias_gather.restype = ctypes.c_int
        lib.fwa_oracle_bias_gather.argtypes = [_dp, _dp, ctypes.c_int, ctypes.c_int]
        lib.fwa_oracle_bias_scatter.restype = ctypes.c_int
        lib.fwa_oracle_bias_scatter.argtypes = [_dp, _dp, ctypes.c_int, ctypes.c_int]
        lib.fwa_oracle_mask_from_labels.restype = ctypes.c_int
        lib.fwa_oracle_mask_from_labels.argtypes = [ctypes.POINTER(ctypes.c_int), _dp, ctypes.c_int, ctypes.c_int,
                                                    ctypes.c_double]
        self._lib = lib
        self.threads_used = 0

    @staticmethod
    def _mask(mask, L):
        mask = _f64(mask)
        if mask is None:
            return None, 0
        nW = mask.shape[0]
        if mask.shape != (nW, L, L):
            raise ValueError("mask must be [nW, L, L]")
        return mask, nW

    def forward(self, q, k, v, heads, scale, bias=None, mask=None, return_p=False, threads=0):
        """O = softmax(scale*Q K^T + B + M) V per window and head (paper eq. 2-4).

        q, k, v: [N, L, C]; bias: None or [heads, L, L]; mask: None or
        [nW, L, L] (window n uses mask[n % nW]).  Returns O [N, L, C] float64,
        and with ``return_p`` also P [N, heads, L, L].
        """
        q = _f64(q)
        N, L, C = q.shape
        k = _f64(k, q.shape)
        v = _f64(v, q.shape)
        bias = _f64(bias, (heads, L, L))
        mask, nW = self._mask(mask, L)
        o = np.empty_like(q)
        p = np.empty((N, heads, L, L), dtype=np.float64) if return_p else None
        used = ctypes.c_int(0)
        rc = self._lib.fwa_oracle_forward(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(p), N, L, C, heads,
                                          float(scale), _ptr(bias), _ptr(mask), nW, int(threads),
                                          ctypes.byref(used))
        if rc != 0:
            raise ValueError(f"fwa_oracle_forward failed with code {rc}")
        self.threads_used = used.value
        return (o, p) if return_p else o

    def backward(self, q, k, v, d_o, heads, scale, bias=None, mask=None, want_dbias=True, threads=0):
        """Gradients w.r.t. q, k, v and the bias (paper Algorithm 2).

        Returns (dq, dk, dv, dbias); dbias is [heads, L, L] summed over all N
        windows, or None when ``want_dbias`` is false.
        """
        q = _f64(q)
        N, L, C = q.shape
        k = _f64(k, q.shape)
        v = _f64(v, q.shape)
        d_o = _f64(d_o, q.shape)
        bias = _f64(bias, (heads, L, L))
        mask, nW = self._mask(mask, L)
        dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
        dbias = np.empty((heads, L, L), dtype=np.float64) if want_dbias else None
        used = ctypes.c_int(0)
        rc = self._lib.fwa_oracle_backward(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(dq), _ptr(dk),
                                           _ptr(dv), _ptr(dbias), N, L, C, heads, float(scale),
                                           _ptr(bias), _ptr(mask), nW, int(threads), ctypes.byref(used))
        if rc != 0:
            raise ValueError(f"fwa_oracle_backward failed with code {rc}")
        self.threads_used = used.value
        return dq, dk, dv, dbias

    def bias_gather(self, table, k):
        """[heads, (2k-1)^2] relative-position table -> [heads, k*k, k*k] bias."""
        table = _f64(table)
        heads = table.shape[0]
        if table.shape != (heads, (2 * k - 1) ** 2):
            raise ValueError("table must be [heads, (2k-1)^2]")
        bias = np.empty((heads, k * k, k * k), dtype=np.float64)
        rc = self._lib.fwa_oracle_bias_gather(_ptr(table), _ptr(bias), heads, k)
        if rc != 0:
            raise ValueError(f"fwa_oracle_bias_gather failed with code {rc}")
        return bias

    def bias_scatter(self, dbias, k):
        """Adjoint of ``bias_gather``: [heads, k*k, k*k] -> [heads, (2k-1)^2]."""
        dbias = _f64(dbias)
        heads = dbias.shape[0]
        if dbias.shape != (heads, k * k, k * k):
            raise ValueError("dbias must be [heads, k*k, k*k]")
        dtable = np.empty((heads, (2 * k - 1) ** 2), dtype=np.float64)
        rc = self._lib.fwa_oracle_bias_scatter(_ptr(dbias), _ptr(dtable), heads, k)
        if rc != 0:
            raise ValueError(f"fwa_oracle_bias_scatter failed with code {rc}")
        return dtable


    def mask_from_labels(self, labels, value=-100.0):
        """[nW, L] integer region labels -> [nW, L, L] additive mask: 0 between tokens of
        equal label, ``value`` elsewhere.  Feed the result to ``forward`` / ``backward``."""
        labels = np.ascontiguousarray(labels, dtype=np.intc)
        if labels.ndim != 2:
            raise ValueError("labels must be [nW, L]")
        nW, L = labels.shape
        mask = np.empty((nW, L, L), dtype=np.float64)
        rc = self._lib.fwa_oracle_mask_from_labels(labels.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), _ptr(mask),
                                                   nW, L, float(value))
        if rc != 0:
            raise ValueError(f"fwa_oracle_mask_from_labels failed with code {rc}")
        return mask


_default = None


def load() -> Oracle:
    """The oracle built from the in-tree source (compiled on first use)."""
    global _default
    if _default is None:
        _default = Oracle(build())
    return _default


def forward(*a, **kw):
    return load().forward(*a, **kw)


def backward(*a, **kw):
    return load().backward(*a, **kw)


def bias_gather(*a, **kw):
    return load().bias_gather(*a, **kw)


def bias_scatter(*a, **kw):
    return load().bias_scatter(*a, **kw)


def mask_from_labels(*a, **kw):
    return load().mask_from_labels(*a, **kw)


def threads_used() -> int:
    """Thread count of the default oracle's last forward/backward call."""
    return load().threads_used
