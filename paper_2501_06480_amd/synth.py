"""Seeded synthetic inputs shaped like the paper's window-attention workloads.

This module only *draws and shapes inputs*; it holds none of the method's
arithmetic, so both the GPU library's tests and the CPU oracle's tests may
use it.  numpy only.

The workloads stand in for Swin Transformer at 224x224 with 7x7 windows
(paper Section 3.2) and for the large-window case the paper's Discussion
rules out for its own hardware:

* Q/K/V/dO: iid N(0,1) drawn in fp32 from a Philox stream keyed by the seed,
  then (for bf16 workloads) rounded once to bf16, round-to-nearest-even, so
  every consumer sees the very same representable values.
* relative-position table: [heads, (2k-1)^2] fp32, N(0, 0.02^2).
* shifted-window mask: [nW, L, L] fp32 with entries 0 / -100, built from the
  published Swin rule: on the H x W token map each axis is cut into the bands
  [0, H-k), [H-k, H-s), [H-s, H) with s the shift; the 9 band pairs are the
  region labels; after window partition, tokens i and j of a window may
  attend to each other iff their labels agree.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


def bf16_round(x: np.ndarray):
    """Round fp32 -> bf16 (nearest even).  Returns (values as fp32, raw uint16 bits)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u                      # NaN never occurs in these inputs; inf stays inf under this add
    r >>= np.uint32(16)
    bits = r.astype(np.uint16)
    r <<= np.uint32(16)
    return r.view(np.float32), bits


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(shape, seed: int, std: float = 1.0) -> np.ndarray:
    x = rng(seed).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def bias_table(heads: int, k: int, seed: int, std: float = 0.02) -> np.ndarray:
    return normal((heads, (2 * k - 1) ** 2), seed, std)


def region_labels(H: int, W: int, k: int, shift: int) -> np.ndarray:
    """[H, W] integer labels of the 9 regions a cyclic shift by `shift` creates."""
    def bands(n):
        b = np.zeros(n, dtype=np.int64)
        b[max(n - k, 0):n - shift] = 1
        b[n - shift:] = 2
        return b
    return bands(H)[:, None] * 3 + bands(W)[None, :]


def window_partition_2d(x: np.ndarray, k: int) -> np.ndarray:
    """[H, W] -> [nW, k*k] with windows in row-major order (paper eq. 1)."""
    H, W = x.shape
    assert H % k == 0 and W % k == 0
    return x.reshape(H // k, k, W // k, k).transpose(0, 2, 1, 3).reshape(-1, k * k)


def shift_labels(H: int, W: int, k: int, shift: int) -> np.ndarray:
    """[nW, L] int32 region labels of the tokens of every window of an H x W map."""
    return window_partition_2d(region_labels(H, W, k, shift), k).astype(np.int32)


def shift_mask(H: int, W: int, k: int, shift: int, neg: float = -100.0) -> np.ndarray:
    """[nW, L, L] fp32 additive mask, 0 where labels agree, `neg` elsewhere."""
    lab = window_partition_2d(region_labels(H, W, k, shift), k)
    same = lab[:, :, None] == lab[:, None, :]
    return np.where(same, np.float32(0.0), np.float32(neg)).astype(np.float32)


@dataclass
class Workload:
    """One attention call: shapes plus how to draw its inputs."""
    name: str
    N: int
    L: int
    C: int
    heads: int
    dtype: str                      # "f32", "bf16" or "f16"
    seed: int
    k: int                          # window side, L == k*k
    map_hw: int = 0                 # token-map side (H == W); 0 = not tied to a map
    use_bias: bool = False
    shift: int = 0                  # 0 = no shift mask
    backward: bool = False
    scale: float = field(init=False)

    def __post_init__(self):
        self.scale = float((self.C // self.heads) ** -0.5)

    @property
    def nW(self) -> int:
        return (self.map_hw // self.k) ** 2 if self.map_hw else 0

    def with_N(self, N: int) -> "Workload":
        """Same recipe on fewer (or more) windows; N stays a multiple of nW if masked."""
        w = Workload(self.name + f"[N={N}]", N, self.L, self.C, self.heads, self.dtype, self.seed,
                     self.k, self.map_hw, self.use_bias, self.shift, self.backward)
        return w


def draw(w: Workload):
    """Draw the inputs of a workload.

    Returns a dict with fp32 arrays ``q, k, v`` (and ``d_o`` for backward
    workloads) holding values already rounded to the workload dtype, the raw
    bf16 bit patterns under ``q_bits`` ... when dtype is bf16, ``table``
    ([heads,(2k-1)^2] fp32 or None), ``mask`` ([nW,L,L] fp32 or None) and
    ``labels`` ([nW,L] int32 region labels the mask was made from, or None).
    """
    out = {}
    names = ["q", "k", "v"] + (["d_o"] if w.backward else [])
    for idx, nm in enumerate(names):
        x = normal((w.N, w.L, w.C), w.seed * 16 + idx)
        if w.dtype == "bf16":
            x, bits = bf16_round(x)
            out[nm + "_bits"] = bits
        elif w.dtype == "f16":
            x = x.astype(np.float16).astype(np.float32)   # rounded once to IEEE half, nearest even
        out[nm] = x
    out["table"] = bias_table(w.heads, w.k, w.seed * 16 + 8) if w.use_bias else None
    out["mask"] = shift_mask(w.map_hw, w.map_hw, w.k, w.shift) if w.shift else None
    out["labels"] = shift_labels(w.map_hw, w.map_hw, w.k, w.shift) if w.shift else None
    return out


def swin_t_stage(stage: int, batch: int = 128, shifted: bool = False, backward: bool = False,
                 seed: Optional[int] = None) -> Workload:
    """Swin-T stage shapes at 224x224 input, 7x7 windows, head dim 32."""
    hw = (56, 28, 14, 7)[stage - 1]
    C = (96, 192, 384, 768)[stage - 1]
    heads = C // 32
    nW = (hw // 7) ** 2
    # A window that covers the whole map is never shifted (Swin convention).
    shift = 3 if (shifted and hw > 7) else 0
    return Workload(f"swin_t_s{stage}{'_shift' if shift else ''}{'_bwd' if backward else ''}",
                    batch * nW, 49, C, heads, "bf16",
                    seed if seed is not None else 1000 + 10 * stage + int(shifted) + 100 * int(backward),
                    7, hw, True, shift, backward)


def config1() -> Workload:
    """Single-head fp32, one 56x56 map, no bias/mask."""
    return Workload("c1_f32_single_head", 64, 49, 32, 1, "f32", 1001, 7, 56)


def config2() -> Workload:
    """Swin-T stage-1 forward, bf16, batch 128, no bias/mask."""
    return Workload("c2_swin_t_s1", 8192, 49, 96, 3, "bf16", 1002, 7, 56)


def config3():
    """All four Swin-T stages, even (bias only) and odd (bias + shift mask) blocks."""
    return [swin_t_stage(s, shifted=sh) for s in (1, 2, 3, 4) for sh in (False, True)]


def config4():
    """Large windows: 12x12 on 48x48 maps and 16x16 on 64x64 maps, batch 64, 4 heads."""
    return [Workload("c4_L144", 64 * 16, 144, 128, 4, "bf16", 1004, 12, 48, True),
            Workload("c4_L256", 64 * 16, 256, 128, 4, "bf16", 1005, 16, 64, True)]


def config5():
    """Forward+backward: stage 1 and stage 3 with bias and shift mask."""
    return [swin_t_stage(1, shifted=True, backward=True), swin_t_stage(3, shifted=True, backward=True)]
