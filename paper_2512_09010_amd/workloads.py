"""Seeded synthetic inputs with the shapes and statistics of the benchmark configurations.

This module serves both the HIP path and the CPU oracle and therefore holds
NONE of the method's arithmetic: it only draws random fields, casts them once
to the I/O dtype and describes the five workloads (grid, dtype, merge
schedule, SPU shape, keep ratio, cut-off).

The fields stand in for visual-encoder / LLM activations of the paper's image,
tiled-image and video workloads (Section 4 evaluates on public suites that are
not reproduced here): smooth 2-D Gaussian random fields (neighbouring patches
are similar, as OIM presumes in Section 3.2) plus white noise.

bfloat16 data travels as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

AXIS_H, AXIS_W = 0, 1
BASE_SEED = 20251209


# ----------------------------------------------------------------------------- dtype plumbing

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even cast fp32 -> bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def cast_io(a: np.ndarray, dtype: str) -> np.ndarray:
    """Cast generated fp32 values once to the I/O dtype ('f32' array or 'bf16' bit patterns)."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """I/O array -> fp64 values (exact)."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


# ----------------------------------------------------------------------------- random fields

def _blur_wrap(a: np.ndarray, ell: float, axis: int) -> np.ndarray:
    """Periodic blur with exp(-t^2 / 2 ell^2) truncated at +-4 ell, rescaled to keep unit variance.

    The truncated kernel is wrapped onto the axis and applied as a circular convolution (through a
    real FFT along the axis, chunked to bound memory), which is exact for any kernel length.
    """
    if ell <= 0:
        return a
    n = a.shape[axis]
    r = int(4.0 * ell + 0.5)
    t = np.arange(-r, r + 1, dtype=np.float64)
    k = np.exp(-0.5 * (t / ell) ** 2)
    k /= k.sum()
    kk = np.zeros(n)
    np.add.at(kk, np.arange(-r, r + 1) % n, k)                  # the kernel may wrap onto itself on a short axis
    kk /= np.sqrt((kk ** 2).sum())                              # i.i.d. N(0,1) in -> unit variance out
    Kf = np.fft.rfft(kk)
    a = np.ascontiguousarray(np.moveaxis(a, axis, -1))
    out = np.empty(a.shape, a.dtype)
    flat_in, flat_out = a.reshape(-1, n), out.reshape(-1, n)
    step = max(1, (1 << 22) // n)
    for i in range(0, flat_in.shape[0], step):
        flat_out[i:i + step] = np.fft.irfft(np.fft.rfft(flat_in[i:i + step], axis=-1) * Kf, n=n, axis=-1)
    return np.ascontiguousarray(np.moveaxis(out, -1, axis))


def grf(rng: np.random.Generator, shape: Tuple[int, ...], ell: float, axes=(-3, -2)) -> np.ndarray:
    """Unit-variance smooth field: i.i.d. N(0,1) per (cell, channel) blurred along the grid axes."""
    a = rng.standard_normal(shape, dtype=np.float32)
    for ax in axes:
        a = _blur_wrap(a, ell, ax)
    return a


def smooth_field(rng, B, H, W, D, ell, noise=0.1):
    """[B,H,W,D] fp32: grf(ell) + noise * N(0,1)."""
    return grf(rng, (B, H, W, D), ell) + np.float32(noise) * rng.standard_normal((B, H, W, D), dtype=np.float32)


def video_field(rng, B, T, H, W, D, ell, rho=0.9, noise=0.1):
    """[B,T,H,W,D] fp32: AR(1) in time (f_t = rho f_{t-1} + sqrt(1-rho^2) g_t) over smooth frames."""
    out = np.empty((B, T, H, W, D), np.float32)
    for t in range(T):
        g = smooth_field(rng, B, H, W, D, ell, noise)
        out[:, t] = g if t == 0 else np.float32(rho) * out[:, t - 1] + np.float32(np.sqrt(1 - rho * rho)) * g
    return out


def multiscale_field(rng, B, H, W, D, ells=(2, 8, 32), t_scale=0.1, t_dof=3):
    """[B,H,W,D] fp32: sum of smooth fields at several length scales + heavy-tailed Student-t noise."""
    a = np.zeros((B, H, W, D), np.float32)
    for ell in ells:
        a += grf(rng, (B, H, W, D), ell)
    a /= np.float32(np.sqrt(len(ells)))
    a += np.float32(t_scale) * rng.standard_t(t_dof, (B, H, W, D)).astype(np.float32)
    return a


def project(rng, x: np.ndarray, d_out: int) -> np.ndarray:
    """Seeded Gaussian projection [..., d_in] -> [..., d_out], P ~ N(0, 1/d_in)."""
    d_in = x.shape[-1]
    P = rng.standard_normal((d_in, d_out), dtype=np.float32) / np.float32(np.sqrt(d_in))
    return (x.reshape(-1, d_in) @ P).reshape(*x.shape[:-1], d_out)


# ----------------------------------------------------------------------------- workloads

@dataclass
class Workload:
    """One benchmark configuration.

    ``oim_calls`` lists the merge calls applied in sequence to the grids; each call is a
    list of (axis, m) passes.  ``tokens_in`` is the number of visual tokens entering OIM
    (the unit of the throughput metric).
    """
    name: str
    dtype: str                      # 'f32' | 'bf16'
    grids: int                      # number of independent H x W grids handed to OIM
    H: int
    W: int
    D: int
    oim_calls: List[List[Tuple[int, int]]]
    spu_B: int
    spu_N: int
    spu_D: int
    keep_ratio: float
    kind: str = "image"             # image | tiles | video | multiscale
    ell: float = 3.0
    group: int = 1                  # grids concatenated into one SPU sample (tiles / frames)
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def tokens_in(self) -> int:
        return self.grids * self.H * self.W

    @property
    def n_keep(self) -> int:
        return min(self.spu_N, max(1, int(np.floor(self.keep_ratio * self.spu_N + 0.5))))

    @property
    def sigma(self) -> int:
        # The paper gives no value for the cut-off; pass-band fraction = keep fraction.
        return max(1, int(np.floor(self.keep_ratio * self.spu_N / 2)))

    def out_grid(self) -> Tuple[int, int]:
        H, W = self.H, self.W
        for call in self.oim_calls:
            for axis, m in call:
                if axis == AXIS_W:
                    W -= m
                else:
                    H -= m
        return H, W


def halving_call(H: int, W: int) -> List[Tuple[int, int]]:
    """One OIM operation = one pass along W then one along H, each merging every source."""
    return [(AXIS_W, (W + 1) // 2), (AXIS_H, (H + 1) // 2)]


def workload(i: int) -> Workload:
    s = BASE_SEED + i
    if i == 0:
        return Workload("cfg0_image_24x24_f32", "f32", 1, 24, 24, 1024, [halving_call(24, 24)],
                        1, 144, 4096, 0.25, "image", 3.0, 1, s)
    if i == 1:
        return Workload("cfg1_batch8_64x64_bf16", "bf16", 8, 64, 64, 1280, [halving_call(64, 64)],
                        8, 1024, 3584, 0.20, "image", 4.0, 1, s)
    if i == 2:
        return Workload("cfg2_batch16_5tiles_24x24_bf16", "bf16", 80, 24, 24, 1024, [halving_call(24, 24)],
                        16, 720, 4096, 0.15, "tiles", 3.0, 5, s)
    if i == 3:
        return Workload("cfg3_batch4_video32_16x16_bf16", "bf16", 128, 16, 16, 1152, [halving_call(16, 16)],
                        4, 2048, 3584, 0.10, "video", 3.0, 32, s)
    if i == 4:
        return Workload("cfg4_batch2_112x112_bf16", "bf16", 2, 112, 112, 1280,
                        [halving_call(112, 112), halving_call(56, 56), halving_call(28, 28)],
                        2, 196, 4096, 0.05, "multiscale", 0.0, 1, s, {"ells": (2, 8, 32)})
    raise ValueError("configs are numbered 0..4")


def mini(i: int) -> Workload:
    """A small relative of configuration i (same kind, dtype and schedule shape) for quick parity runs."""
    w = workload(i)
    if i == 0:
        return w
    if i == 1:
        return Workload("mini1", "bf16", 2, 16, 16, 320, [halving_call(16, 16)], 2, 64, 448, 0.20, "image", 2.0, 1, w.seed)
    if i == 2:
        return Workload("mini2", "bf16", 6, 12, 12, 256, [halving_call(12, 12)], 2, 108, 512, 0.15, "tiles", 2.0, 3, w.seed)
    if i == 3:
        return Workload("mini3", "bf16", 8, 8, 8, 192, [halving_call(8, 8)], 2, 64, 384, 0.10, "video", 2.0, 4, w.seed)
    return Workload("mini4", "bf16", 1, 28, 28, 160, [halving_call(28, 28), halving_call(14, 14)], 1, 49, 256, 0.05,
                    "multiscale", 0.0, 1, w.seed, {"ells": (1, 3, 8)})


def oim_input(w: Workload, reseed: int = 0) -> np.ndarray:
    """OIM input of a workload, cast once to its I/O dtype: [grids,H,W,D] (fp32 values or bf16 bits)."""
    rng = np.random.default_rng(w.seed + 1000 * reseed)
    if w.kind in ("image", "tiles"):
        a = smooth_field(rng, w.grids, w.H, w.W, w.D, w.ell)
    elif w.kind == "video":
        a = video_field(rng, w.grids // w.group, w.group, w.H, w.W, w.D, w.ell).reshape(w.grids, w.H, w.W, w.D)
    else:
        a = multiscale_field(rng, w.grids, w.H, w.W, w.D, w.extra.get("ells", (2, 8, 32)))
    return cast_io(a, w.dtype)


def spu_input(w: Workload, reseed: int = 0) -> np.ndarray:
    """SPU input of a workload: [spu_B, spu_N, spu_D] in the I/O dtype.

    A field of the same family drawn directly on the merged grid (length scales divided by the
    linear reduction factor), at the encoder width, pushed through a seeded Gaussian projection
    to the LLM width.  Sequence order: tile-major / frame-major, then raster.
    """
    rng = np.random.default_rng(w.seed + 500 + 1000 * reseed)
    Ho, Wo = w.out_grid()
    shrink = w.H / Ho
    if w.kind in ("image", "tiles"):
        a = smooth_field(rng, w.grids, Ho, Wo, w.D, w.ell / shrink)
    elif w.kind == "video":
        a = video_field(rng, w.grids // w.group, w.group, Ho, Wo, w.D, w.ell / shrink).reshape(w.grids, Ho, Wo, w.D)
    else:
        a = multiscale_field(rng, w.grids, Ho, Wo, w.D, tuple(e / shrink for e in w.extra.get("ells", (2, 8, 32))))
    a = a.reshape(w.spu_B, w.group * Ho * Wo, w.D)
    assert a.shape[1] == w.spu_N, (a.shape, w.spu_N)
    return cast_io(project(rng, a, w.spu_D), w.dtype)


def spu_input_from_merged(w: Workload, merged: np.ndarray, reseed: int = 0) -> np.ndarray:
    """SPU input of a workload made from a merged grid: [grids,Ho,Wo,D] values (any float type) ->
    [spu_B, spu_N, spu_D] in the I/O dtype, by the seeded Gaussian projection to the LLM width.

    This is the hand-over the configurations describe (OIM output, projected, then SPU); whoever calls it
    supplies the merged tokens - the HIP path its own, the oracle its own.  Sequence order: tile-major /
    frame-major, then raster.
    """
    rng = np.random.default_rng(w.seed + 700 + 1000 * reseed)
    Ho, Wo = w.out_grid()
    a = np.asarray(merged, dtype=np.float32).reshape(w.spu_B, w.group * Ho * Wo, w.D)
    assert a.shape[1] == w.spu_N, (a.shape, w.spu_N)
    return cast_io(project(rng, a, w.spu_D), w.dtype)
