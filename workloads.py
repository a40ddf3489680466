"""Seeded synthetic inputs and the geometry of the five benchmark workloads.

This module only draws random arrays and names shapes.  It holds none of the
method's arithmetic (no filtering, pooling, normalisation or cost), so both the
CPU oracle's tests and the HIP path's tests may take their inputs from here
without sharing any code of the method itself.

The arrays stand in for the natural photographs the paper trains on (Sec. 4:
whitened 300x300x3 images): 1/f "pink" noise reproduces the amplitude spectrum
of natural images, which keeps contrast normalisation and the sparsity term
away from degenerate inputs.  Everything is drawn in fp64 on the host from
``numpy.random.default_rng(seed)`` and cast to fp32; the same fp32 arrays go to
the oracle (up-cast) and to the GPU.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class LCGeom:
    """Geometry of one locally connected layer (Sec. 3.1: receptive field,
    stride, filters per location; mini-batch)."""

    B: int
    H: int
    W: int
    C: int
    R: int
    S: int
    F: int

    @property
    def LH(self) -> int:
        return (self.H - self.R) // self.S + 1

    @property
    def LW(self) -> int:
        return (self.W - self.R) // self.S + 1

    @property
    def L(self) -> int:
        return self.LH * self.LW

    @property
    def K(self) -> int:
        return self.R * self.R * self.C

    @property
    def params(self) -> int:
        return self.L * self.K * self.F

    @property
    def flop_per_pass(self) -> int:
        return 2 * self.B * self.K * self.F * self.L

    def with_batch(self, B: int) -> "LCGeom":
        return LCGeom(B, self.H, self.W, self.C, self.R, self.S, self.F)

    def as_tuple(self) -> Tuple[int, ...]:
        return (self.B, self.H, self.W, self.C, self.R, self.S, self.F)


# The five workloads (1-based, as the benchmark description numbers them).
CONFIG_GEOM: Dict[str, LCGeom] = {
    "cfg1": LCGeom(B=8, H=32, W=32, C=3, R=8, S=4, F=16),
    "cfg2": LCGeom(B=64, H=96, W=96, C=3, R=16, S=8, F=64),
    "cfg3": LCGeom(B=128, H=200, W=200, C=3, R=20, S=4, F=32),
    "cfg4": LCGeom(B=256, H=64, W=64, C=32, R=8, S=2, F=128),
    # three-stage step: LC (valid) -> 3x3 L2 pool (valid) -> 5x5 LCN (same size)
    "cfg5_s1": LCGeom(B=128, H=128, W=128, C=3, R=16, S=2, F=16),
    "cfg5_s2": LCGeom(B=128, H=55, W=55, C=16, R=6, S=2, F=32),
    "cfg5_s3": LCGeom(B=128, H=23, W=23, C=32, R=6, S=2, F=32),
}
# The first layer exactly as the architecture section states it (Sec. 3.1: 300x300x3 input, 16x16
# receptive field, stride 4 -> 72x72 fields, a 4x4x24 output block = 384 filters per field; the
# mini-batch of 192 is the one the same section's training paragraph gives).  1.53e9 parameters: fits one GPU whole.
PAPER_LAYER1 = LCGeom(B=192, H=300, W=300, C=3, R=16, S=4, F=384)

# The dense third layer of the same section (62x62x24 responses -> 4096 units) is the one-field case of
# the same contraction: R = H = W, so L = 1, K = 92,256 and F = 4096 (3.8e8 parameters).
PAPER_LAYER3 = LCGeom(B=192, H=62, W=62, C=24, R=62, S=1, F=4096)

CONFIG_IMAGE_KIND = {
    "cfg1": "gaussian", "cfg2": "pink", "cfg3": "pink", "cfg4": "halfnormal",
    "cfg5_s1": "pink", "cfg5_s2": "halfnormal", "cfg5_s3": "halfnormal",
}

POOL_KSIZE, POOL_STRIDE, POOL_EPS = 3, 1, 1e-6
LCN_KSIZE, LCN_SIGMA, LCN_EPS = 5, 1.0, 1e-4
SAE_LAMBDA, SAE_EPS, SAE_LR = 0.1, 1e-6, 1e-3
SAE_LAMBDA_DENSE = 0.01     # the sparsity weight the paper gives for its dense third layer (next to Eq. 1)


def _standardise(x: np.ndarray) -> np.ndarray:
    """Per-image zero mean and unit variance over all of H*W*C."""
    flat = x.reshape(x.shape[0], -1)
    flat = flat - flat.mean(axis=1, keepdims=True)
    flat = flat / flat.std(axis=1, keepdims=True)
    return flat.reshape(x.shape)


def gaussian_images(rng: np.random.Generator, B: int, H: int, W: int, C: int) -> np.ndarray:
    return _standardise(rng.standard_normal((B, H, W, C))).astype(np.float32)


def pink_images(rng: np.random.Generator, B: int, H: int, W: int, C: int) -> np.ndarray:
    """White Gaussian field per image and channel, shaped to a 1/f amplitude
    spectrum (frequency in cycles per image, DC removed), then standardised."""
    fy = np.fft.fftfreq(H) * H
    fx = np.fft.rfftfreq(W) * W
    f = np.sqrt(fy[:, None] ** 2 + fx[None, :] ** 2)
    gain = 1.0 / np.maximum(f, 1.0 / H)
    gain[0, 0] = 0.0
    out = np.empty((B, H, W, C), dtype=np.float64)
    for b in range(B):
        white = rng.standard_normal((C, H, W))
        spec = np.fft.rfft2(white, axes=(1, 2)) * gain[None]
        out[b] = np.moveaxis(np.fft.irfft2(spec, s=(H, W), axes=(1, 2)), 0, -1)
    return _standardise(out).astype(np.float32)


def halfnormal_maps(rng: np.random.Generator, B: int, H: int, W: int, C: int) -> np.ndarray:
    return np.abs(rng.standard_normal((B, H, W, C))).astype(np.float32)


def images(kind: str, rng: np.random.Generator, B: int, H: int, W: int, C: int) -> np.ndarray:
    if kind == "gaussian":
        return gaussian_images(rng, B, H, W, C)
    if kind == "pink":
        return pink_images(rng, B, H, W, C)
    if kind == "halfnormal":
        return halfnormal_maps(rng, B, H, W, C)
    raise ValueError(kind)


def lc_inputs(g: LCGeom, kind: str = "pink", seed: int = 0, with_bias: bool = False):
    """x, w, dy (and optionally a bias) for one layer, as fp32 arrays.

    Sub-streams are spawned in the fixed order x, w, dy, b so that a change to
    one array's shape never moves another array's values.
    Layouts: x [B,H,W,C]; w [LH,LW,K,F] with k=(kh*R+kw)*C+c; dy [B,LH,LW,F].
    """
    rx, rw, rdy, rb = np.random.default_rng(seed).spawn(4)
    x = images(kind, rx, g.B, g.H, g.W, g.C)
    w = (rw.standard_normal((g.LH, g.LW, g.K, g.F)) / np.sqrt(g.K)).astype(np.float32)
    dy = rdy.standard_normal((g.B, g.LH, g.LW, g.F)).astype(np.float32)
    if with_bias:
        bias = (0.1 * rb.standard_normal((g.LH, g.LW, g.F))).astype(np.float32)
        return x, w, dy, bias
    return x, w, dy


def lc_inputs_blocked(g: LCGeom, kind: str = "pink", seed: int = 0, threads: int = 8):
    """x, w, dy for a layer too large for `lc_inputs` to draw in fp64 in one piece.

    w and dy are drawn directly in fp32, one row of fields (fixed i) per sub-stream, so the values
    do not depend on the number of worker threads; x comes from the same image generators.
    """
    from concurrent.futures import ThreadPoolExecutor

    rx, rw, rdy = np.random.default_rng(seed).spawn(3)
    x = images(kind, rx, g.B, g.H, g.W, g.C)
    w = np.empty((g.LH, g.LW, g.K, g.F), dtype=np.float32)
    dy = np.empty((g.B, g.LH, g.LW, g.F), dtype=np.float32)
    scale = np.float32(1.0 / np.sqrt(g.K))

    def fill_row(args):
        i, r_w, r_dy = args
        r_w.standard_normal(out=w[i], dtype=np.float32)
        w[i] *= scale
        dy[:, i] = r_dy.standard_normal((g.B, g.LW, g.F), dtype=np.float32)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(fill_row, zip(range(g.LH), rw.spawn(g.LH), rdy.spawn(g.LH))))
    return x, w, dy


def feature_maps(B: int, H: int, W: int, C: int, seed: int = 0, signed: bool = True) -> np.ndarray:
    """Generic activations for the pooling / normalisation tests."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, H, W, C))
    if not signed:
        x = np.abs(x)
    return x.astype(np.float32)


def to_bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest-even bf16 and return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)
