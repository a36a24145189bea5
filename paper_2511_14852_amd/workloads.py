"""Seeded synthetic workloads for the Chebyshev-KAN layer.

This module only names shapes and draws random inputs.  It holds none of the
layer's arithmetic, so the GPU path and the CPU oracle can both consume the
same bits without sharing any of the method's code.

The five workloads follow the configurations this build is measured on:
one small layer, a tabular-regression-shaped stack (huge batch, tiny widths),
a speech-shaped stack, an audio-enhancement-shaped stack and one large square
layer.  The stacks mirror the "widths a->b->c->d, one degree per model" form of
the paper's benchmark suite (Table 2); the real datasets are replaced by
normal-distributed features of the same row counts and widths.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 251114852


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # position in the configuration list (1-based)
    batch: int
    widths: Tuple[int, ...]    # layer l maps widths[l] -> widths[l+1]
    degree: int
    x_mean: float = 0.0
    x_std: float = 1.0
    note: str = ""

    @property
    def layers(self) -> List[Tuple[int, int]]:
        return [(self.widths[l], self.widths[l + 1]) for l in range(len(self.widths) - 1)]


WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1", 1, 256, (64, 64), 4, note="single small layer"),
    "c2": Workload("c2", 2, 65536, (8, 64, 64, 1), 6, note="tabular-regression-shaped stack"),
    "c3": Workload("c3", 3, 64 * 512, (80, 512, 512, 256), 3, note="speech-shaped stack, 64 sequences x 512 frames"),
    "c4": Workload("c4", 4, 16 * 1000, (257, 512, 512, 257), 5, x_mean=-2.0, x_std=1.5,
                   note="audio-enhancement-shaped stack, 16 clips x 1000 STFT frames"),
    "c5": Workload("c5", 5, 16384, (1024, 1024), 8, note="large square layer"),
    # the paper's own single-layer operator shapes (Table 5): tiny batch, high degree
    "p1": Workload("p1", 11, 128, (40, 256), 8, note="paper operator shape 1 (speech-like)"),
    "p2": Workload("p2", 12, 64, (256, 512), 15, note="paper operator shape 2 (VoiceBank-like)"),
    "p3": Workload("p3", 13, 32, (512, 1024), 24, note="paper operator shape 3 (house-price-like)"),
}

_KIND = {"x": 0, "C": 1, "dy": 2}


def tensor_seed(cfg_index: int, layer: int, kind: str) -> int:
    return BASE_SEED + 1000 * cfg_index + 10 * layer + _KIND[kind]


def _normal(seed: int, shape, mean: float, std: float) -> np.ndarray:
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=shape)          # fp64 draws
    return np.ascontiguousarray((a * std + mean).astype(np.float32))


def make_x(batch: int, n_in: int, seed: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """Row-major [batch, in] fp32 inputs ~ N(mean, std^2)."""
    return _normal(seed, (batch, n_in), mean, std)


def make_coeff(n_in: int, n_out: int, degree: int, seed: int) -> np.ndarray:
    """Row-major [in, out, degree+1] fp32 coefficients ~ N(0, 1/(in*(degree+1)))."""
    std = 1.0 / np.sqrt(float(n_in) * float(degree + 1))
    return _normal(seed, (n_in, n_out, degree + 1), 0.0, std)


def make_dy(batch: int, n_out: int, seed: int) -> np.ndarray:
    """Row-major [batch, out] fp32 upstream gradient ~ N(0,1)."""
    return _normal(seed, (batch, n_out), 0.0, 1.0)


def workload_inputs(w: Workload, batch: int | None = None):
    """Host tensors of a workload: first-layer x, per-layer C, last-layer dy.

    `batch` overrides the row count (used for bounded CPU samples and small
    parity cases); the draws for a smaller batch are a prefix-independent fresh
    draw with the same seed, which is all the tests rely on.
    """
    b = w.batch if batch is None else int(batch)
    x0 = make_x(b, w.widths[0], tensor_seed(w.index, 0, "x"), w.x_mean, w.x_std)
    coeffs = [make_coeff(i, o, w.degree, tensor_seed(w.index, l, "C"))
              for l, (i, o) in enumerate(w.layers)]
    dy_last = make_dy(b, w.widths[-1], tensor_seed(w.index, len(w.layers) - 1, "dy"))
    return x0, coeffs, dy_last


def layer_flops(batch: int, n_in: int, n_out: int, degree: int) -> int:
    """Useful contraction flops of one layer's forward + backward.

    forward 2*B*I*O*(d+1), coefficient gradient the same, input gradient
    2*B*I*O*d (T'_0 = 0 contributes nothing).
    """
    return 2 * batch * n_in * n_out * (3 * degree + 2)


def layer_bytes(batch: int, n_in: int, n_out: int, degree: int) -> int:
    """Algorithmic HBM bytes of one layer's forward + backward in fp32.

    forward reads x, C and writes y; backward reads x, C, dy and writes dx, dC.
    The basis tensor and any partial buffers are not counted: fusion removes
    the first and the second is implementation overhead.
    """
    k = degree + 1
    fwd = batch * n_in + n_in * n_out * k + batch * n_out
    bwd = batch * n_in + n_in * n_out * k + batch * n_out + batch * n_in + n_in * n_out * k
    return 4 * (fwd + bwd)
