"""Seeded synthetic inputs: coordinate grids and SIREN-style initial weights.

This module serves both the GPU library's callers and the CPU oracle's tests,
so it holds none of the method's arithmetic (no rotation, no quantizer, no
network evaluation) -- only the data recipe:

* coordinates: a side x side pixel grid on [-1, 1]^2, row-major, (x, y) pairs,
  standing in for the image-fitting workloads of the paper's experiments
  (Sec. 4.1-4.2: 2-D images, 3-channel or 1-channel output);
* weights: uniform, first layer on [-1/2, 1/2] (the range the paper reports for
  layer 1, Sec. 3.1), later layers on +-sqrt(6/fan_in)/omega0, biases on
  +-1/sqrt(fan_in); drawn from a counter-based splitmix64 stream so that any
  implementation can regenerate them from (seed, index).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """Outputs start .. start+count-1 of the splitmix64 stream seeded with `seed`.

    Output i is mix(seed + (i+1)*GAMMA) with the published finaliser
    (xor-shift 30, multiply, xor-shift 27, multiply, xor-shift 31), mod 2^64.
    """
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform(seed: int, start: int, count: int, lo: float, hi: float) -> np.ndarray:
    """count fp32 values uniform on [lo, hi): top 24 bits of each splitmix64 output."""
    u = (splitmix64(seed, start, count) >> np.uint64(40)).astype(np.float64) / float(1 << 24)
    return (lo + (hi - lo) * u).astype(np.float32)


def grid_coords(side: int) -> np.ndarray:
    """(side*side, 2) fp32: coords[i*side + j] = (v_j, v_i), v_t = -1 + 2t/(side-1)."""
    v = (-1.0 + 2.0 * np.arange(side, dtype=np.float64) / float(max(side - 1, 1)))
    xx, yy = np.meshgrid(v, v, indexing="xy")  # xx[i, j] = v_j, yy[i, j] = v_i
    return np.stack([xx.reshape(-1), yy.reshape(-1)], axis=1).astype(np.float32)


def siren_init(dims: List[int], omega0: float, seed: int) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """Weights W[l] (dims[l+1] x dims[l], row-major) and biases b[l], layer-major draw order:
    all of W[0], then b[0], then W[1], ..."""
    W, b = [], []
    pos = 0
    for l in range(len(dims) - 1):
        fan_in, fan_out = dims[l], dims[l + 1]
        bound = 0.5 if l == 0 else float(np.sqrt(6.0 / fan_in) / omega0)
        W.append(uniform(seed, pos, fan_out * fan_in, -bound, bound).reshape(fan_out, fan_in))
        pos += fan_out * fan_in
        bb = float(1.0 / np.sqrt(fan_in))
        b.append(uniform(seed, pos, fan_out, -bb, bb))
        pos += fan_out
    return W, b


def wire_init(dims_c: List[int], omega0: float, seed: int) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """Complex weights Wc[l] (dims_c[l+1] x dims_c[l], complex64) and biases bc[l] for a network
    with complex-valued hidden features (the second architecture of the paper's Table 1): the
    first layer real on [-1/2, 1/2] (real coordinates in), later layers with real and imaginary
    parts each uniform on +-sqrt(3/fan_in)/omega0 (so that |w|^2 has the variance of the
    real-valued initialisation above), biases likewise on +-1/sqrt(2 fan_in), the last layer's
    bias real.  Draw order: Re W[0], Im W[0] (skipped for the first layer), Re b[0], Im b[0]
    (skipped for the last layer), Re W[1], ..."""
    W, b = [], []
    pos = 0
    L = len(dims_c) - 1
    for l in range(L):
        fan_in, fan_out = dims_c[l], dims_c[l + 1]
        bound = 0.5 if l == 0 else float(np.sqrt(3.0 / fan_in) / omega0)
        re = uniform(seed, pos, fan_out * fan_in, -bound, bound).reshape(fan_out, fan_in)
        pos += fan_out * fan_in
        im = np.zeros_like(re)
        if l > 0:
            im = uniform(seed, pos, fan_out * fan_in, -bound, bound).reshape(fan_out, fan_in)
            pos += fan_out * fan_in
        W.append((re + 1j * im).astype(np.complex64))
        bb = float(1.0 / np.sqrt(2.0 * fan_in))
        bre = uniform(seed, pos, fan_out, -bb, bb)
        pos += fan_out
        bim = np.zeros_like(bre)
        if l < L - 1:
            bim = uniform(seed, pos, fan_out, -bb, bb)
            pos += fan_out
        b.append((bre + 1j * bim).astype(np.complex64))
    return W, b


@dataclass(frozen=True)
class Workload:
    name: str
    dims: Tuple[int, ...]
    side: int
    omega0: float = 30.0
    bits: Tuple[int, ...] = (8,)
    seed: int = 0

    @property
    def n_coords(self) -> int:
        return self.side * self.side

    def int8_ops_per_coord(self) -> int:
        """2 ops per MAC over the un-padded layer shapes."""
        return 2 * sum(self.dims[l] * self.dims[l + 1] for l in range(len(self.dims) - 1))


def _siren(width: int, hidden: int) -> Tuple[int, ...]:
    return (2,) + (width,) * hidden + (3,)


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", _siren(64, 3), 64, seed=0xD4000001),
    "C2": Workload("C2", _siren(256, 4), 256, seed=0xD4000002),
    "C3": Workload("C3", _siren(256, 5), 512, seed=0xD4000003),
    "C4": Workload("C4", _siren(256, 5), 1024, bits=(4, 6, 8), seed=0xD4000004),
    "C5": Workload("C5", _siren(512, 6), 2048, seed=0xD4000005),
}


def make(name: str):
    """(workload, coords, W, b) for a named configuration."""
    wl = WORKLOADS[name]
    W, b = siren_init(list(wl.dims), wl.omega0, wl.seed)
    return wl, grid_coords(wl.side), W, b
