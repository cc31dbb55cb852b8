"""Seeded synthetic inputs: FNO-shaped complex gradients and initial weights.

This module only draws random inputs.  It holds none of the optimizer's
arithmetic (no selection, no projection, no Adam), so both the GPU path and the
CPU oracle may be fed from it.  Everything is generated on the host with
numpy's counter-based Philox generator.

The shapes follow the paper's FNO spectral weights (in-channels, out-channels,
modes_x, half-spectrum modes_y; e.g. 128 channels x 128 modes -> 128x128x128x65,
appendix table of architectures) and its qualitative picture of a gradient: a
smooth low-rank part plus sharp, sparse outliers whose positions persist over
many steps (section "Robust decomposition of gradients").  They stand in for
gradients of FNO layers trained on the paper's PDE datasets, which are not
available here.

CN(0, s2) below means real and imaginary parts are independent N(0, s2 / 2).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 250102379


@dataclass(frozen=True)
class Workload:
    name: str
    shape: Tuple[int, ...]
    ranks: Tuple[int, ...]       # Tucker rank per mode
    k: int                       # sparse entries, ceil(density * numel)
    density: Tuple[int, int]     # density as an exact fraction (num, den)
    T: int                       # refresh period
    steps: int                   # steps of the full job
    layers: int = 1
    grad_dtype: str = "c64"      # "c64" or "cbf16" (bf16 (re, im) pairs)
    kind: str = "noise_outliers" # or "lowrank_t_outliers"
    outlier_frac: Tuple[int, int] = (5, 1000)
    config_id: int = 0
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    alpha: float = 1.0
    lam: float = 1.0
    weight_decay: float = 0.0
    planted_rank: Tuple[int, ...] = (16, 16, 8, 4)   # "lowrank_t_outliers": Tucker rank of the planted signal

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n


# The five benchmark configurations.  Ranks and k are literal numbers here (the
# arithmetic that derives them from ratios is the method's and lives elsewhere).
WORKLOADS = {
    "cfg1": Workload("cfg1", (16, 16, 8, 5), (8, 8, 4, 3), 103, (1, 100), 5, 10, config_id=1),
    "cfg2": Workload("cfg2", (64, 64, 32, 17), (16, 16, 8, 4), 44565, (2, 100), 50, 200,
                     kind="lowrank_t_outliers", outlier_frac=(1, 100), config_id=2),
    "cfg3": Workload("cfg3", (128, 128, 64, 33), (32, 32, 16, 8), 346031, (1, 100), 100, 100,
                     layers=4, config_id=3),
    "cfg4": Workload("cfg4", (128, 128, 128, 65), (32, 32, 32, 16), 681575, (5, 1000), 200, 200,
                     config_id=4),
    "cfg5": Workload("cfg5", (32, 32, 32, 32, 17), (8, 8, 8, 8, 4), 178258, (1, 100), 100, 500,
                     grad_dtype="cbf16", config_id=5),
}


# Stand-in for the gradient of the robust-decomposition comparison (section "Robust decomposition
# of gradients", the reconstruction-error figure: a complex 64^3 x 32 gradient of an FNO layer,
# sparse 5 % + low rank 20 %, low rank 20 % + sparse 5 %, pure low rank 25 %): a planted low-rank
# signal, noise, and heavy-tailed outliers at 1 % of the positions.  Ranks and k below are those of
# the 5 % + 20 % strategy; 25 % per mode is (16, 16, 16, 8).
RECON_DIAGNOSTIC = Workload("recon", (64, 64, 64, 32), (13, 13, 13, 6), 419431, (5, 100), 1, 1,
                            kind="lowrank_t_outliers", outlier_frac=(1, 100), config_id=6,
                            planted_rank=(8, 8, 8, 4))


def _rng(*key_words: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=np.array(
        [int(key_words[0]) & 0xFFFFFFFFFFFFFFFF,
         (int(key_words[1]) if len(key_words) > 1 else 0) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)))


def complex_normal(rng: np.random.Generator, shape, variance: float = 1.0) -> np.ndarray:
    """CN(0, variance) as complex64."""
    out = np.empty(shape, dtype=np.complex64)
    s = np.float32(np.sqrt(variance / 2.0))
    v = out.view(np.float32).reshape(-1)
    # fill in chunks to bound the float64 temporaries numpy creates
    n = v.size
    step = 1 << 24
    for a in range(0, n, step):
        b = min(n, a + step)
        v[a:b] = rng.standard_normal(b - a, dtype=np.float32) * s
    return out


def outlier_positions(numel: int, frac: Tuple[int, int], seed: int) -> np.ndarray:
    """round(frac * numel) distinct linear positions, fixed by `seed`."""
    m = int(round(frac[0] * numel / frac[1]))
    rng = _rng(seed, 0x0A11CE)
    if m == 0:
        return np.zeros(0, dtype=np.int64)
    # distinct positions without materialising a permutation of numel
    pos = np.unique(rng.integers(0, numel, size=int(m * 1.2) + 16, dtype=np.int64))
    while pos.size < m:
        extra = rng.integers(0, numel, size=m, dtype=np.int64)
        pos = np.unique(np.concatenate([pos, extra]))
    pos = rng.permutation(pos)[:m]
    return np.sort(pos)


def float32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16).  Finite inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def complex64_to_bf16_pairs(g: np.ndarray) -> np.ndarray:
    """complex64 array -> uint16 array with a trailing axis of 2: (re, im) bf16 bits."""
    f = np.ascontiguousarray(g, dtype=np.complex64).view(np.float32).reshape(g.shape + (2,))
    return float32_to_bf16_bits(f)


def _planted_factors(w: Workload):
    """Fixed orthonormal factors of the planted low-rank signal (cfg2)."""
    true_rank = tuple(w.planted_rank)
    Q = []
    for n, (i, r) in enumerate(zip(w.shape, true_rank)):
        rng = _rng(BASE_SEED + 1000 * w.config_id, 0xFAC + n)
        a = rng.standard_normal((i, r)) + 1j * rng.standard_normal((i, r))
        q, _ = np.linalg.qr(a)
        Q.append(q.astype(np.complex64))
    return Q, true_rank


def gradient(w: Workload, step: int, layer: int = 0, scale: float = 1.0) -> np.ndarray:
    """Gradient of workload `w` at `step` for `layer`.

    Returns complex64 of shape w.shape, or for "cbf16" workloads a uint16 array
    of shape w.shape + (2,) holding bf16 (re, im) bit patterns."""
    seed = BASE_SEED + 1000 * w.config_id + step
    rng = _rng(seed, 0x6D + 7919 * layer)
    numel = w.numel
    pos = outlier_positions(numel, w.outlier_frac, 97 + w.config_id + 131 * layer)
    if w.kind == "noise_outliers":
        g = complex_normal(rng, w.shape, 1.0)
        flat = g.reshape(-1)
        flat[pos] *= np.float32(20.0)
    elif w.kind == "lowrank_t_outliers":
        Q, true_rank = _planted_factors(w)
        csize = int(np.prod(true_rank))
        core = complex_normal(rng, true_rank, 1.0) * np.float32(np.sqrt(numel / csize))
        sig = core
        for n, q in enumerate(Q):
            sig = np.moveaxis(np.tensordot(q, sig, axes=(1, n)), 0, n)
        # C-contiguous on purpose: the outliers below are added through a flat VIEW
        g = np.ascontiguousarray(sig, dtype=np.complex64) + complex_normal(rng, w.shape, 0.1)
        assert g.flags.c_contiguous
        t = rng.standard_t(2.0, size=(pos.size, 2)).astype(np.float32) * np.float32(10.0)
        flat = g.reshape(-1)
        flat[pos] += (t[:, 0] + 1j * t[:, 1]).astype(np.complex64)
    else:
        raise ValueError(w.kind)
    if scale != 1.0:
        g *= np.float32(scale)
    if w.grad_dtype == "cbf16":
        return complex64_to_bf16_pairs(g)
    return g


def initial_weight(w: Workload, layer: int = 0) -> np.ndarray:
    """W_0 ~ CN(0, 0.02^2), complex64."""
    rng = _rng(BASE_SEED + 1000 * w.config_id, 0x77 + 7919 * layer)
    return complex_normal(rng, w.shape, 0.02 ** 2)


def small_case(shape, seed: int, outlier_frac=(1, 100), dtype: str = "c64",
               ties: bool = False) -> np.ndarray:
    """A generic seeded gradient for edge-case tests (odd shapes, ties)."""
    rng = _rng(seed, 0x5CA1E)
    g = complex_normal(rng, tuple(shape), 1.0)
    flat = g.reshape(-1)
    pos = outlier_positions(flat.size, outlier_frac, seed + 1)
    flat[pos] *= np.float32(20.0)
    if ties and flat.size >= 8:
        # plant equal-magnitude groups: g, -g, i*g, conj(g) share one key
        src = flat[0]
        flat[1] = -src
        flat[flat.size // 2] = 1j * src
        flat[-1] = np.conj(src)
    if dtype == "cbf16":
        return complex64_to_bf16_pairs(g)
    return g
