"""Seeded synthetic inputs for the structured-tensor kernels.

This module only draws numbers.  It holds none of the arithmetic of the
method (no index maps, no kernels): array lengths are passed in by the
caller or listed as literals in ``CONFIGS``.  Both the GPU tests/bench and
the CPU oracle tests take their inputs from here, so the two sides always
see the same bytes.

Generator: a counter-based 64-bit mixer (the SplitMix64 finaliser applied to
``seed + (index+1) * golden_gamma``), so element ``index`` of an array depends
on ``(seed, index)`` only and any slice can be drawn on its own.

* ``uniform``  : the top 24 bits ``k`` give ``(k + 0.5) * 2**-23 - 1`` which is
  exactly representable in fp32, lies strictly inside (-1, 1) and is never 0.
* ``normal``   : Box-Muller in fp64 on two 53-bit uniforms in (0, 1), scaled by
  ``std`` and then rounded once to fp32.

The synthetic arrays stand in for the paper's synthetic kernel sweeps
(covariance creation over a swept number of features; TTM / MTTKRP over
structured operands); the paper's public-data experiment is not reproduced.
"""
from __future__ import annotations

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(seed: int, idx: np.ndarray) -> np.ndarray:
    """SplitMix64 output for counters ``idx`` (uint64 array) under ``seed``."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + (idx + np.uint64(1)) * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform(seed: int, count: int, start: int = 0) -> np.ndarray:
    """``count`` fp32 values in (-1, 1), elements ``start .. start+count-1``."""
    out = np.empty(count, dtype=np.float32)
    for lo in range(0, count, _CHUNK):
        hi = min(count, lo + _CHUNK)
        idx = np.arange(start + lo, start + hi, dtype=np.uint64)
        k = (_mix(seed, idx) >> np.uint64(40)).astype(np.float64)
        out[lo:hi] = ((k + 0.5) * 2.0 ** -23 - 1.0).astype(np.float32)
    return out


def normal(seed: int, count: int, std: float = 1.0, start: int = 0) -> np.ndarray:
    """``count`` fp32 draws from N(0, std**2), elements ``start ..``."""
    out = np.empty(count, dtype=np.float32)
    for lo in range(0, count, _CHUNK):
        hi = min(count, lo + _CHUNK)
        idx = np.arange(start + lo, start + hi, dtype=np.uint64)
        a = _mix(seed, idx * np.uint64(2))
        b = _mix(seed, idx * np.uint64(2) + np.uint64(1))
        u1 = ((a >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        u2 = ((b >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:hi] = (g * std).astype(np.float32)
    return out


def seed_for(config_index: int, array_index: int) -> int:
    """Seed of array ``array_index`` (0-based, in the listed order) of config 1..5."""
    return 0x53540000 + 16 * config_index + array_index


# The five workloads.  Entry counts are literals (they are also what the
# index-map tests check the closed forms against).
CONFIGS = {
    1: dict(kernel="mttkrp_sym3", n=64, R=16, entries=45_760, b_dist="uniform"),
    2: dict(kernel="batax_utri", n=8192, beta=0.5, entries=33_558_528),
    3: dict(kernel="ttm_band", n=512, w=8, nl=512, R=64, band_pairs=8_632),
    4: dict(kernel="mttkrp_sym3", n=512, R=64, entries=22_500_864, b_dist="normal"),
    5: dict(kernel="moment3_sym", N=2_000_000, n=64, entries=45_760),
}


def mttkrp_inputs(n: int, R: int, entries: int, b_dist: str = "uniform",
                  config_index: int = 1):
    """Packed symmetric 3-tensor (``entries`` values) and factor ``B`` (n x R)."""
    Tc = uniform(seed_for(config_index, 0), entries)
    if b_dist == "uniform":
        B = uniform(seed_for(config_index, 1), n * R)
    else:
        B = normal(seed_for(config_index, 1), n * R, std=1.0 / np.sqrt(float(n)))
    return Tc, B.reshape(n, R)


def batax_inputs(n: int, entries: int, config_index: int = 2):
    """Packed upper-triangular ``A`` (``entries`` values) and vector ``x``."""
    Ap = uniform(seed_for(config_index, 0), entries)
    x = uniform(seed_for(config_index, 1), n)
    return Ap, x


def ttm_inputs(band_pairs: int, nl: int, R: int, config_index: int = 3):
    """Packed band fibres ``[band_pairs][nl]`` and matrix ``U`` (nl x R)."""
    Tc = uniform(seed_for(config_index, 0), band_pairs * nl).reshape(band_pairs, nl)
    U = uniform(seed_for(config_index, 1), nl * R).reshape(nl, R)
    return Tc, U


def moment_inputs(N: int, n: int, config_index: int = 5, start_sample: int = 0):
    """Sample matrix ``X`` (N x n), standard normal, rows ``start_sample ..``."""
    X = normal(seed_for(config_index, 0), N * n, std=1.0, start=start_sample * n)
    return X.reshape(N, n)
