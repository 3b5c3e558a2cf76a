"""Seeded synthetic workloads for the DD-EF-SGD hot path.

This module only manufactures *inputs*: the curvature vector lambda, the optimum x*, the
start point x0 of the diagonal quadratic f(x) = 1/2 sum_j lambda_j (x_j - x*_j)^2, and the
(bandwidth, latency) trace that drives the adaptive (delta, tau) schedule.  It holds none of
the method's arithmetic (no gradient, no error feedback, no top-k, no DeCo rule) and imports
neither the HIP binding nor the CPU oracle, so both sides can be fed the same arrays.

The five named workloads stand in for the paper's training tasks (Section 5.2: ResNet,
ViT-B ~86 M and GPT-2 124 M parameter vectors, 4-32 workers, compression ratios of 10 % or
less): same flat vector lengths, worker counts, delta and tau ranges, with gradients coming
from the quadratic instead of a network.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

NOISE_NONE = 0
NOISE_GAUSS = 1
NOISE_STUDENT_T3 = 2

_CHUNK = 1 << 24


@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    n: int
    deltas: Tuple[float, ...]
    tau: int
    tau_max: int
    lr: float
    steps: int
    seed: int
    noise_kind: int
    noise_scale: float
    lambda_lo_exp: float = -3.0      # lambda ~ 10^U[lo, 0]
    n_blocks: int = 0                # >0: per-block lambda scale (ResNet-like layout)
    adaptive_period: int = 0         # >0: (delta, tau) re-chosen every this many steps
    note: str = ""


WORKLOADS = {
    "C1": Workload("C1", 1_000_000, 4, (0.01,), 2, 2, 0.05, 20, 0, NOISE_GAUSS, 0.1),
    "C2": Workload("C2", 11_700_000, 8, (0.01,), 4, 4, 0.05, 100, 1, NOISE_GAUSS, 0.1,
                   lambda_lo_exp=-4.0, n_blocks=62),
    "C3": Workload("C3", 124_000_000, 8, (0.001,), 8, 8, 0.05, 50, 2, NOISE_STUDENT_T3, 0.05),
    "C4": Workload("C4", 1_300_000_000, 4, (0.1, 0.01, 0.001), 4, 4, 0.05, 10, 3, NOISE_GAUSS, 0.05),
    "C5": Workload("C5", 124_000_000, 16, (0.01,), 0, 16, 0.05, 500, 4, NOISE_GAUSS, 0.05,
                   adaptive_period=50),
}


def get(name: str, d: Optional[int] = None, n: Optional[int] = None) -> Workload:
    """Named workload, optionally shrunk (same recipe, smaller d / n) for parity tests."""
    w = WORKLOADS[name]
    if d is not None:
        w = replace(w, d=int(d))
    if n is not None:
        w = replace(w, n=int(n))
    return w


def _fill_chunks(out: np.ndarray, fn) -> None:
    d = out.shape[0]
    for lo in range(0, d, _CHUNK):
        hi = min(d, lo + _CHUNK)
        out[lo:hi] = fn(hi - lo)


def block_layout(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Seeded partition of [0, d) into n_blocks layer-like blocks and a scale per block.

    Block weights 10^U[3, 6.4] (layers from a thousand to a few million parameters), sizes
    proportional to the weights with the remainder given to the last block; scale per block
    10^U[lambda_lo_exp, 0].  Returns (block start offsets of length n_blocks+1, scales).
    """
    rng = np.random.default_rng([w.seed, 0xB10C])
    wt = 10.0 ** rng.uniform(3.0, 6.4, size=w.n_blocks)
    sizes = np.floor(wt / wt.sum() * w.d).astype(np.int64)
    sizes = np.maximum(sizes, 1)
    sizes[-1] += w.d - int(sizes.sum())
    if sizes[-1] < 1:
        raise ValueError("d too small for the block layout")
    starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    scales = (10.0 ** rng.uniform(w.lambda_lo_exp, 0.0, size=w.n_blocks)).astype(np.float32)
    return starts, scales


def make_problem(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(lambda, xstar, x0) as contiguous float32 arrays of length d, from the workload's seed."""
    d = w.d
    lam = np.empty(d, dtype=np.float32)
    xstar = np.empty(d, dtype=np.float32)
    x0 = np.empty(d, dtype=np.float32)
    if w.n_blocks > 0:
        starts, scales = block_layout(w)
        for b in range(w.n_blocks):
            lam[starts[b]:starts[b + 1]] = scales[b]
    else:
        rl = np.random.default_rng([w.seed, 1])
        lo = w.lambda_lo_exp
        _fill_chunks(lam, lambda m: (10.0 ** rl.uniform(lo, 0.0, size=m)).astype(np.float32))
    rs = np.random.default_rng([w.seed, 2])
    _fill_chunks(xstar, lambda m: rs.standard_normal(m, dtype=np.float32))
    r0 = np.random.default_rng([w.seed, 3])
    _fill_chunks(x0, lambda m: r0.standard_normal(m, dtype=np.float32))
    return lam, xstar, x0


@dataclass(frozen=True)
class NetworkTrace:
    """One (bandwidth, latency) observation per adaptation period."""
    bandwidth_bps: np.ndarray   # bits/s, log-uniform over [0.1, 10] Gbps
    latency_s: np.ndarray       # seconds, uniform over [10, 300] ms
    v_g_bits: float             # dense fp32 gradient volume, 32*d bits
    t_comp_s: float             # synthetic per-iteration compute time
    delta_bounds: Tuple[float, float] = (1e-4, 1e-1)
    tau_bounds: Tuple[int, int] = (0, 16)


def network_trace(w: Workload, t_comp_s: float = 0.02) -> NetworkTrace:
    """Seeded trace for the adaptive workload: one draw per period of `adaptive_period` steps."""
    if w.adaptive_period <= 0:
        raise ValueError("workload has no adaptive schedule")
    periods = (w.steps + w.adaptive_period - 1) // w.adaptive_period
    rng = np.random.default_rng([w.seed, 0x7ACE])
    bw = 10.0 ** rng.uniform(np.log10(0.1e9), np.log10(10e9), size=periods)
    lat = rng.uniform(0.010, 0.300, size=periods)
    return NetworkTrace(bw, lat, 32.0 * float(w.d), float(t_comp_s),
                        tau_bounds=(0, w.tau_max))


def random_vector(seed: int, d: int, kind: str = "normal") -> np.ndarray:
    """Auxiliary seeded fp32 vectors for unit tests of the selection (ties, denormals, ...)."""
    rng = np.random.default_rng([seed, 0x5E1])
    if kind == "normal":
        return rng.standard_normal(d, dtype=np.float32)
    if kind == "heavy":
        return (rng.standard_t(3, size=d) * 0.05).astype(np.float32)
    if kind == "few_values":       # many exact ties
        return rng.integers(-3, 4, size=d).astype(np.float32) * np.float32(0.25)
    if kind == "all_equal":
        return np.full(d, 0.5, dtype=np.float32)
    if kind == "signed_zero":
        v = np.zeros(d, dtype=np.float32)
        v[::2] = -0.0
        return v
    if kind == "denormal":
        bits = rng.integers(0, 1 << 12, size=d, dtype=np.uint32)
        bits |= rng.integers(0, 2, size=d, dtype=np.uint32) << np.uint32(31)
        return bits.view(np.float32)
    if kind == "wide":             # magnitudes over (almost) the whole finite exponent range;
        # the top is left free so that a handful of such vectors can be summed without overflow
        bits = rng.integers(0, 0x7D800000, size=d, dtype=np.uint32)
        bits |= rng.integers(0, 2, size=d, dtype=np.uint32) << np.uint32(31)
        return bits.view(np.float32)
    raise ValueError(kind)
