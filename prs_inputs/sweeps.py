"""Counter-based, seeded generators for the five sweep workloads.

Every value is a pure function of (seed, config index, field index), so any
slice of a sweep can be regenerated independently and in any order.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_UNI = 0x13104645
SEED_LARGE_P = 0x13104646
SEED_REPLAY = 0x13104647

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


@dataclass
class SweepConfigs:
    """Structure-of-arrays batch of configurations.

    p      int32   number of processors
    q_req  int32   requested number of segments
    m      int64   message size (bytes; plain units in the integer sweep)
    alpha, beta, gamma   int64 or float64, per `cost`
    cost   "i64" or "f64"
    """

    p: np.ndarray
    q_req: np.ndarray
    m: np.ndarray
    alpha: np.ndarray
    beta: np.ndarray
    gamma: np.ndarray
    cost: str

    def __len__(self) -> int:
        return int(self.p.shape[0])

    def take(self, idx) -> "SweepConfigs":
        idx = np.asarray(idx)
        return SweepConfigs(self.p[idx].copy(), self.q_req[idx].copy(), self.m[idx].copy(),
                            self.alpha[idx].copy(), self.beta[idx].copy(), self.gamma[idx].copy(),
                            self.cost)


def _mix64(z: np.ndarray) -> np.ndarray:
    """Bijective 64-bit finaliser (xor-shift-multiply), vectorised."""
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
    return z


def _uniform01(seed: int, index: np.ndarray, field: int) -> np.ndarray:
    """u in [0,1) with 53 random bits, keyed by (seed, index, field)."""
    with np.errstate(over="ignore"):
        k = _mix64(np.full(index.shape, seed, dtype=np.uint64) + np.uint64(0x9E3779B97F4A7C15))
        k = _mix64(k ^ (index.astype(np.uint64) * np.uint64(0xD1342543DE82EF95)))
        k = _mix64(k + np.uint64(field) * np.uint64(0xA0761D6478BD642F))
    return (k >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def _log_uniform_int(u: np.ndarray, lo: int, hi: int) -> np.ndarray:
    v = np.floor(lo * np.power((hi + 1.0) / lo, u))
    return np.clip(v, lo, hi).astype(np.int64)


def _log_uniform_real(u: np.ndarray, lo: float, hi: float) -> np.ndarray:
    return lo * np.power(hi / lo, u)


def tiny_sweep(gammas=(0, 1)) -> SweepConfigs:
    """All (p, q, alpha, gamma) with p in 2..16, q in 1..8, alpha in {0,1,2,4},
    beta = 1, integer time units, unit-size segments (m = q).  No randomness."""
    rows = [(p, q, a, g) for p in range(2, 17) for q in range(1, 9)
            for a in (0, 1, 2, 4) for g in gammas]
    arr = np.array(rows, dtype=np.int64)
    n = arr.shape[0]
    return SweepConfigs(
        p=arr[:, 0].astype(np.int32), q_req=arr[:, 1].astype(np.int32), m=arr[:, 1].copy(),
        alpha=arr[:, 2].copy(), beta=np.ones(n, dtype=np.int64), gamma=arr[:, 3].copy(), cost="i64")


def random_sweep(n: int, seed: int, p_range, q_range, m_range,
                 alpha_range=(1e-6, 1e-4), beta_range=(1e-10, 1e-8),
                 gamma_range=(1e-11, 1e-9), first: int = 0) -> SweepConfigs:
    """n configurations with log-uniform (p, m, q_req, alpha, beta, gamma),
    real-valued (fp64) costs.  `first` offsets the config index so that slices
    of a larger sweep can be drawn on their own."""
    idx = np.arange(first, first + n, dtype=np.uint64)
    p = _log_uniform_int(_uniform01(seed, idx, 0), *p_range).astype(np.int32)
    m = _log_uniform_int(_uniform01(seed, idx, 1), *m_range)
    q = _log_uniform_int(_uniform01(seed, idx, 2), *q_range).astype(np.int32)
    alpha = _log_uniform_real(_uniform01(seed, idx, 3), *alpha_range)
    beta = _log_uniform_real(_uniform01(seed, idx, 4), *beta_range)
    gamma = _log_uniform_real(_uniform01(seed, idx, 5), *gamma_range)
    return SweepConfigs(p=p, q_req=q, m=m, alpha=alpha, beta=beta, gamma=gamma, cost="f64")


def uni_sweep(n: int = 100_000, first: int = 0) -> SweepConfigs:
    """The 100,000-configuration sweep used under both port models:
    p in [2,1024], m in [1 B, 64 MiB], q_req in [1,512]."""
    return random_sweep(n, SEED_UNI, (2, 1024), (1, 512), (1, 1 << 26), first=first)


def large_p_sweep(n: int = 10_000, first: int = 0) -> SweepConfigs:
    """Large machine sweep: p in [1024,65536], q_req in [64,4096],
    m in [1 MiB, 1 GiB]."""
    return random_sweep(n, SEED_LARGE_P, (1024, 65536), (64, 4096), (1 << 20, 1 << 30), first=first)


def replay_config() -> SweepConfigs:
    """Single configuration whose uni-greedy schedule is replayed on data:
    p = 256, 64 segments, m = 2^24 B (2^22 four-byte elements)."""
    return SweepConfigs(p=np.array([256], np.int32), q_req=np.array([64], np.int32),
                        m=np.array([1 << 24], np.int64), alpha=np.array([1e-5]),
                        beta=np.array([1e-9]), gamma=np.array([1e-10]), cost="f64")


def replay_buffers(p: int, n_elems: int, dtype: str, seed: int = SEED_REPLAY,
                   elem_index: np.ndarray | None = None) -> np.ndarray:
    """p buffers of n_elems values: int32 uniform in [-2^20, 2^20], int64 uniform in
    [-2^40, 2^40], or fp32 / fp64 standard normal (Box-Muller on two counter-based
    uniforms).  Each value is
    a function of (seed, buffer, element), so `elem_index` may select any
    subset of element columns of the full-size problem."""
    if elem_index is None:
        elem_index = np.arange(n_elems, dtype=np.uint64)
    e = np.asarray(elem_index, dtype=np.uint64)
    kinds = {"i32": np.int32, "f32": np.float32, "i64": np.int64, "f64": np.float64}
    if dtype not in kinds:
        raise ValueError("dtype must be one of " + ", ".join(kinds))
    out = np.empty((p, e.shape[0]), dtype=kinds[dtype])
    for i in range(p):
        key = e + np.uint64(i) * np.uint64(n_elems)
        if dtype == "i32":
            u = _uniform01(seed, key, 0)
            out[i] = (np.floor(u * (2 ** 21 + 1)) - 2 ** 20).astype(np.int32)
        elif dtype == "i64":
            u = _uniform01(seed, key, 3)
            out[i] = (np.floor(u * (2 ** 41 + 1)) - 2 ** 40).astype(np.int64)
        else:
            u1 = _uniform01(seed, key, 1)
            u2 = _uniform01(seed, key, 2)
            r = np.sqrt(-2.0 * np.log1p(-u1))
            out[i] = (r * np.cos(2.0 * np.pi * u2)).astype(kinds[dtype])
    return out
