"""Seeded synthetic inputs shaped like the five benchmark configurations (Brownian-like paths).

This module holds no arithmetic of the signature-kernel method: it only draws paths.  It is the one
module shared by the CPU oracle's tests and the HIP path's tests/benchmark.

Recipe for every path: x[0] = 0, x[i] = sum of the first i increments; increments are drawn with
numpy's ``default_rng(seed)`` in float64.  The paper benchmarks on shapes only (Table 2 gives
(B, L, d) triples, no dataset), so these stand in for nothing else.
"""
from dataclasses import dataclass

import numpy as np

FLAG_TIME_AUG = 1


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str          # "pairs" or "gram"
    n_x: int           # B for pairs, N for gram
    n_y: int           # B for pairs, M for gram
    L: int
    d: int
    lam: int
    flags: int
    backward: bool
    seed_x: int
    seed_y: int
    inc_var_num: float  # increment variance = inc_var_num / (L * var_d)
    var_d: int
    drift: float        # per-path drift vector ~ U(-drift, drift), spread over unit time

    @property
    def cells_per_pair(self) -> int:
        return ((self.L - 1) << self.lam) ** 2

    @property
    def pairs(self) -> int:
        return self.n_x if self.kind == "pairs" else self.n_x * self.n_y


def brownian_paths(seed: int, count: int, L: int, d: int, inc_var: float, drift: float = 0.0) -> np.ndarray:
    """count paths of L points in R^d starting at 0 with i.i.d. N(0, inc_var) increments plus, when
    drift > 0, a per-path drift vector mu ~ U(-drift, drift)^d contributing mu/(L-1) per step."""
    rng = np.random.default_rng(seed)
    inc = rng.normal(0.0, np.sqrt(inc_var), size=(count, max(L - 1, 0), d))
    if drift > 0.0 and L > 1:
        mu = rng.uniform(-drift, drift, size=(count, 1, d))
        inc = inc + mu / (L - 1)
    x = np.zeros((count, L, d), dtype=np.float64)
    if L > 1:
        x[:, 1:, :] = np.cumsum(inc, axis=1)
    return x


WORKLOADS = {
    # 8 pairs, L=32, d=2, N(0,1/L), dyadic order 0, forward
    "c1": Workload("c1", "pairs", 8, 8, 32, 2, 0, 0, False, 1001, 1002, 1.0, 1, 0.0),
    # 128 pairs, L=256, d=5, N(0,1/L), time augmentation, dyadic order 1, forward + backward
    "c2": Workload("c2", "pairs", 128, 128, 256, 5, 1, FLAG_TIME_AUG, True, 2001, 2002, 1.0, 1, 0.0),
    # Gram 256 x 256, L=128, d=3, N(0,0.5/L) + drift U(-0.5,0.5), dyadic order 1, forward + backward
    "c3": Workload("c3", "gram", 256, 256, 128, 3, 1, 0, True, 3001, 3002, 0.5, 1, 0.5),
    # 32 pairs, L=2048, d=8, N(0,1/L), dyadic order 2, forward + backward
    "c4": Workload("c4", "pairs", 32, 32, 2048, 8, 2, 0, True, 4001, 4002, 1.0, 1, 0.0),
    # Gram 1024 x 1024, L=64, d=16, N(0,1/(dL)), dyadic order 0, forward + backward
    "c5": Workload("c5", "gram", 1024, 1024, 64, 16, 0, 0, True, 5001, 5002, 1.0, 16, 0.0),
}


def make(name: str, n_x: int = None, n_y: int = None, L: int = None):
    """Returns (workload, X, Y) in float64; n_x / n_y / L override the batch sizes and length (used by
    the parity tests to cut a configuration down to what the oracle finishes in seconds)."""
    w = WORKLOADS[name]
    if n_x is not None or n_y is not None or L is not None:
        w = Workload(w.name, w.kind, n_x or w.n_x, n_y or w.n_y, L or w.L, w.d, w.lam, w.flags, w.backward,
                     w.seed_x, w.seed_y, w.inc_var_num, w.var_d, w.drift)
    var = w.inc_var_num / (w.L * w.var_d)
    X = brownian_paths(w.seed_x, w.n_x, w.L, w.d, var, w.drift)
    Y = brownian_paths(w.seed_y, w.n_y, w.L, w.d, var, w.drift)
    return w, X, Y


def upstream_weights(seed: int, shape) -> np.ndarray:
    """Seeded N(0,1) upstream gradients dF/dk (or dF/dK) for backward tests."""
    return np.random.default_rng(seed).normal(0.0, 1.0, size=shape)


# Truncated signatures (paper Table 1 gives shapes (B, L, d, N) only, no dataset): Brownian-like paths with
# N(0, 1/L) increments per channel, so that the entries of level k are of order 1/sqrt(k!).
SIGNATURE_WORKLOADS = {
    "s1": (128, 256, 4, 6, 6001),
    "s2": (128, 512, 8, 5, 6002),
    "s3": (128, 1024, 16, 4, 6003),
}


def make_signature(name: str, B: int = None, L: int = None):
    """Returns ((B, L, d, N), X[B,L,d]) in float64; B / L override the batch size and the length."""
    B0, L0, d, N, seed = SIGNATURE_WORKLOADS[name]
    B = B or B0
    L = L or L0
    return (B, L, d, N), brownian_paths(seed, B, L, d, 1.0 / L0)
