"""Seeded synthetic inputs shaped like the paper's layers.

The paper measures on synthetic random matrices (Sec. IV-A) with shapes taken from
Transformer / LSTM layers (Sec. II-C); the five configurations below are the ones this
repository is measured on.  This module only draws random numbers: it holds none of the
method's arithmetic and serves the GPU library's callers and the CPU oracle's callers alike.

Conventions: B int8 [q][m][n] of +1/-1, alpha float32 [q][m], X float32 [b][n].
Draw order for a workload: X, then B_1..B_q, then alpha_1..alpha_q, from
``numpy.random.default_rng(seed)``.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

BASE_SEED = 200509904


@dataclass(frozen=True)
class Workload:
    name: str
    m: int
    n: int
    q: int
    batch: int
    mu: int
    alpha_kind: str  # "uniform", "two_level", "sorted_desc"
    alpha_lo: float = 0.05
    alpha_hi: float = 1.0
    seed: int = BASE_SEED

    @property
    def chunks(self) -> int:
        return -(-self.n // self.mu)

    @property
    def key_bytes(self) -> int:
        """Bytes of packed signs the method has to read: q*m*ceil(n/8)."""
        return self.q * self.m * (-(-self.n // 8))

    @property
    def algorithmic_bytes(self) -> int:
        """key bytes + alpha + X + Y, the traffic the method itself needs per call."""
        return self.key_bytes + 4 * self.q * self.m + 4 * self.n * self.batch + 4 * self.m * self.batch

    @property
    def lookups(self) -> int:
        return self.q * self.m * self.chunks * self.batch

    @property
    def dense_equiv_ops(self) -> int:
        return 2 * self.m * self.n * self.batch * self.q

    def scaled_m(self, m: int, name: str | None = None) -> "Workload":
        return replace(self, m=m, name=name or "%s_m%d" % (self.name, m))

    def with_mu(self, mu: int) -> "Workload":
        return replace(self, mu=mu, name="%s_mu%d" % (self.name, mu))


CONFIGS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("cfg1_fc512_b1", 512, 512, 1, 1, 8, "uniform", 0.1, 1.0, BASE_SEED + 1),
        Workload("cfg2_gemv2048_q2_b1", 2048, 2048, 2, 1, 8, "two_level", 0.1, 1.0, BASE_SEED + 2),
        Workload("cfg3_lstm4096x1024_q3_b8", 4096, 1024, 3, 8, 8, "sorted_desc", 0.05, 1.0, BASE_SEED + 3),
        Workload("cfg4_sq4096_q3_b32", 4096, 4096, 3, 32, 8, "uniform", 0.05, 1.0, BASE_SEED + 4),
        Workload("cfg5_ffn_up_q2_b128", 16384, 4096, 2, 128, 8, "uniform", 0.05, 1.0, BASE_SEED + 50),
        Workload("cfg5_ffn_down_q2_b128", 4096, 16384, 2, 128, 8, "uniform", 0.05, 1.0, BASE_SEED + 51),
    ]
}


def draw_X(rng: np.random.Generator, batch: int, n: int) -> np.ndarray:
    return rng.standard_normal((batch, n), dtype=np.float32)


def draw_B(rng: np.random.Generator, q: int, m: int, n: int) -> np.ndarray:
    """iid uniform +1/-1 as int8, drawn one plane at a time to bound memory."""
    B = np.empty((q, m, n), dtype=np.int8)
    for i in range(q):
        bits = rng.integers(0, 2, size=(m, n), dtype=np.int8)
        np.multiply(bits, 2, out=bits)
        np.subtract(bits, 1, out=bits)
        B[i] = bits
    return B


def draw_alpha(rng: np.random.Generator, w: Workload) -> np.ndarray:
    q, m = w.q, w.m
    if w.alpha_kind == "two_level":
        # plane 1 carries the large scale, later planes the small one
        planes = [rng.uniform(0.5, 1.0, size=m)]
        planes += [rng.uniform(0.1, 0.5, size=m) for _ in range(q - 1)]
        a = np.stack(planes)
    else:
        a = np.stack([rng.uniform(w.alpha_lo, w.alpha_hi, size=m) for _ in range(q)])
        if w.alpha_kind == "sorted_desc":
            a = -np.sort(-a, axis=0)
    return a.astype(np.float32)


def make_inputs(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Returns (B, alpha, X) for a workload, fully determined by ``w.seed``."""
    rng = np.random.default_rng(w.seed)
    X = draw_X(rng, w.batch, w.n)
    B = draw_B(rng, w.q, w.m, w.n)
    alpha = draw_alpha(rng, w)
    return B, alpha, X


def make_exact_inputs(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Inputs on which every fp32 partial sum is exactly representable: X holds small
    integers (|x| <= 8) and alpha powers of two, so any summation order gives the same bits."""
    rng = np.random.default_rng(w.seed + 7919)
    X = rng.integers(-8, 9, size=(w.batch, w.n)).astype(np.float32)
    B = draw_B(rng, w.q, w.m, w.n)
    alpha = (2.0 ** rng.integers(-3, 2, size=(w.q, w.m))).astype(np.float32)
    return B, alpha, X
