"""Seeded synthetic gradient workloads shared by the CPU oracle side and the HIP side.

This module holds input recipes only: it draws random gradient arrays, block
tables and initial models.  None of the method's arithmetic (error feedback,
compression, averaging, AMSGrad) lives here, and it imports neither the oracle
nor the HIP binding.

The five named workloads stand in for the paper's experiments (CIFAR-10 CNN
training and LibSVM logistic regression, Section 7 and Appendix E), whose data
sets are not available: only the parameter counts and the heavy-tailed,
scale-heterogeneous shape of gradients are imitated.  Every array is a pure
function of (seed, step, worker), so any step can be regenerated on its own.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

TOPK = 0
BLOCKSIGN = 1

# hyper-parameters common to all workloads
BETA1 = 0.9
BETA2 = 0.999
EPS = 1e-8
LR = 1e-3


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    n: int                      # workers
    d: int                      # model dimension
    compressor: int             # TOPK | BLOCKSIGN
    k: int = 0                  # Top-k: number kept per worker
    block: int = 0              # block-sign: uniform block length (0 = use block_offsets)
    steps: int = 1
    noise: str = "normal"       # normal | laplace | student_t3_ties | normal_bf16
    scale_lo: float = 1e-3
    scale_hi: float = 1.0
    layer_blocks: int = 0       # >0: this many variable-length blocks
    beta1: float = BETA1
    beta2: float = BETA2
    eps: float = EPS
    lr: float = LR

    # ---- derived inputs -------------------------------------------------
    def scales(self) -> np.ndarray:
        """Per-coordinate scale, log-uniform in [scale_lo, scale_hi], drawn once."""
        rng = np.random.default_rng([self.seed, 0x5CA1E])
        u = rng.random(self.d, dtype=np.float64)
        lo, hi = math.log(self.scale_lo), math.log(self.scale_hi)
        return np.exp(lo + (hi - lo) * u).astype(np.float32)

    def theta0(self) -> np.ndarray:
        rng = np.random.default_rng([self.seed, 0x7E7A])
        return (0.01 * rng.standard_normal(self.d, dtype=np.float32)).astype(np.float32)

    def block_offsets(self) -> np.ndarray | None:
        """int64 offsets[0..n_blocks], offsets[0]=0, offsets[-1]=d; None for Top-k."""
        if self.compressor != BLOCKSIGN:
            return None
        if self.layer_blocks > 0:
            rng = np.random.default_rng([self.seed, 0xB10C])
            lo = math.log(64.0)
            hi = math.log(min(2.4e6, max(128.0, self.d / 4.0)))
            raw = np.exp(lo + (hi - lo) * rng.random(self.layer_blocks))
            lens = np.floor(raw * (self.d / raw.sum())).astype(np.int64)
            lens = np.maximum(lens, 1)
            lens[np.argmax(lens)] += self.d - int(lens.sum())
            assert lens.min() >= 1 and int(lens.sum()) == self.d
            return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        nb = (self.d + self.block - 1) // self.block
        off = np.minimum(np.arange(nb + 1, dtype=np.int64) * self.block, self.d)
        return off

    def _worker_grad(self, step: int, worker: int, s: np.ndarray, hi_idx) -> np.ndarray:
        rng = np.random.default_rng([self.seed, 1 + step, worker])
        d = self.d
        if self.noise == "normal":
            g = rng.standard_normal(d, dtype=np.float32) * s
        elif self.noise == "laplace":
            g = (rng.laplace(0.0, 1.0, d) * s).astype(np.float32)
        elif self.noise == "student_t3_ties":
            g = (rng.standard_t(3.0, d) * s).astype(np.float32)
            # duplicated magnitudes: 2 % of positions copy |g| of a partner taken
            # from the 2 % of coordinates with the largest scale, random sign
            m = max(1, d // 50)
            pos = rng.integers(0, d, m)
            par = hi_idx[rng.integers(0, hi_idx.size, m)]
            sign = np.where(rng.random(m) < 0.5, np.float32(-1.0), np.float32(1.0))
            g[pos] = np.abs(g[par]) * sign
            # 0.1 % exact zeros, fresh positions
            z = rng.integers(0, d, max(1, d // 1000))
            g[z] = np.float32(0.0)
        elif self.noise == "normal_bf16":
            g = rng.standard_normal(d, dtype=np.float32) * s
            u = g.view(np.uint32)
            u = (u + (((u >> 16) & 1) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
            g = u.view(np.float32)
        else:
            raise ValueError(self.noise)
        return np.ascontiguousarray(g, dtype=np.float32)

    def grads(self, step: int, scales: np.ndarray | None = None, threads: int = 8,
              out: np.ndarray | None = None) -> np.ndarray:
        """Gradients of all workers at one step: float32 [n, d], C-contiguous."""
        s = self.scales() if scales is None else scales
        hi_idx = None
        if self.noise == "student_t3_ties":
            top = max(1, self.d // 50)
            hi_idx = np.argpartition(s, self.d - top)[self.d - top:]
        g = np.empty((self.n, self.d), dtype=np.float32) if out is None else out

        def fill(i):
            g[i] = self._worker_grad(step, i, s, hi_idx)

        if threads > 1 and self.n > 1:
            with ThreadPoolExecutor(max_workers=min(threads, self.n)) as ex:
                list(ex.map(fill, range(self.n)))
        else:
            for i in range(self.n):
                fill(i)
        return g

    def scaled(self, d: int, n: int | None = None, steps: int | None = None) -> "Workload":
        """Same recipe at a smaller size (k and block table scale with d)."""
        kw = dict(d=d, name=f"{self.name}@d={d}")
        if n is not None:
            kw["n"] = n
        if steps is not None:
            kw["steps"] = steps
        if self.compressor == TOPK:
            kw["k"] = max(1, round(self.k * d / self.d))
        return dataclasses.replace(self, **kw)

    def algorithmic_bytes(self) -> int:
        """Bytes the method itself must move per step: read g, read e, write e per
        (worker, coordinate); read and write theta, m, v, vhat per coordinate."""
        return 12 * self.n * self.d + 32 * self.d


CONFIGS = [
    Workload("cfg0_topk_n4_d65536", seed=0, n=4, d=65_536, compressor=TOPK, k=655, steps=10,
             noise="normal", scale_lo=1e-3, scale_hi=1.0),
    Workload("cfg1_blocksign4096_n16_d1199882", seed=1, n=16, d=1_199_882, compressor=BLOCKSIGN,
             block=4096, steps=20, noise="laplace", scale_lo=1e-4, scale_hi=1e-1),
    Workload("cfg2_topk_n16_d11173962", seed=2, n=16, d=11_173_962, compressor=TOPK, k=111_740,
             steps=20, noise="student_t3_ties", scale_lo=1e-4, scale_hi=1.0),
    Workload("cfg3_layersign_n32_d25557032", seed=3, n=32, d=25_557_032, compressor=BLOCKSIGN,
             layer_blocks=161, steps=10, noise="normal", scale_lo=1e-5, scale_hi=1.0),
    Workload("cfg4_topk_n8_d110000000", seed=4, n=8, d=110_000_000, compressor=TOPK, k=110_000,
             steps=5, noise="normal_bf16", scale_lo=1e-6, scale_hi=1e-1),
]


def get(idx: int) -> Workload:
    return CONFIGS[idx]


# ----------------------------------------------------------------------------------------------
# Nonconvex logistic regression (Section 6.1, eq. (7)): log-loss plus lam * sum x_j^2 / (1 + x_j^2),
# n workers with equal shares of the samples, full-batch local gradients.  The LibSVM sets of the
# paper are not available here; the data below only imitate their shape (a few hundred binary
# features, about a dozen set per sample, +-1 labels from a noisy linear rule).  This produces the
# inputs g_i of a step from the current model; none of the optimiser's arithmetic lives here.

def logreg_problem(seed: int = 0, samples: int = 4000, d: int = 300, n: int = 20, density: float = 0.04):
    rng = np.random.default_rng([seed, 7])
    a = (rng.random((samples, d)) < density).astype(np.float64)
    x_true = rng.standard_normal(d)
    score = a @ x_true
    y = np.where(score + 0.1 * rng.standard_normal(samples) > np.median(score), 1.0, -1.0)
    return a.reshape(n, samples // n, d), y.reshape(n, samples // n)


def logreg_grads(a: np.ndarray, y: np.ndarray, x: np.ndarray, lam: float = 0.1) -> np.ndarray:
    """Local full-batch gradients [n, d] (float32) of eq. (7) at the model x."""
    x = np.asarray(x, dtype=np.float64)
    z = -y * (a @ x)
    s = 1.0 / (1.0 + np.exp(-z))
    g = -(a * (y * s)[..., None]).mean(axis=1)
    return (g + lam * 2.0 * x / (1.0 + x * x) ** 2).astype(np.float32)
