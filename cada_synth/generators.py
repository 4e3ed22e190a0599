"""Seeded synthetic inputs with the shapes of the paper's workloads.

Stand-ins for the datasets of the paper's Section "Simulations" (covtype-,
MNIST- and CIFAR10-shaped inputs); nothing of those datasets is used.  This
module draws data, labels, initial iterates and minibatch index schedules.  It
holds none of CADA's arithmetic and serves both the CPU oracle's tests and the
GPU library's tests, which import neither each other nor anything else in
common.

All generators return a ``Problem``: features ``X`` as float32 ``[sum N_m, d0]``
(worker m owns rows ``[m*N_m, (m+1)*N_m)``), labels ``y`` (float32 +-1 for the
logistic models, int32 class ids for the MLPs) and the initial iterate
``theta0`` (float32 ``[p]``).  For the counter-based recipe ``X`` is ``None``
and rows come from ``Problem.rows``.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import philox
from .configs import CadaConfig


@dataclass
class Problem:
    cfg: CadaConfig
    X: Optional[np.ndarray]
    y: Optional[np.ndarray]
    theta0: np.ndarray
    shift: Optional[np.ndarray] = None      # counter_gauss only: float32 [M, p]

    def rows(self, m: int, local_rows: np.ndarray):
        """Features/labels of worker m's samples ``local_rows`` (worker-local ids)."""
        if self.X is not None:
            g = m * self.cfg.N_m + np.asarray(local_rows, dtype=np.int64)
            return self.X[g], self.y[g]
        from . import native
        if native.have_cpu():          # same function, in C
            return native.rows_cpu(self.cfg.seed, m, local_rows, self.cfg.d0, self.shift[m])
        return philox.counter_rows(self.cfg.seed, m, local_rows, self.cfg.d0, self.shift[m])


def _rng(cfg: CadaConfig, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([cfg.seed, stream]))


def mlp_theta0(cfg: CadaConfig, rng: np.random.Generator) -> np.ndarray:
    """Uniform(-1/sqrt(in), 1/sqrt(in)) for each layer's weights and biases; layout
    layer by layer: W_l row-major [in_l, out_l], then b_l [out_l]."""
    parts = []
    d = cfg.layer_dims
    for i in range(len(d) - 1):
        bound = 1.0 / np.sqrt(d[i])
        parts.append(rng.uniform(-bound, bound, size=d[i] * d[i + 1]))
        parts.append(rng.uniform(-bound, bound, size=d[i + 1]))
    return np.concatenate(parts).astype(np.float32)


def _teacher_labels(X: np.ndarray, dims, rng: np.random.Generator, center: float) -> np.ndarray:
    """argmax of a fixed random ReLU network applied to (X - center)."""
    Ws = [rng.normal(0.0, 1.0 / np.sqrt(dims[i]), size=(dims[i], dims[i + 1])).astype(np.float32)
          for i in range(len(dims) - 1)]
    out = np.empty(X.shape[0], dtype=np.int32)
    for s in range(0, X.shape[0], 16384):
        a = X[s:s + 16384] - np.float32(center)
        for i, W in enumerate(Ws):
            a = a @ W
            if i + 1 < len(Ws):
                a = np.maximum(a, 0.0)
        out[s:s + 16384] = np.argmax(a, axis=1)
    return out


def gauss_shifted(cfg: CadaConfig) -> Problem:
    """x ~ N(mu_m, I), mu_m ~ N(0, 0.25 I); y = sign(x.theta* + logistic noise)."""
    rng = _rng(cfg, 0)
    p, M, N = cfg.p, cfg.M, cfg.N_m
    theta_star = rng.normal(size=p)
    mu = rng.normal(scale=0.5, size=(M, p))
    X = (rng.normal(size=(M, N, p)) + mu[:, None, :]).astype(np.float32).reshape(M * N, p)
    noise = rng.logistic(size=M * N)
    y = np.where(X.astype(np.float64) @ theta_star + noise >= 0, 1.0, -1.0).astype(np.float32)
    return Problem(cfg, X, y, np.zeros(p, dtype=np.float32))


def sparse_uniform(cfg: CadaConfig) -> Problem:
    """x ~ U[0,1] with 80% of the entries zeroed (stored dense); labels from a planted
    direction, threshold at the median score so the classes balance; 5% flipped."""
    rng = _rng(cfg, 0)
    p, M, N = cfg.p, cfg.M, cfg.N_m
    X = rng.random(size=(M * N, p), dtype=np.float32)
    X[rng.random(size=(M * N, p), dtype=np.float32) < np.float32(0.8)] = 0.0
    theta_star = rng.normal(size=p)
    s = X.astype(np.float64) @ theta_star
    y = np.where(s - np.median(s) >= 0, 1.0, -1.0)
    flip = rng.random(size=M * N) < 0.05
    y[flip] = -y[flip]
    return Problem(cfg, X, y.astype(np.float32), np.zeros(p, dtype=np.float32))


def counter_gauss(cfg: CadaConfig) -> Problem:
    """x ~ N(s_m, I/p) from the counter-based recipe in philox.py; s_m ~ N(0, 0.25/p I)."""
    rng = _rng(cfg, 0)
    shift = rng.normal(scale=0.5 / np.sqrt(cfg.p), size=(cfg.M, cfg.p)).astype(np.float32)
    return Problem(cfg, None, None, np.zeros(cfg.p, dtype=np.float32), shift=shift)


def teacher_uniform(cfg: CadaConfig) -> Problem:
    """x ~ U[0,1]^d0; label = argmax of a fixed random teacher MLP, 10% replaced by
    uniformly random classes."""
    rng = _rng(cfg, 0)
    M, N, d0, C = cfg.M, cfg.N_m, cfg.d0, cfg.n_classes
    X = rng.random(size=(M * N, d0), dtype=np.float32)
    y = _teacher_labels(X, (d0, 64, C), rng, 0.5)
    noisy = rng.random(size=M * N) < 0.10
    y[noisy] = rng.integers(0, C, size=int(noisy.sum()), dtype=np.int32)
    return Problem(cfg, X, y, mlp_theta0(cfg, _rng(cfg, 1)))


def teacher_dirichlet(cfg: CadaConfig) -> Problem:
    """x ~ N(0,1)^d0 labelled by a random teacher; worker m's class mix is
    q_m ~ Dirichlet(0.5), class counts ~ Multinomial(N_m, q_m), rows drawn per
    class from a labelled pool (reused cyclically when a class runs short)."""
    rng = _rng(cfg, 0)
    M, N, d0, C = cfg.M, cfg.N_m, cfg.d0, cfg.n_classes
    pool_n = 2 * M * N
    pool = rng.standard_normal(size=(pool_n, d0), dtype=np.float32)
    lab = _teacher_labels(pool, (d0, 64, C), rng, 0.0)
    by_class = [np.flatnonzero(lab == c) for c in range(C)]
    cursor = [0] * C
    X = np.empty((M * N, d0), dtype=np.float32)
    y = np.empty(M * N, dtype=np.int32)
    for m in range(M):
        q = rng.dirichlet(np.full(C, 0.5))
        avail = np.array([len(b) > 0 for b in by_class], dtype=np.float64)
        q = q * avail
        q = q / q.sum()
        counts = rng.multinomial(N, q)
        take = []
        for c in range(C):
            for _ in range(int(counts[c])):
                take.append(by_class[c][cursor[c] % len(by_class[c])])
                cursor[c] += 1
        take = np.asarray(take, dtype=np.int64)
        take = take[rng.permutation(N)]
        X[m * N:(m + 1) * N] = pool[take]
        y[m * N:(m + 1) * N] = lab[take]
    return Problem(cfg, X, y, mlp_theta0(cfg, _rng(cfg, 1)))


RECIPES = {
    "gauss_shifted": gauss_shifted,
    "sparse_uniform": sparse_uniform,
    "counter_gauss": counter_gauss,
    "teacher_uniform": teacher_uniform,
    "teacher_dirichlet": teacher_dirichlet,
}


def make_problem(cfg: CadaConfig) -> Problem:
    return RECIPES[cfg.data](cfg)


def make_schedule(cfg: CadaConfig, K: Optional[int] = None, stream: int = 7) -> np.ndarray:
    """Minibatch index schedule idx[K, M, B] (int32, worker-local row ids): B distinct
    rows per worker per step, independent across steps.  Sampling is an input of
    both implementations, never part of either."""
    K = cfg.K if K is None else K
    rng = _rng(cfg, stream)
    base = np.tile(np.arange(cfg.N_m, dtype=np.int32), (cfg.M, 1))
    out = np.empty((K, cfg.M, cfg.B), dtype=np.int32)
    for k in range(K):
        out[k] = rng.permuted(base, axis=1)[:, :cfg.B]
    return out
