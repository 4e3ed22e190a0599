"""The five seeded synthetic workloads, as plain data.

This module holds hyper-parameters and shapes only: none of CADA's arithmetic
lives here.  Symbols follow the paper: ``M`` workers, ``p`` parameters,
``d_max`` past steps averaged on the right-hand side of the communication rule
(Section 2.2, conditions (workerrule1)/(workerrule2)), ``D`` the maximum delay
that forces an upload and, for CADA1, the snapshot period (Algorithm 1).

Where a workload leaves a hyper-parameter open, the value is taken from the
paper's own tables: alpha = 0.005, beta = (0.9, 0.999), lambda = 1e-5, D = 100
for the logistic tasks (supplementary Table "covtype", Section "Simulation
details"), alpha = 0.0005 for the neural-network tasks (Table "MNIST").
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Tuple

RULE_ALWAYS = 0   # every worker uploads every iteration (distributed Adam/AMSGrad baseline, Section 4)
RULE_CADA1 = 1
RULE_CADA2 = 2
RULE_LAG = 3      # stochastic LAG, condition (LAGrule) of Section 2.1
SERVER_AMSGRAD = 0
SERVER_SGD = 1    # theta <- theta - alpha * nabla, the update stochastic LAG follows


@dataclass(frozen=True)
class CadaConfig:
    name: str
    model: str                    # "logreg" | "mlp"
    layer_dims: Tuple[int, ...]   # logreg: (p,) ; mlp: (d0, d1, ..., dL)
    M: int                        # workers
    N_m: int                      # samples per worker (uniform)
    B: int                        # minibatch rows per worker per step
    K: int                        # iterations
    rule: int                     # RULE_*
    D: int                        # max delay / CADA1 snapshot period
    d_max: int = 10
    c: float = 0.5
    alpha: float = 0.005
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    lam: float = 0.0              # l2 coefficient (logistic only)
    gemm_dtype: str = "fp32"      # "fp32" | "bf16" (MLP contractions)
    seed: int = 0
    data: str = ""                # name of the input recipe in generators.py
    server: int = SERVER_AMSGRAD  # SERVER_*
    alpha_K0: int = 0             # 0: constant stepsize; else alpha_k = alpha K0/(k+K0) (Theorem 2)

    @property
    def p(self) -> int:
        if self.model == "logreg":
            return int(self.layer_dims[0])
        d = self.layer_dims
        return int(sum(d[i] * d[i + 1] + d[i + 1] for i in range(len(d) - 1)))

    @property
    def d0(self) -> int:
        return int(self.layer_dims[0])

    @property
    def n_classes(self) -> int:
        return int(self.layer_dims[-1]) if self.model == "mlp" else 2

    def scaled(self, **kw) -> "CadaConfig":
        """A copy with some fields replaced (reduced shapes for tests)."""
        return dataclasses.replace(self, **kw)


CFG1 = CadaConfig(
    name="cfg1_logreg_p54_cada2", model="logreg", layer_dims=(54,), M=10, N_m=1000, B=10,
    K=200, rule=RULE_CADA2, D=50, d_max=10, c=0.5, alpha=0.005, lam=1e-5, seed=1000,
    data="gauss_shifted")

CFG2 = CadaConfig(
    name="cfg2_logreg_p784_cada1", model="logreg", layer_dims=(784,), M=20, N_m=3000, B=32,
    K=2000, rule=RULE_CADA1, D=100, d_max=10, c=1.0, alpha=0.005, lam=1e-5, seed=2000,
    data="sparse_uniform")

CFG3 = CadaConfig(
    name="cfg3_logreg_p65536_cada2", model="logreg", layer_dims=(65536,), M=100, N_m=4096,
    B=256, K=500, rule=RULE_CADA2, D=100, d_max=10, c=0.3, alpha=0.005, lam=1e-5, seed=3000,
    data="counter_gauss")

CFG4 = CadaConfig(
    name="cfg4_mlp_784_512_10_cada2", model="mlp", layer_dims=(784, 512, 10), M=64, N_m=6000,
    B=128, K=1000, rule=RULE_CADA2, D=100, d_max=10, c=0.5, alpha=0.0005, gemm_dtype="bf16",
    seed=4000, data="teacher_uniform")

CFG5 = CadaConfig(
    name="cfg5_mlp_3072_1024_1024_10_cada1", model="mlp", layer_dims=(3072, 1024, 1024, 10),
    M=16, N_m=3125, B=256, K=500, rule=RULE_CADA1, D=200, d_max=10, c=0.5, alpha=0.0005,
    gemm_dtype="bf16", seed=5000, data="teacher_dirichlet")

ALL = {1: CFG1, 2: CFG2, 3: CFG3, 4: CFG4, 5: CFG5}
