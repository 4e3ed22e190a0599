"""Builds a CadaOracle from a workload description.  TEST INFRASTRUCTURE ONLY
(see cada_oracle.py); duck-typed on the config so it imports nothing but the
oracle itself."""
from __future__ import annotations

from .cada_oracle import CadaOracle


def oracle_for(cfg, problem, **override) -> CadaOracle:
    kw = dict(model=cfg.model, layer_dims=cfg.layer_dims, M=cfg.M, rule=cfg.rule, D=cfg.D,
              d_max=cfg.d_max, c=cfg.c, alpha=cfg.alpha, beta1=cfg.beta1, beta2=cfg.beta2,
              eps=cfg.eps, lam=cfg.lam, theta0=problem.theta0, rows=problem.rows,
              server=getattr(cfg, "server", 0), alpha_K0=getattr(cfg, "alpha_K0", 0))
    kw.update(override)
    return CadaOracle(**kw)
