"""Full-data objective and accuracy (cada_eval) against the oracle's evaluate(), after a few
iterations under mask replay so that both stand at (nearly) the same iterate."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators
from paper_2012_15469_amd.binding import Cada

from common import upload, to_dev, oracle_run

pytestmark = pytest.mark.gpu

CASES = [
    (configs.CFG1.scaled(K=30), 1e-5),
    (configs.CFG2.scaled(M=6, N_m=333, K=30, D=10), 1e-5),                 # N_m no multiple of anything
    (configs.CFG3.scaled(layer_dims=(8200,), M=4, N_m=130, B=32, K=12, D=5, alpha=0.02, c=1e-4), 1e-5),
    (configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=301, B=70, K=15, D=8), 1e-3),
    (configs.CFG5.scaled(name="mlp3_ragged", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=10, D=8), 1e-3),
]


@pytest.mark.parametrize("cfg,tol", CASES, ids=lambda v: v.name if hasattr(v, "name") else None)
def test_objective_and_accuracy_match_oracle(cfg, tol):
    prob = generators.make_problem(cfg)
    if prob.X is None:
        Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
        prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    sched = generators.make_schedule(cfg)
    o, tr = oracle_run(cfg, prob, sched)
    X, y, th0 = upload(prob)
    eng = Cada.from_config(cfg, X, y, th0)
    first = eng.evaluate().cpu().numpy()            # at theta0, before any step
    eng.run(to_dev(sched.astype(np.int32)), to_dev(tr["mask"]))
    got = eng.evaluate().cpu().numpy()
    again = eng.evaluate().cpu().numpy()
    st = eng.state()
    torch.cuda.synchronize()
    assert int(st["error_flags"].item()) == 0
    want = o.evaluate([cfg.N_m] * cfg.M)
    o0 = type(o)(model=cfg.model, layer_dims=cfg.layer_dims, M=cfg.M, rule=cfg.rule, D=cfg.D, d_max=cfg.d_max, c=cfg.c,
                 alpha=cfg.alpha, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, lam=cfg.lam, theta0=prob.theta0, rows=prob.rows)
    want0 = o0.evaluate([cfg.N_m] * cfg.M)
    print(cfg.name, "theta0:", first, want0, " after K:", got, want)
    assert np.array_equal(got, again), "evaluation is deterministic and leaves the state alone"
    for g, w in ((first, want0), (got, want)):
        assert abs(g[0] - w[0]) <= tol * abs(w[0])
        assert abs(g[1] - w[1]) <= 3.0 / cfg.N_m          # samples whose margin is at rounding level
    # the run continues unharmed after an evaluation
    eng.step(to_dev(sched[0].astype(np.int32)))
    torch.cuda.synchronize()
