"""GPU parity of the rule variants that share the kernels of Algorithm 1: always-upload
(the distributed Adam/AMSGrad baseline of Section 4) and stochastic LAG (condition (LAGrule),
Section 2.1) with the SGD update it is stated for and with the server update of
(CADA-1)-(CADA-3); logistic model (both gradient paths) and MLP."""
import numpy as np
import pytest

from cada_synth import configs, generators

from paper_2012_15469_amd.binding import PATH_TWO_PASS, PATH_SINGLE_PASS, PATH_WHOLE_STEPS

from common import check_protocol, upload

pytestmark = pytest.mark.gpu
FP32_TOL = 1e-5


def _case(cfg):
    prob = generators.make_problem(cfg)
    return prob, upload(prob), generators.make_schedule(cfg)


@pytest.mark.parametrize("rule,server,c,alpha", [
    (configs.RULE_ALWAYS, configs.SERVER_AMSGRAD, 0.5, 0.005),
    (configs.RULE_LAG, configs.SERVER_SGD, 2000.0, 0.1),
    (configs.RULE_LAG, configs.SERVER_AMSGRAD, 200.0, 0.005),
])
def test_logistic_small(rule, server, c, alpha):
    cfg = configs.CFG1.scaled(rule=rule, server=server, c=c, alpha=alpha, K=120, D=20)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4)
    print(rule, server, stats)
    free = tr["tau"] < cfg.D
    if rule == configs.RULE_ALWAYS:
        assert tr["mask"].all() and o.uploads_total == cfg.M * cfg.K
    else:
        assert 0.05 < tr["mask"][free].mean() < 0.95, "the case must mix rule-driven uploads and skips"


@pytest.mark.parametrize("rule,server,c", [(configs.RULE_LAG, configs.SERVER_SGD, 3e4), (configs.RULE_ALWAYS, configs.SERVER_AMSGRAD, 0.3)])
def test_logistic_single_pass_kernel(rule, server, c):
    cfg = configs.CFG3.scaled(layer_dims=(8200,), M=5, N_m=256, B=72, K=30, D=10, rule=rule, server=server, alpha=0.02, c=c)
    prob = generators.make_problem(cfg)
    Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
    prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    sched = generators.make_schedule(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, upload(prob), sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_SINGLE_PASS,
                                       single_pass_clusters=2, expect_phase="logreg_single_pass")
    print(rule, server, stats, tr["mask"].mean())


@pytest.mark.parametrize("rule,server,c,alpha", [
    (configs.RULE_ALWAYS, configs.SERVER_AMSGRAD, 0.5, 0.0005),
    (configs.RULE_LAG, configs.SERVER_SGD, 500.0, 0.05),
])
def test_mlp_reduced(rule, server, c, alpha):
    cfg = configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=40, D=8,
                              rule=rule, server=server, c=c, alpha=alpha)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, 2e-2, lhs_rtol=None, own_mask_exact=False, free_margin=None)
    big = tr["lhs"] > 1e-9 * tr["lhs"].max()
    rel = np.abs(rep["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big]
    print(rule, server, stats, "lhs rel median %.2e" % np.median(rel), "mask mean", tr["mask"].mean())
    assert np.median(rel) < 1e-3
    assert stats["own_disagreements"] <= max(2, 0.03 * tr["mask"].size)


@pytest.mark.parametrize("small", [1, 0])
def test_decaying_stepsize(small):
    """alpha_k = alpha K0/(k+K0), Theorem 2."""
    cfg = configs.CFG1.scaled(alpha=0.05, alpha_K0=15, K=120, D=20, c=0.5)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_WHOLE_STEPS if small else PATH_TWO_PASS)
    print(small, stats)
    free = tr["tau"] < cfg.D
    assert 0.05 < tr["mask"][free].mean() < 0.95


def test_softmax_regression_is_a_one_layer_network():
    """Multi-class logistic regression (supplement, experiment settings) = the MLP path with a
    single weight layer: one forward contraction, the loss, one weight-gradient contraction."""
    cfg = configs.CFG4.scaled(name="softmax_reg", layer_dims=(150, 10), M=5, N_m=300, B=70, K=40, D=8, c=5.0, alpha=0.002)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, 2e-2, lhs_rtol=None, own_mask_exact=False, free_margin=None)
    big = tr["lhs"] > 1e-9 * tr["lhs"].max()
    rel = np.abs(rep["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big]
    print(stats, "lhs rel median %.2e" % np.median(rel), "mask mean", tr["mask"].mean())
    assert np.median(rel) < 1e-2 and stats["theta_rel_l2"] < 1e-4
    assert stats["own_disagreements"] <= max(2, 0.03 * tr["mask"].size)


def test_uneven_samples_per_worker():
    """Workers own different numbers of samples (supplement: the data are split unevenly)."""
    import torch
    from oracle.cada_oracle import CadaOracle
    from paper_2012_15469_amd.binding import Cada
    from common import to_dev
    cfg = configs.CFG1.scaled(K=60, D=10)
    prob = generators.make_problem(cfg)
    n = np.array([37, 1000, 12, 400, 999, 64, 10, 250, 500, 77])[:cfg.M]          # B = 10 <= every N_m
    off = np.concatenate([[0], np.cumsum(n)])
    X = np.concatenate([prob.X[m * cfg.N_m: m * cfg.N_m + n[m]] for m in range(cfg.M)])
    y = np.concatenate([prob.y[m * cfg.N_m: m * cfg.N_m + n[m]] for m in range(cfg.M)])
    rows = lambda m, loc: (X[off[m] + np.asarray(loc)], y[off[m] + np.asarray(loc)])
    rng = np.random.default_rng(3)
    sched = np.stack([np.stack([rng.choice(n[m], size=cfg.B, replace=False) for m in range(cfg.M)]) for _ in range(cfg.K)]).astype(np.int32)
    o = CadaOracle(model=cfg.model, layer_dims=cfg.layer_dims, M=cfg.M, rule=cfg.rule, D=cfg.D, d_max=cfg.d_max, c=cfg.c,
                   alpha=cfg.alpha, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, lam=cfg.lam, theta0=prob.theta0, rows=rows)
    o.run(sched)
    tr = o.trace_arrays()
    for path in (PATH_WHOLE_STEPS, PATH_TWO_PASS):
        eng = Cada(model=cfg.model, layer_dims=cfg.layer_dims, M=cfg.M, B=cfg.B, n_samples=list(n), X=to_dev(X), y=to_dev(y),
                   theta0=to_dev(prob.theta0), rule=cfg.rule, D=cfg.D, d_max=cfg.d_max, c=cfg.c, alpha=cfg.alpha,
                   beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, lam=cfg.lam, trace_steps=cfg.K, path=path)
        eng.run(to_dev(sched))
        ev = eng.evaluate().cpu().numpy()
        st = eng.state()
        torch.cuda.synchronize()
        assert int(st["error_flags"].item()) == 0
        assert np.array_equal(st["trace_mask"].cpu().numpy(), tr["mask"])
        th = st["theta"].cpu().numpy().astype(np.float64) + st["theta_lo"].cpu().numpy().astype(np.float64)
        assert np.linalg.norm(th - o.theta) / np.linalg.norm(o.theta) < 1e-5
        want = o.evaluate(n)
        assert abs(ev[0] - want[0]) < 1e-5 * want[0] and abs(ev[1] - want[1]) < 2e-3
