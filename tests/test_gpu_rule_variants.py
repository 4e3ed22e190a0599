"""GPU parity of the rule variants that share the kernels of Algorithm 1: always-upload
(the distributed Adam/AMSGrad baseline of Section 4) and stochastic LAG (condition (LAGrule),
Section 2.1) with the SGD update it is stated for and with the server update of
(CADA-1)-(CADA-3); logistic model (both gradient paths) and MLP."""
import numpy as np
import pytest

from cada_synth import configs, generators

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
def test_logistic_single_pass_kernel(rule, server, c, monkeypatch):
    monkeypatch.setenv("CADA_FUSED", "1")
    monkeypatch.setenv("CADA_FUSED_CLUSTERS", "2")
    cfg = configs.CFG3.scaled(layer_dims=(8200,), M=5, N_m=256, B=72, K=30, D=10, rule=rule, server=server, alpha=0.02, c=c)
    prob = generators.make_problem(cfg)
    Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
    prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    sched = generators.make_schedule(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, upload(prob), sched, FP32_TOL, lhs_rtol=1e-4)
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
