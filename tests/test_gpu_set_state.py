"""cada_set_state through the C ABI: the library picks up the oracle's state in the middle of a
run (iterate, moments, stored gradients, reference points, stored innovations, delays, squared
steps) and continues on the oracle's trajectory -- decisions, delays, left- and right-hand sides
and iterates of the following steps agree with the oracle that never stopped."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators
from oracle.cada_oracle import margins
from oracle.driver import oracle_for
from paper_2012_15469_amd.binding import Cada, CadaError, PATH_TWO_PASS, PATH_WHOLE_STEPS

from common import upload, to_dev, inject_oracle_state, library_state, rel_l2, MARGIN

pytestmark = pytest.mark.gpu

CASES = [
    (configs.CFG1.scaled(K=90, D=12), 37, 1e-4, {}),                                     # whole iterations in one launch, CADA2
    (configs.CFG1.scaled(name="cfg1_cada1", K=90, D=12, rule=configs.RULE_CADA1), 37, 1e-4, {}),
    (configs.CFG2.scaled(K=70, N_m=300, D=20), 33, 1e-4, {"path": PATH_TWO_PASS}),       # two streaming passes, CADA1
    (configs.CFG2.scaled(name="cfg2_cada2", K=70, N_m=300, D=20, rule=configs.RULE_CADA2, c=0.05), 45, 1e-4, {}),
    (configs.CFG3.scaled(name="fused_cada2", layer_dims=(8192,), M=5, N_m=128, B=32, K=30, D=6, alpha=0.02, c=1e-4), 13, 1e-4, {}),
    (configs.CFG4.scaled(name="mlp2_cada2", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=40, D=8, c=20.0), 19, 2e-2, {}),
    (configs.CFG5.scaled(name="mlp3_cada1", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=30, D=8, c=2.0), 17, 2e-2, {}),
]


def _rows(prob, cfg):
    if prob.X is None:
        Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
        prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    return prob


@pytest.mark.parametrize("cfg,K1,tol,kw", CASES, ids=lambda v: getattr(v, "name", None))
def test_continue_from_oracle_state(cfg, K1, tol, kw):
    prob = _rows(generators.make_problem(cfg), cfg)
    dev = upload(prob)
    sched = generators.make_schedule(cfg)
    K = cfg.K
    o = oracle_for(cfg, prob)
    o.run(sched[:K1])
    eng = Cada.from_config(cfg, *dev, trace_steps=K, **kw)
    inject_oracle_state(eng, o)
    assert eng.k == K1
    o.run(sched[K1:])
    tr = o.trace_arrays()
    mg = margins(tr["lhs"], tr["rhs"])
    eng.run(to_dev(sched[K1:].astype(np.int32)), to_dev(tr["mask"][K1:]))
    st = library_state(eng)
    assert st["k"] == K and st["error_flags"][0] == 0
    assert np.array_equal(st["trace_mask"][K1:], tr["mask"][K1:])
    assert np.array_equal(st["trace_tau"][K1:], tr["tau"][K1:])
    assert np.array_equal(st["tau"], o.tau) and st["uploads_total"][0] == o.uploads_total
    own_diff = st["trace_own_mask"][K1:] != tr["own_mask"][K1:]
    free = tr["tau"][K1:] < cfg.D
    assert 0.02 < tr["mask"][K1:][free].mean() < 0.98, "rule-driven uploads and skips must mix after the hand-over"
    err = rel_l2(st["theta64"], o.theta)
    big = tr["lhs"][K1:] > 1e-9 * tr["lhs"].max()
    rel = (np.abs(st["trace_lhs"][K1:] - tr["lhs"][K1:]) / np.maximum(tr["lhs"][K1:], 1e-300))[big]
    print(cfg.name, "theta %.2e  lhs rel median %.2e max %.2e  own-rule disagreements %d" % (err, np.median(rel), rel.max(), own_diff.sum()))
    assert err <= tol
    if tol <= 1e-4:       # float32 arithmetic: decisions may differ only within the margin, LHS/RHS to 1e-4
        assert not (own_diff & (mg[K1:] > MARGIN)).any()
        assert rel.max() <= 1e-4
        np.testing.assert_allclose(st["trace_rhs"][K1:], tr["rhs"][K1:], rtol=1e-4)
        assert rel_l2(st["h"], o.h) < 1e-4 and rel_l2(st["vhat"], o.vhat) < 1e-4
    else:
        assert np.median(rel) < 1e-2
        np.testing.assert_allclose(st["trace_rhs"][K1:], tr["rhs"][K1:], rtol=2e-2)
    np.testing.assert_allclose(st["ring"], o.ring, rtol=max(tol, 1e-4))
    eng.close()


def test_set_state_argument_errors():
    cfg = configs.CFG1.scaled(K=4)
    prob = generators.make_problem(cfg)
    dev = upload(prob)
    eng = Cada.from_config(cfg, *dev)
    o = oracle_for(cfg, prob)
    o.run(generators.make_schedule(cfg)[:3])
    z = torch.zeros(cfg.p, device="cuda")
    G = torch.zeros(cfg.M, cfg.p, device="cuda")
    tau = torch.ones(cfg.M, dtype=torch.int32, device="cuda")
    ring = torch.zeros(cfg.d_max, device="cuda")
    with pytest.raises(CadaError, match="reference"):
        eng.set_state(k=3, theta=z, h=z, vhat=z, stored_gradients=G, tau=tau, ring=ring)
    with pytest.raises(CadaError, match="k must be"):
        eng.set_state(k=-1, theta=z, h=z, vhat=z, stored_gradients=G, tau=tau, ring=ring, reference=G)
    assert eng.k == 0
    # a delay outside [1, D] is clamped and reported
    tau[2] = cfg.D + 5
    eng.set_state(k=3, theta=z, h=z, vhat=z, stored_gradients=G, tau=tau, ring=ring, reference=G)
    st = library_state(eng)
    assert st["error_flags"][0] & 4 and st["tau"][2] == cfg.D and st["k"] == 3
    eng.close()


def test_replay_beyond_the_retained_iterates_is_flagged():
    """A replay mask that keeps a CADA2 worker silent for more than D iterations asks for an iterate
    that is no longer retained: error bit 3, no fault."""
    cfg = configs.CFG1.scaled(K=8, D=3)
    prob = generators.make_problem(cfg)
    dev = upload(prob)
    sched = generators.make_schedule(cfg)
    replay = np.zeros((cfg.K, cfg.M), dtype=np.uint8)
    replay[0] = 1
    for path in (PATH_TWO_PASS, PATH_WHOLE_STEPS):
        eng = Cada.from_config(cfg, *dev, trace_steps=cfg.K, path=path)
        eng.run(to_dev(sched[:3].astype(np.int32)), to_dev(replay[:3]))
        assert library_state(eng)["error_flags"][0] == 0
        eng.run(to_dev(sched[3:].astype(np.int32)), to_dev(replay[3:]))
        assert library_state(eng)["error_flags"][0] & 8
        eng.close()
