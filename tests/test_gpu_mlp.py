"""GPU parity of the MLP path (bf16 MFMA contractions, float32 master iterate) with the
fp64 oracle, through the C ABI.  Tolerances: theta after K steps under mask replay within
2e-2 relative L2 (bf16 contractions); the library's own rule decisions are compared with the
oracle's at every step and the disagreements are counted and bounded."""
import numpy as np
import pytest

from cada_synth import configs, generators

from common import check_protocol, upload, run_library, oracle_run, rel_l2

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2


def _case(cfg):
    prob = generators.make_problem(cfg)
    return prob, upload(prob), generators.make_schedule(cfg)


@pytest.mark.parametrize("cfg", [
    configs.CFG4.scaled(name="mlp2_tiny", layer_dims=(20, 16, 10), M=3, N_m=60, B=6, K=40, D=6, alpha=0.002),
    configs.CFG5.scaled(name="mlp3_tiny", layer_dims=(24, 16, 16, 10), M=3, N_m=60, B=6, K=40, D=6, alpha=0.002),
    configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=30, D=8),
    configs.CFG5.scaled(name="mlp3_ragged", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=30, D=8),
    # more tiles than CUs in every contraction shape: workgroups work through several tiles, the
    # last of them overhanging (1100 = 8 x 128 + 76 columns, 200 = 6 x 32 + 8 contraction indices)
    configs.CFG5.scaled(name="mlp3_many_tiles", layer_dims=(200, 1100, 136, 10), M=40, N_m=200, B=128, K=4, D=8),
    # the loss in the last layer's epilogue at the ends of its class range (32 is the most the path serves, an odd
    # count leaves half a class pair empty) and with a last block of rows that is nearly empty (B = 33)
    configs.CFG4.scaled(name="mlp2_32_classes", layer_dims=(64, 48, 32), M=3, N_m=200, B=33, K=4, D=8),
    configs.CFG4.scaled(name="mlp2_2_classes", layer_dims=(64, 48, 2), M=3, N_m=200, B=40, K=4, D=8),
    configs.CFG4.scaled(name="softmax_3_classes", layer_dims=(50, 3), M=3, N_m=200, B=96, K=4, D=8),
    configs.CFG5.scaled(name="softmax_31_classes_cada1", layer_dims=(50, 31), M=3, N_m=200, B=65, K=4, D=8),
], ids=lambda c: c.name)
def test_first_step_gradients_match_oracle(cfg):
    """Step 0: every worker uploads, so the stored gradients are the fresh gradients at
    theta0 -- a direct check of every contraction and of the parameter layout."""
    prob, dev, sched = _case(cfg)
    o, tr = oracle_run(cfg, prob, sched[:1])
    out = run_library(cfg, dev, sched[:1])
    assert out["error_flags"][0] == 0 and out["trace_mask"].all()
    errs = [rel_l2(out["stored"][m], o.G[m]) for m in range(cfg.M)]
    print(cfg.name, "per-worker gradient rel L2:", ["%.2e" % e for e in errs])
    # bf16 inputs (relative rounding 2^-9 per element) and, on the tiny cases, single ReLU
    # units whose pre-activation changes sign under that rounding
    assert max(errs) < 5e-2 and float(np.median(errs)) < 2e-2, errs
    # per-layer check so that a layout slip in one block of the vector cannot hide
    off = 0
    d = cfg.layer_dims
    for l in range(len(d) - 1):
        for n in (d[l] * d[l + 1], d[l + 1]):
            e = rel_l2(out["stored"][:, off:off + n], o.G[:, off:off + n])
            print("  layer", l, "block of", n, "rel L2 %.2e" % e)
            assert e < 5e-2, (l, n, e)
            off += n
    assert rel_l2(out["theta64"], o.theta) < 1e-3


# c is set per case so that rule-driven uploads and skips mix (with the workloads' c = 0.5
# these reduced shapes upload almost always).  K stays short on the 3-layer cases: a ReLU
# network's trajectory is piecewise smooth, and once two runs differ by ~1e-6 single
# (unit, sample) pre-activations start to fall on different sides of zero, which kicks the
# runs apart at a rate no finite-precision implementation can avoid (the fp64 oracle started
# from an iterate perturbed by 1e-5 relative drifts by 1.7e-2 in 50 steps on mlp3_ragged).
@pytest.mark.parametrize("cfg", [
    configs.CFG4.scaled(name="mlp2_tiny", layer_dims=(20, 16, 10), M=3, N_m=60, B=6, K=60, D=6, alpha=0.002),
    configs.CFG5.scaled(name="mlp3_tiny", layer_dims=(24, 16, 16, 10), M=3, N_m=60, B=6, K=60, D=6, alpha=0.002),
    configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=50, D=8, c=20.0),
    configs.CFG5.scaled(name="mlp3_ragged", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=30, D=8, c=2.0),
    configs.CFG4.scaled(name="mlp2_cada1", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=50, D=8, c=20.0, rule=configs.RULE_CADA1),
    configs.CFG5.scaled(name="mlp3_cada2", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=30, D=8, c=2.0, rule=configs.RULE_CADA2),
    configs.CFG5.scaled(name="mlp2_32_classes_cada1", layer_dims=(64, 48, 32), M=4, N_m=200, B=33, K=30, D=8, c=5.0),
], ids=lambda c: c.name)
def test_reduced_protocol(cfg):
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, BF16_TOL, lhs_rtol=None, own_mask_exact=False, free_margin=None)
    big = tr["lhs"] > 1e-9 * tr["lhs"].max()
    rel = np.abs(rep["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big]
    stats["lhs_rel_median"], stats["lhs_rel_p99"] = float(np.median(rel)), float(np.quantile(rel, 0.99))
    print(cfg.name, stats)
    w = np.argsort(-rel)[:5]
    print("  worst LHS rel errors", rel[w], "lhs", tr["lhs"][big][w], "gpu", rep["trace_lhs"][big][w])
    free = tr["tau"] < cfg.D
    assert 0.02 < tr["mask"][free].mean() < 0.98, "the case must mix rule-driven uploads and skips"
    # the delta-form left-hand side keeps bf16-level relative accuracy
    assert stats["lhs_rel_median"] < 1e-2 and stats["lhs_rel_p99"] < 0.2
    assert stats["own_disagreements"] <= max(2, 0.03 * tr["mask"].size)


@pytest.mark.parametrize("cfg", [
    configs.CFG5.scaled(name="mlp3_many_tiles_cada1", layer_dims=(200, 1100, 136, 10), M=40, N_m=200, B=128, K=6, D=4, c=50.0),
    configs.CFG5.scaled(name="mlp3_many_tiles_cada2", layer_dims=(200, 1100, 136, 10), M=40, N_m=200, B=128, K=6, D=4, c=50.0,
                        rule=configs.RULE_CADA2),
], ids=lambda c: c.name)
def test_many_tiles_per_workgroup(cfg):
    """Several tiles per workgroup in every contraction shape, over steps with stored innovations
    (CADA1) and per-worker reference points (CADA2), a snapshot refresh and forced uploads."""
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, BF16_TOL, lhs_rtol=None, own_mask_exact=False, free_margin=None)
    big = tr["lhs"] > 1e-9 * tr["lhs"].max()
    rel = np.abs(rep["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big]
    print(cfg.name, stats, "lhs rel median %.2e max %.2e" % (float(np.median(rel)), float(rel.max())))
    assert float(np.median(rel)) < 1e-2 and float(np.quantile(rel, 0.99)) < 0.2
    assert stats["own_disagreements"] <= max(2, 0.03 * tr["mask"].size)


@pytest.mark.parametrize("rule", [configs.RULE_CADA1, configs.RULE_CADA2], ids=["cada1", "cada2"])
def test_out_of_range_sample_is_clamped_and_flagged(rule):
    """A sample id past the worker's shard is clamped to its last row and reported; runs repeat bit for bit."""
    cfg = configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=6, D=3, c=20.0, rule=rule)
    prob, dev, sched = _case(cfg)
    bad = sched.copy(); bad[2, 3, 69] = cfg.N_m + 7; bad[4, 0, 0] = -3
    out = run_library(cfg, dev, bad)
    assert out["error_flags"][0] & 1
    fixed = bad.copy(); fixed[2, 3, 69] = cfg.N_m - 1; fixed[4, 0, 0] = 0
    ref = run_library(cfg, dev, fixed)
    assert not ref["error_flags"][0] & 1
    for key in ("theta", "h", "vhat", "trace_mask", "trace_lhs", "trace_rhs"):
        assert np.array_equal(out[key], ref[key]), key


def test_more_workers_than_a_wavefront_share_reference_points():
    """CADA2 with 70 workers: the search for the first worker with the same delay runs over more
    than one wavefront's worth of workers, and most reference points are shared."""
    cfg = configs.CFG4.scaled(name="mlp2_70_workers", layer_dims=(20, 16, 10), M=70, N_m=40, B=6, K=14, D=4, c=20.0,
                              alpha=0.002, rule=configs.RULE_CADA2)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, BF16_TOL, lhs_rtol=None, own_mask_exact=False, free_margin=None)
    print(cfg.name, stats)
    free = tr["tau"] < cfg.D
    assert 0.02 < tr["mask"][free].mean() < 0.98, "the case must mix rule-driven uploads and skips"
    assert stats["own_disagreements"] <= max(2, 0.03 * tr["mask"].size)


def test_reference_point_far_from_the_iterate():
    """Large steps and a rule that never fires: each worker's reference point ages until the forced
    upload, so the logits at the iterate and at the reference point differ by tens -- the softmax
    difference must stay finite and accurate there (its small-difference form cancels)."""
    cfg = configs.CFG4.scaled(name="mlp2_far", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=26, D=12, c=1e9, alpha=0.02)
    prob, dev, sched = _case(cfg)
    o, tr = oracle_run(cfg, prob, sched)
    from oracle.cada_oracle import mlp_logits
    # the premise: some logits move by more than 10 between an iterate and a 12-step old one
    out = run_library(cfg, dev, sched, replay=tr["mask"])
    assert out["error_flags"][0] == 0
    assert np.isfinite(out["trace_lhs"]).all()
    assert tr["lhs"].max() > 1e2 * np.median(tr["lhs"][1]), "the case must reach large differences"
    big = tr["lhs"] > 1e-9 * tr["lhs"].max()
    rel = np.abs(out["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big]
    print(cfg.name, "lhs rel median %.2e max %.2e" % (np.median(rel), rel.max()), "theta", rel_l2(out["theta64"], o.theta))
    assert np.median(rel) < 1e-2 and rel.max() < 0.2
    assert np.array_equal(out["trace_own_mask"], tr["own_mask"])
    assert rel_l2(out["theta64"], o.theta) < BF16_TOL
