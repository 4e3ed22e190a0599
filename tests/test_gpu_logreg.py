"""GPU parity of the logistic path with the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators

from paper_2012_15469_amd.binding import PATH_TWO_PASS, PATH_SINGLE_PASS, PATH_WHOLE_STEPS

from common import check_protocol, upload, run_library, oracle_run, rel_l2

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4      # theta relative L2 after K steps (float32 path)


def _case(cfg):
    prob = generators.make_problem(cfg)
    return prob, upload(prob), generators.make_schedule(cfg)


# small: 1 = whole iterations in one launch (cada_logreg_small.hip), 0 = one launch per kernel
@pytest.mark.parametrize("small", [1, 0])
def test_cfg1_full(small):
    cfg = configs.CFG1
    prob, dev, sched = _case(cfg)
    stats, *_ = check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_WHOLE_STEPS if small else PATH_TWO_PASS)
    print("cfg1", stats)
    assert stats["h_rel_l2"] < 1e-4 and stats["vhat_rel_l2"] < 1e-4 and stats["ring_rel"] < 1e-4
    assert stats["stored_rel_l2"] < 1e-5


@pytest.mark.parametrize("small", [1, 0])
def test_cfg2_full(small):
    cfg = configs.CFG2
    prob, dev, sched = _case(cfg)
    stats, *_ = check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_WHOLE_STEPS if small else PATH_TWO_PASS)
    print("cfg2", stats)
    assert stats["stored_rel_l2"] < 1e-5


@pytest.mark.parametrize("p,rule,fused", [(8200, 2, 0), (8200, 1, 0), (4099, 2, 0), (4099, 1, 0), (8200, 2, 1), (8200, 1, 1),
                                          (1027, 2, -1), (1027, 1, -1)])
def test_cfg3_reduced_ragged(p, rule, fused):
    """The high-dimensional recipe at reduced size: several column chunks with a ragged
    tail (p = 8200 = 8192 + 8), a row count that is no multiple of the row group (B = 20)
    and the scalar-load path (p = 4099 is not a multiple of 4)."""
    # fused 1: the single-pass register-resident kernel; 0: the two streaming passes;
    # -1: the multi-step kernel for small problems (a worker's minibatch must fit in LDS: p = 1027)
    path = {1: PATH_SINGLE_PASS, 0: PATH_TWO_PASS, -1: PATH_WHOLE_STEPS}[fused]
    # c is lowered from the workload's 0.3: a minibatch spans only B of the p directions, so
    # with c = 0.3 the rule never fires at this size and only forced uploads would be tested
    cfg = configs.CFG3.scaled(layer_dims=(p,), M=5, N_m=64, B=20, K=60, D=10, rule=rule, alpha=0.02, c=1e-4)
    prob = generators.make_problem(cfg)
    if p % 2:   # the counter recipe needs an even p: fall back to host-generated Gaussians
        cfg = cfg.scaled(data="gauss_shifted")
        prob = generators.make_problem(cfg)
        prob.X *= np.float32(1.0 / np.sqrt(p))
    else:
        Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
        prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    sched = generators.make_schedule(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, upload(prob), sched, FP32_TOL, lhs_rtol=1e-4, path=path,
                                       expect_phase={1: "logreg_single_pass", 0: "logreg_two_pass", -1: "logreg_whole_steps"}[fused])
    print(p, rule, stats)
    free = tr["tau"] < cfg.D
    assert 0.1 < tr["mask"][free].mean() < 0.9, "the case must mix rule-driven uploads and skips"


# even B: two rows per iteration; odd B: one row per iteration
# B = 32, 33: the shortest minibatches of the variant that changes worker without waiting for its loads; 30, 31: the longest of the other
@pytest.mark.parametrize("rule,B,clusters", [(2, 48, 0), (1, 48, 0), (2, 100, 2), (1, 72, 2), (2, 200, 1), (2, 51, 0), (1, 75, 2),
                                             (2, 32, 2), (1, 33, 2), (2, 31, 1), (1, 30, 2), (2, 34, 1)])
def test_single_pass_kernel_steady_state(rule, B, clusters):
    """The single-pass kernel's unrolled steady-state loop only runs once a cluster of
    workgroups streams more than 40 rows: longer minibatches, and fewer clusters than workers
    so that a cluster changes worker (reference point, gradient store) in mid-stream."""
    # K = 30: later the left-hand sides are differences of nearly converged iterates, and both
    # logistic paths lose digits there alike (the cancellation, not the kernel, sets the error)
    cfg = configs.CFG3.scaled(layer_dims=(8200,), M=5, N_m=256, B=B, K=30, D=10, rule=rule, alpha=0.02, c=1e-4)
    prob = generators.make_problem(cfg)
    Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
    prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    sched = generators.make_schedule(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, upload(prob), sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_SINGLE_PASS,
                                       single_pass_clusters=clusters, expect_phase="logreg_single_pass")
    print(rule, B, clusters, stats)


@pytest.mark.parametrize("rule,clusters", [(2, 0), (1, 2)])
def test_single_pass_kernel_wide_clusters(rule, clusters):
    """p = 131072: clusters of 64 workgroups, each exchange lane sums two partials per value.  With two
    clusters for three workers a cluster changes worker in mid-stream."""
    cfg = configs.CFG3.scaled(layer_dims=(131072,), M=3, N_m=96, B=48, K=14, D=5, rule=rule, alpha=0.02, c=1e-4)
    prob = generators.make_problem(cfg)
    Xs, ys = zip(*(prob.rows(m, np.arange(cfg.N_m)) for m in range(cfg.M)))
    prob.X, prob.y = np.concatenate(Xs), np.concatenate(ys)
    sched = generators.make_schedule(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, upload(prob), sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_SINGLE_PASS,
                                       single_pass_clusters=clusters, expect_phase="logreg_single_pass")
    print(rule, clusters, stats)
    free = tr["tau"] < cfg.D
    assert 0.02 < tr["mask"][free].mean() < 0.98, "the case must mix rule-driven uploads and skips"


@pytest.mark.parametrize("p,rule", [(54, 2), (64, 1)])
def test_whole_steps_with_more_rows_than_threads(p, rule):
    """The whole-step kernel with a minibatch of 300 rows (more than the 256 threads of a workgroup, and no multiple
    of the rows a wavefront fetches at a time), rows of 16-byte multiples (p = 64) and not (p = 54): the fetch of the
    first step, the prefetch of the following ones and the labels all go through their loops more than once."""
    cfg = configs.CFG1.scaled(name="rows300", layer_dims=(p,), M=3, N_m=1000, B=300, K=40, D=6, rule=rule, c=0.05)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_WHOLE_STEPS, expect_phase="logreg_whole_steps")
    print(p, rule, stats, tr["mask"].mean())


@pytest.mark.parametrize("M,p,rule", [(70, 54, 2), (33, 64, 1), (17, 54, 1)])
def test_whole_steps_with_many_workers(M, p, rule):
    """The whole-step kernel with more workers than a wavefront has lanes (the barrier's words are polled in two
    rounds) and more than the 16 or 32 whose rows the aggregate asks for at a time, on the 16-byte and the scalar path."""
    cfg = configs.CFG1.scaled(name="many%d" % M, layer_dims=(p,), M=M, N_m=80, B=8, K=40, D=6, rule=rule, c=0.05)
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4, path=PATH_WHOLE_STEPS, expect_phase="logreg_whole_steps")
    print(M, p, rule, stats, tr["mask"].mean())
    free = tr["tau"] < cfg.D
    assert 0.02 < tr["mask"][free].mean() < 0.98, "the case must mix rule-driven uploads and skips"


def test_special_cases_c0_and_huge_c():
    cfg = configs.CFG1.scaled(c=0.0, K=50)
    prob, dev, sched = _case(cfg)
    out = run_library(cfg, dev, sched)
    assert out["trace_mask"].all() and out["uploads_total"][0] == cfg.M * cfg.K
    cfg = configs.CFG1.scaled(c=1e30, K=120)
    sched = generators.make_schedule(cfg)
    out = run_library(cfg, dev, sched)
    for k in range(cfg.K):
        assert out["trace_mask"][k].all() == (k % cfg.D == 0) and out["trace_mask"][k].any() == (k % cfg.D == 0)


def test_single_worker_and_single_row():
    cfg = configs.CFG1.scaled(M=1, B=1, N_m=50, K=40, D=5)
    prob, dev, sched = _case(cfg)
    check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4)


def test_duplicate_rows_and_out_of_range_flag():
    cfg = configs.CFG1.scaled(K=8)
    prob, dev, sched = _case(cfg)
    sched[:, :, 1] = sched[:, :, 0]                    # duplicate rows are legal
    check_protocol(cfg, prob, dev, sched, FP32_TOL, lhs_rtol=1e-4)
    bad = sched.copy(); bad[3, 2, 0] = cfg.N_m + 5     # clamped to the last row and flagged
    out = run_library(cfg, dev, bad)
    assert out["error_flags"][0] & 1
    fixed = bad.copy(); fixed[3, 2, 0] = cfg.N_m - 1
    ref = run_library(cfg, dev, fixed)
    assert np.array_equal(out["theta"], ref["theta"])


def test_runs_are_bitwise_reproducible():
    cfg = configs.CFG2.scaled(K=100)
    prob, dev, sched = _case(cfg)
    a = run_library(cfg, dev, sched)
    b = run_library(cfg, dev, sched)
    for key in ("theta", "h", "vhat", "trace_mask", "trace_lhs", "trace_rhs", "ring"):
        assert np.array_equal(a[key], b[key]), key


def test_step_by_step_equals_run():
    from paper_2012_15469_amd.binding import Cada
    from common import to_dev
    cfg = configs.CFG1.scaled(K=30)
    prob, dev, sched = _case(cfg)
    ref = run_library(cfg, dev, sched)
    eng = Cada.from_config(cfg, *dev, trace_steps=cfg.K)
    idx = to_dev(sched)
    for k in range(cfg.K):
        eng.step(idx[k])
        if k == 10:   # reading the state mid-run must not disturb it
            torch.cuda.synchronize(); _ = eng.state()["ring"].cpu()
    torch.cuda.synchronize()
    st = eng.state(); torch.cuda.synchronize()
    assert np.array_equal(st["theta"].cpu().numpy(), ref["theta"])
    assert np.array_equal(st["ring"].cpu().numpy(), ref["ring"])


def test_bad_arguments_are_errors():
    from paper_2012_15469_amd import binding as b
    cfg = configs.CFG1
    prob, dev, sched = _case(cfg)
    with pytest.raises(b.CadaError, match="B must be"):
        b.Cada.from_config(cfg.scaled(B=0), *dev)
    with pytest.raises(b.CadaError, match="rule"):
        b.Cada.from_config(cfg, *dev, rule=7)
    with pytest.raises(b.CadaError, match="d_max"):
        b.Cada.from_config(cfg.scaled(d_max=0), *dev)
    with pytest.raises(b.CadaError, match="does not match"):
        b.Cada.from_config(cfg, dev[0], dev[1], dev[2][:50].contiguous())


def test_largest_minibatch_two_pass():
    """B = 4096, the largest minibatch the interface takes: the second pass keeps 16 bytes per row in
    LDS (64 KB), which needs the kernel's allowance raised."""
    cfg = configs.CFG1.scaled(name="big_batch", layer_dims=(64,), M=2, N_m=4500, B=4096, K=4, D=3, c=1e-3)
    prob, dev, sched = _case(cfg)
    o, tr = oracle_run(cfg, prob, sched)
    out = run_library(cfg, dev, sched, replay=tr["mask"], path=PATH_TWO_PASS, expect_phase="logreg_two_pass")
    assert out["error_flags"][0] == 0
    assert np.array_equal(out["trace_own_mask"], tr["own_mask"])
    assert rel_l2(out["theta64"], o.theta) < FP32_TOL
    big = tr["lhs"] > 0
    assert (np.abs(out["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big]).max() < 1e-4
