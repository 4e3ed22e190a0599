"""The high-dimensional logistic workload at its full size (M=100, p=65536, B=256, 4096
samples per worker: 107 GB of features generated in HBM), in the launch configuration
bench.py times, against stored oracle results written by tests/golden/make_goldens.py."""
import os

import numpy as np
import pytest
import torch

from cada_synth import configs, generators, native

from common import run_library, to_dev

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def full_dataset():
    cfg = configs.CFG3
    free, _ = torch.cuda.mem_get_info()
    need = cfg.M * cfg.N_m * cfg.p * 4
    if free < need + (8 << 30):
        pytest.skip("needs %.0f GB of free HBM" % (need / 1e9))
    prob = generators.make_problem(cfg)
    X = torch.empty((cfg.M * cfg.N_m, cfg.p), dtype=torch.float32, device="cuda")
    y = torch.empty(cfg.M * cfg.N_m, dtype=torch.float32, device="cuda")
    native.fill_device(cfg, to_dev(prob.shift), X, y)
    torch.cuda.synchronize()
    yield cfg, prob, (X, y, to_dev(prob.theta0))
    del X, y
    torch.cuda.empty_cache()


def test_device_dataset_matches_host_rows(full_dataset):
    cfg, prob, (X, y, _) = full_dataset
    rng = np.random.default_rng(5)
    for m in (0, 37, 99):
        rows = np.sort(rng.choice(cfg.N_m, size=6, replace=False))
        Xc, yc = native.rows_cpu(cfg.seed, m, rows, cfg.p, prob.shift[m])
        g = torch.from_numpy(m * cfg.N_m + rows).cuda()
        assert np.array_equal(X[g].cpu().numpy(), Xc) and np.array_equal(y[g].cpu().numpy(), yc)
    assert 0.4 < float((y > 0).float().mean()) < 0.6


@pytest.mark.parametrize("name,c", [("cfg3_full_c0.3", 0.3), ("cfg3_full_c1e-4", 1e-4)])
def test_full_size_steps_match_stored_oracle(full_dataset, name, c):
    from tests_golden_fingerprint import fingerprint
    cfg, prob, dev = full_dataset
    cfg = cfg.scaled(c=c)
    path = os.path.join(GOLD, name + ".npz")
    g = np.load(path)
    K = int(g["K"])
    sched = generators.make_schedule(cfg, K)
    assert fingerprint(cfg, prob, sched) == int(g["fingerprint"]), "stored oracle results are stale: rerun make_goldens.py"
    out = run_library(cfg, dev, sched)
    margin = np.abs(g["lhs"] - g["rhs"][:, None]) / np.maximum(g["rhs"][:, None], 1e-300)
    diff = out["trace_mask"] != g["mask"]
    assert not (diff & (margin > 1e-5)).any(), np.argwhere(diff)[:5]
    if not diff.any():      # same decisions, so the trajectories are comparable to the end
        stride = int(g["theta_stride"])
        th = out["theta64"][::stride]
        err = np.linalg.norm(th - g["theta"]) / np.linalg.norm(g["theta"])
        assert err <= 1e-4, err
        assert abs(np.linalg.norm(out["theta64"]) / float(g["theta_norm"]) - 1) < 1e-5
        assert abs(np.linalg.norm(out["h"].astype(np.float64)) / float(g["h_norm"]) - 1) < 1e-5
        assert abs(np.linalg.norm(out["vhat"].astype(np.float64)) / float(g["vhat_norm"]) - 1) < 1e-5
        assert np.array_equal(out["tau"], g["tau_final"]) and out["uploads_total"][0] == int(g["uploads_total"])
        big = g["lhs"] > 0
        rel = np.abs(out["trace_lhs"] - g["lhs"])[big] / g["lhs"][big]
        assert rel.max() <= 1e-4, rel.max()
        np.testing.assert_allclose(out["trace_rhs"], g["rhs"], rtol=1e-5)
        np.testing.assert_allclose(out["ring"], g["ring"], rtol=1e-5)
    if name.endswith("1e-4"):
        free = g["tau"] < cfg.D
        assert 0.05 < g["mask"][free].mean() < 0.95, "rule decisions must mix"
