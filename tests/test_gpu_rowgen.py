"""The device row generator reproduces the host definition bit for bit."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators, native, philox

pytestmark = pytest.mark.gpu


def test_device_rows_equal_host_rows():
    cfg = configs.CFG3.scaled(layer_dims=(4096,), M=3, N_m=70, B=8)
    prob = generators.make_problem(cfg)
    X = torch.empty((cfg.M * cfg.N_m, cfg.p), dtype=torch.float32, device="cuda")
    y = torch.empty(cfg.M * cfg.N_m, dtype=torch.float32, device="cuda")
    native.fill_device(cfg, torch.from_numpy(prob.shift).cuda(), X, y, rows_per_call=64)
    torch.cuda.synchronize()
    Xh, yh = X.cpu().numpy(), y.cpu().numpy()
    for m in range(cfg.M):
        Xc, yc = native.rows_cpu(cfg.seed, m, np.arange(cfg.N_m), cfg.p, prob.shift[m])
        assert np.array_equal(Xh[m * cfg.N_m:(m + 1) * cfg.N_m], Xc)
        assert np.array_equal(yh[m * cfg.N_m:(m + 1) * cfg.N_m], yc)
    Xn, yn = philox.counter_rows(cfg.seed, 2, np.array([0, 69]), cfg.p, prob.shift[2])
    assert np.array_equal(Xh[[2 * cfg.N_m, 2 * cfg.N_m + 69]], Xn) and np.array_equal(yh[[2 * cfg.N_m, 2 * cfg.N_m + 69]], yn)
