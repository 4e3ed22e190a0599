"""Checkpoint / resume through the C ABI: a run continued from a saved block, in the same
context or in a fresh one, is bitwise the run that was never interrupted."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators
from paper_2012_15469_amd.binding import Cada, CadaError

from common import upload, to_dev

pytestmark = pytest.mark.gpu


def _final(eng):
    torch.cuda.synchronize()
    st = eng.state()
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy().copy() if torch.is_tensor(v) else v) for k, v in st.items()}, eng.stored_gradients().cpu().numpy()


@pytest.mark.parametrize("cfg", [
    configs.CFG1.scaled(K=60),
    configs.CFG2.scaled(K=40, N_m=200),
    configs.CFG4.scaled(name="mlp2_small", layer_dims=(40, 24, 10), M=4, N_m=100, B=16, K=24, D=6),
], ids=lambda c: c.name)
def test_resume_is_bitwise_the_uninterrupted_run(cfg):
    prob = generators.make_problem(cfg)
    X, y, th0 = upload(prob)
    sched = to_dev(generators.make_schedule(cfg).astype(np.int32))
    K, K1 = cfg.K, cfg.K // 3
    ref = Cada.from_config(cfg, X, y, th0, trace_steps=K)
    for k in range(K):
        ref.step(sched[k])
    want, want_g = _final(ref)

    a = Cada.from_config(cfg, X, y, th0, trace_steps=K)
    for k in range(K1):
        a.step(sched[k])
    block = a.checkpoint()
    for k in range(K1, K1 + 5):          # run on, then rewind the same context
        a.step(sched[k])
    a.restore(block)
    assert a.k == K1
    for k in range(K1, K):
        a.step(sched[k])
    b = Cada.from_config(cfg, X, y, th0, trace_steps=K)      # and a fresh context
    b.restore(block)
    for k in range(K1, K):
        b.step(sched[k])
    for eng in (a, b):
        got, got_g = _final(eng)
        assert got["k"] == want["k"] == K
        for name in ("theta", "theta_lo", "h", "vhat", "tau", "ring", "uploads_total", "trace_mask", "trace_lhs"):
            assert np.array_equal(got[name], want[name]), name
        assert np.array_equal(got_g, want_g)


def test_block_of_another_configuration_is_refused():
    cfg = configs.CFG1.scaled(K=4)
    prob = generators.make_problem(cfg)
    X, y, th0 = upload(prob)
    a = Cada.from_config(cfg, X, y, th0)
    block = a.checkpoint()
    # d_max changes a few bytes inside one 256-byte piece of the workspace: same size, other header
    b = Cada.from_config(cfg.scaled(d_max=cfg.d_max - 1), X, y, th0)
    if b.checkpoint().numel() == block.numel():
        with pytest.raises(CadaError):
            b.restore(block)
    with pytest.raises(CadaError):
        a.restore(torch.zeros_like(block))
    a.restore(block)            # a valid block still loads afterwards
