"""cada_eval_noalloc, the entry point for callers that cannot allocate: its result equals
cada_eval's bit for bit (same kernels, the scratch in a fixed array inside the library), on two
calls in a row, the second on a smaller problem; sizes beyond its maximum are refused."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators
from paper_2012_15469_amd import binding
from paper_2012_15469_amd.binding import Cada

from common import upload, to_dev

pytestmark = pytest.mark.gpu


def _engine(cfg, steps):
    prob = generators.make_problem(cfg)
    dev = upload(prob)
    eng = Cada.from_config(cfg, *dev)
    eng.run(to_dev(generators.make_schedule(cfg, steps).astype(np.int32)))
    return eng, prob


def test_noalloc_evaluation_equals_cada_eval():
    big, prob_big = _engine(configs.CFG2.scaled(name="eval_big", N_m=700, K=12), 12)
    small, _ = _engine(configs.CFG1.scaled(name="eval_small", M=6, N_m=90, K=7), 7)
    out = torch.empty(2, 2, dtype=torch.float64, device="cuda")
    want = torch.empty(2, 2, dtype=torch.float64, device="cuda")
    for i, eng in enumerate((big, small)):          # the second call reuses the array with a smaller input
        binding.cada_eval(eng.ctx, want[i].data_ptr())
        binding.cada_eval_noalloc(eng.ctx, out[i].data_ptr())
    torch.cuda.synchronize()
    got, ref = out.cpu().numpy(), want.cpu().numpy()
    print("noalloc", got.tolist(), "cada_eval", ref.tolist())
    assert np.array_equal(got, ref)
    assert np.isfinite(got).all() and 0.0 < got[0, 0] < 1.0 and 0.4 < got[0, 1] <= 1.0
    # against the oracle's definition as well (the bar cada_eval itself is held to)
    from oracle.driver import oracle_for
    cfg = configs.CFG2.scaled(name="eval_big", N_m=700, K=12)
    o = oracle_for(cfg, prob_big)
    st = big.state()
    torch.cuda.synchronize()
    o.theta = st["theta"].cpu().numpy().astype(np.float64) + st["theta_lo"].cpu().numpy().astype(np.float64)
    loss, acc = o.evaluate([cfg.N_m] * cfg.M)
    assert abs(got[0, 0] - loss) < 1e-5 * loss and abs(got[0, 1] - acc) < 2e-3
    # once more on the larger problem: what the smaller call left behind does not leak in
    binding.cada_eval_noalloc(big.ctx, out[1].data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(out[1].cpu().numpy(), ref[0])
    big.close(); small.close()


def test_noalloc_refuses_what_exceeds_its_array():
    cfg = configs.CFG1.scaled(name="eval_many", M=binding.EVAL_NOALLOC_MAX_M + 1, N_m=12, B=4, K=2)
    eng, _ = _engine(cfg, 2)
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    with pytest.raises(binding.CadaError, match="at most"):
        binding.cada_eval_noalloc(eng.ctx, out.data_ptr())
    eng.close()
    mlp, _ = _engine(configs.CFG4.scaled(name="eval_mlp", layer_dims=(40, 24, 10), M=4, N_m=100, B=16, K=2, D=6), 2)
    with pytest.raises(binding.CadaError, match="logistic"):
        binding.cada_eval_noalloc(mlp.ctx, out.data_ptr())
    mlp.close()
    torch.cuda.synchronize()
    assert float(out.abs().sum()) == 0.0
