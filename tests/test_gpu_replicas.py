"""Independent runs advanced together in one launch (cada_run_replicas): every replica must end
exactly where it ends when run alone, and agree with the fp64 oracle like a single run does."""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators

from common import upload, to_dev, oracle_run, rel_l2

pytestmark = pytest.mark.gpu


def _replicas(base, n):
    out = []
    for r in range(n):
        cfg = base.scaled(name="%s_r%d" % (base.name, r), seed=base.seed + 17 * r)
        prob = generators.make_problem(cfg)
        out.append((cfg, prob, upload(prob), generators.make_schedule(cfg)))
    return out


def _state(eng):
    torch.cuda.synchronize()
    st = eng.state()
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy().copy() if isinstance(v, torch.Tensor) else v) for k, v in st.items()}


@pytest.mark.parametrize("base,n", [
    (configs.CFG1.scaled(name="rep_cada2", K=60), 5),
    (configs.CFG2.scaled(name="rep_cada1", M=6, N_m=400, B=16, K=40, layer_dims=(200,)), 4),
], ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_replicas_equal_single_runs_and_oracle(base, n):
    from paper_2012_15469_amd.binding import Cada
    reps = _replicas(base, n)
    K = base.K
    engines = [Cada.from_config(cfg, *dev, trace_steps=K, whole_steps=True) for cfg, _, dev, _ in reps]
    scheds = [to_dev(s.astype(np.int32)) for _, _, _, s in reps]
    # two calls, so that a launch continues from the state the previous one left
    k1 = K // 3
    Cada.run_replicas(engines, [s[:k1].contiguous() for s in scheds])
    Cada.run_replicas(engines, [s[k1:].contiguous() for s in scheds])
    together = [_state(e) for e in engines]
    for (cfg, prob, dev, sched), st, idx in zip(reps, together, scheds):
        assert st["error_flags"][0] == 0 and st["k"] == K
        alone = Cada.from_config(cfg, *dev, trace_steps=K, whole_steps=True)
        alone.run(idx)
        ref = _state(alone)
        alone.close()
        for key in ("theta", "theta_lo", "h", "vhat", "tau", "ring", "trace_mask", "trace_lhs", "trace_rhs"):
            assert np.array_equal(st[key], ref[key]), (cfg.name, key)
        o, tr = oracle_run(cfg, prob, sched)
        assert np.array_equal(st["trace_mask"], tr["mask"]), cfg.name
        th = st["theta"].astype(np.float64) + st["theta_lo"].astype(np.float64)
        err = rel_l2(th, o.theta)
        print(cfg.name, "uploads %.2f" % tr["mask"].mean(), "theta rel L2 %.2e" % err)
        assert err < 1e-5
    for e in engines:
        e.close()


def test_replica_arguments_are_checked():
    from paper_2012_15469_amd import binding
    from paper_2012_15469_amd.binding import Cada
    (cfg, prob, dev, sched), = _replicas(configs.CFG1.scaled(name="rep_args", K=4), 1)
    idx = to_dev(sched.astype(np.int32))
    whole = Cada.from_config(cfg, *dev, whole_steps=True)
    with pytest.raises(binding.CadaError, match="twice"):
        Cada.run_replicas([whole, whole], [idx, idx])
    other = Cada.from_config(cfg.scaled(B=cfg.B + 1), *dev, whole_steps=True)
    with pytest.raises(binding.CadaError, match="differs"):
        binding.cada_run_replicas([whole.ctx, other.ctx], [idx.data_ptr(), idx.data_ptr()], None, 1)
    plain = Cada.from_config(configs.CFG2.scaled(name="rep_plain", M=6, N_m=400, B=16, K=4), *upload(
        generators.make_problem(configs.CFG2.scaled(name="rep_plain", M=6, N_m=400, B=16, K=4))), path=binding.PATH_TWO_PASS)
    with pytest.raises(binding.CadaError, match="WHOLE_STEPS"):
        binding.cada_run_replicas([plain.ctx], [idx.data_ptr()], None, 1)
    plain.close()
    whole.close(); other.close()
