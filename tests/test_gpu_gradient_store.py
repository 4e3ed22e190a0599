"""The bf16 gradient store of the MLP path (CADA_STORE_BF16) through the C ABI.

The server keeps every worker's last uploaded gradient (the terms of the aggregate in (CADA-1), Section 1.2); with
this store each is rounded to bf16 (nearest even) when it is written.  What that must and must not change:
  * the stored value is exactly the rounded float32 gradient, in every block of the parameter vector;
  * the rule's left-hand side, formed from the innovation before anything is rounded, is bit for bit the same;
  * against the fp64 oracle the iterates stay within the tolerance of the bf16 path (2e-2 relative L2 under replay
    of the oracle's decisions), and each stored element is within 2^-8 of the oracle's relative to the row's scale.
"""
import numpy as np
import pytest
import torch

from cada_synth import configs, generators
from oracle.driver import oracle_for
from paper_2012_15469_amd.binding import Cada, CadaError, STORE_BF16

from common import check_protocol, upload, run_library, oracle_run, rel_l2, to_dev, inject_oracle_state, library_state

pytestmark = pytest.mark.gpu
BF16_TOL = 2e-2


def _case(cfg):
    prob = generators.make_problem(cfg)
    return prob, upload(prob), generators.make_schedule(cfg)


def _round_bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


@pytest.mark.parametrize("cfg", [
    # odd row lengths (133): the element-wise store; 10 and 7 classes: the last layer's kernel
    configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=30, D=8),
    configs.CFG5.scaled(name="mlp3_ragged", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=30, D=8),
    # several tiles per workgroup, overhanging tiles, the 8-byte stores of whole wavefront parts
    configs.CFG5.scaled(name="mlp3_many_tiles", layer_dims=(200, 1100, 136, 10), M=40, N_m=200, B=128, K=4, D=8),
    configs.CFG4.scaled(name="mlp2_many_tiles", layer_dims=(200, 1100, 10), M=40, N_m=200, B=128, K=4, D=8),
], ids=lambda c: c.name)
def test_stored_gradient_is_the_rounded_gradient(cfg):
    prob, dev, sched = _case(cfg)
    f32 = run_library(cfg, dev, sched[:1])
    b16 = run_library(cfg, dev, sched[:1], gradient_store=STORE_BF16)
    assert f32["error_flags"][0] == 0 and b16["error_flags"][0] == 0 and b16["trace_mask"].all()
    assert np.array_equal(b16["stored"], _round_bf16(f32["stored"]))
    assert np.array_equal(b16["trace_lhs"], f32["trace_lhs"])
    # the aggregate of step 0 is the mean of the stored rows, whichever store holds them
    # (float32 sums of M terms: accurate relative to the terms' magnitudes, not to a sum that cancels)
    rows = b16["stored"].astype(np.float64)
    assert (np.abs(b16["nabla"] - rows.mean(axis=0)) <= 4e-6 * np.abs(rows).mean(axis=0) + 1e-12).all()
    o, tr = oracle_run(cfg, prob, sched[:1])
    # against the oracle: what the float32 store is off by (the bf16 contractions) plus at most one rounding
    for m in range(cfg.M):
        assert rel_l2(b16["stored"][m], o.G[m]) <= rel_l2(f32["stored"][m], o.G[m]) + 2.0 ** -8
    assert rel_l2(b16["theta64"], o.theta) < 1e-3


@pytest.mark.parametrize("cfg", [
    configs.CFG4.scaled(name="mlp2_ragged", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=50, D=8, c=20.0),
    configs.CFG5.scaled(name="mlp3_ragged", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=30, D=8, c=2.0),
    configs.CFG5.scaled(name="mlp3_many_tiles_cada1", layer_dims=(200, 1100, 136, 10), M=40, N_m=200, B=128, K=6, D=4, c=50.0),
    configs.CFG4.scaled(name="mlp2_always", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=20, D=8, rule=configs.RULE_ALWAYS),
], ids=lambda c: c.name)
def test_reduced_protocol_with_bf16_store(cfg):
    """Free run and replay against the fp64 oracle, forced uploads and (CADA1) snapshot refreshes included."""
    prob, dev, sched = _case(cfg)
    stats, o, tr, rep = check_protocol(cfg, prob, dev, sched, BF16_TOL, lhs_rtol=None, own_mask_exact=False, free_margin=None,
                                       gradient_store=STORE_BF16)
    big = tr["lhs"] > 1e-9 * max(tr["lhs"].max(), 1e-300)
    rel = np.abs(rep["trace_lhs"] - tr["lhs"])[big] / tr["lhs"][big] if big.any() else np.zeros(1)
    print(cfg.name, stats, "lhs rel median %.2e p99 %.2e" % (float(np.median(rel)), float(np.quantile(rel, 0.99))))
    assert float(np.median(rel)) < 1e-2 and float(np.quantile(rel, 0.99)) < 0.2
    assert stats["own_disagreements"] <= max(2, 0.03 * tr["mask"].size)
    assert stats["stored_rel_l2"] < 5e-2
    assert rel_l2(rep["nabla"], o.nabla) < 5e-2


def test_set_state_rounds_and_the_run_continues():
    """Hand-over of the oracle's state in mid-run: the stored gradients come back as their bf16 roundings,
    and the following steps stay on the oracle's trajectory."""
    cfg = configs.CFG4.scaled(name="mlp2_cada2", layer_dims=(150, 133, 10), M=5, N_m=300, B=70, K=40, D=8, c=20.0)
    prob, dev, sched = _case(cfg)
    K1 = 19
    o = oracle_for(cfg, prob)
    o.run(sched[:K1])
    eng = Cada.from_config(cfg, *dev, trace_steps=cfg.K, gradient_store=STORE_BF16)
    inject_oracle_state(eng, o)
    assert np.array_equal(eng.stored_gradients().cpu().numpy(), _round_bf16(o.G))
    o.run(sched[K1:])
    tr = o.trace_arrays()
    eng.run(to_dev(sched[K1:].astype(np.int32)), to_dev(tr["mask"][K1:]))
    st = library_state(eng)
    assert st["k"] == cfg.K and st["error_flags"][0] == 0
    assert np.array_equal(st["tau"], o.tau) and st["uploads_total"][0] == o.uploads_total
    err = rel_l2(st["theta64"], o.theta)
    print(cfg.name, "theta after the hand-over %.2e" % err)
    assert err <= BF16_TOL
    eng.close()


def test_checkpoint_round_trip_is_bitwise():
    cfg = configs.CFG5.scaled(name="mlp3_ragged", layer_dims=(200, 136, 72, 7), M=4, N_m=300, B=130, K=12, D=4, c=2.0)
    prob, dev, sched = _case(cfg)
    idx = to_dev(sched.astype(np.int32))
    a = Cada.from_config(cfg, *dev, trace_steps=cfg.K, gradient_store=STORE_BF16)
    a.run(idx[:5])
    block = a.checkpoint()
    a.run(idx[5:])
    ref = library_state(a)
    b = Cada.from_config(cfg, *dev, trace_steps=cfg.K, gradient_store=STORE_BF16)
    b.restore(block)
    b.run(idx[5:])
    got = library_state(b)
    for key in ("theta", "theta_lo", "h", "vhat", "tau", "ring"):
        assert np.array_equal(ref[key], got[key]), key
    assert np.array_equal(a.stored_gradients().cpu().numpy(), b.stored_gradients().cpu().numpy())
    # a block of the float32 store does not fit a context with the bf16 store
    c = Cada.from_config(cfg, *dev, trace_steps=cfg.K)
    from paper_2012_15469_amd import binding
    assert binding.cada_checkpoint_bytes(c.ctx) > block.numel()
    assert binding._lib.cada_checkpoint_load(c.ctx, block.data_ptr()) == -1 and "different configuration" in binding.cada_last_error()
    for e in (a, b, c):
        e.close()


def test_refused_where_the_store_is_read_by_the_rule_or_the_model_has_none():
    lag = configs.CFG4.scaled(name="mlp2_lag", layer_dims=(20, 16, 10), M=3, N_m=60, B=6, K=4, D=6, rule=configs.RULE_LAG)
    prob, dev, _ = _case(lag)
    with pytest.raises(CadaError, match="LAG"):
        Cada.from_config(lag, *dev, gradient_store=STORE_BF16)
    lr = configs.CFG1.scaled(K=4)
    prob, dev, _ = _case(lr)
    with pytest.raises(CadaError, match="MLP"):
        Cada.from_config(lr, *dev, gradient_store=STORE_BF16)
