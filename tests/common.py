"""Shared helpers of the GPU parity tests: upload a seeded problem, run the library
through its C ABI binding, and compare with the CPU oracle under the protocol
  (i)  free run: masks equal up to the first disagreement, which must sit where the
       oracle's rule margin |LHS-RHS|/RHS is <= 1e-5;
  (ii) replay of the oracle's masks: the library's own rule decision is compared at every
       step (disagreements only at margins <= 1e-5 for float32 arithmetic) and theta after
       K steps must agree to the stated relative L2 error.
"""
from __future__ import annotations

import numpy as np
import torch

from cada_synth import generators
from oracle.cada_oracle import margins
from oracle.driver import oracle_for

MARGIN = 1e-5


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def upload(prob):
    """Device copies (X, y, theta0) of a host-resident problem."""
    X = to_dev(prob.X)
    y = to_dev(prob.y)
    return X, y, to_dev(prob.theta0)


def run_library(cfg, dev, sched, replay=None, expect_phase=None, **kw):
    """K = len(sched) steps through cada_run; returns the state as numpy arrays.
    expect_phase: name of a kernel phase the context must run (the path a test asked for was taken)."""
    from paper_2012_15469_amd.binding import Cada, cada_profile_phase_names
    X, y, th0 = dev
    K = sched.shape[0]
    eng = Cada.from_config(cfg, X, y, th0, trace_steps=K, **kw)
    if expect_phase is not None:
        assert expect_phase in cada_profile_phase_names(eng.ctx), cada_profile_phase_names(eng.ctx)
    idx = to_dev(sched.astype(np.int32))
    rp = None if replay is None else to_dev(np.ascontiguousarray(replay, dtype=np.uint8))
    eng.run(idx, rp)
    torch.cuda.synchronize()
    st = eng.state()
    torch.cuda.synchronize()
    out = {k: (v.cpu().numpy().copy() if isinstance(v, torch.Tensor) else v) for k, v in st.items()}
    out["stored"] = eng.stored_gradients().cpu().numpy()
    out["theta64"] = out["theta"].astype(np.float64) + out["theta_lo"].astype(np.float64)
    eng.close()
    return out


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def oracle_run(cfg, prob, sched, replay=None):
    o = oracle_for(cfg, prob)
    o.run(sched, replay)
    return o, o.trace_arrays()


def check_protocol(cfg, prob, dev, sched, theta_tol, lhs_rtol=None, own_mask_exact=True, report=None,
                   free_margin=MARGIN, **kw):
    o, tr = oracle_run(cfg, prob, sched)
    mg = margins(tr["lhs"], tr["rhs"])
    K = sched.shape[0]
    # (i) free run
    free = run_library(cfg, dev, sched, **kw)
    assert free["error_flags"][0] == 0
    diff = free["trace_mask"] != tr["mask"]
    first_bad = None
    if diff.any():
        kk = int(np.argmax(diff.any(axis=1)))
        first_bad = kk
        for m in np.flatnonzero(diff[kk]):
            assert free_margin is None or mg[kk, m] <= free_margin, (
                "free run: first mask disagreement at step %d worker %d has oracle margin %.3e" % (kk, m, mg[kk, m]))
    # (ii) replay of the oracle's masks
    rep = run_library(cfg, dev, sched, replay=tr["mask"], **kw)
    assert rep["error_flags"][0] == 0
    assert np.array_equal(rep["trace_mask"], tr["mask"])
    assert np.array_equal(rep["trace_tau"], tr["tau"])
    own_diff = rep["trace_own_mask"] != tr["own_mask"]
    wide = own_diff & (mg > MARGIN)
    if own_mask_exact:
        assert wide.sum() == 0, "own-rule disagreements outside the margin: %d (first at %s)" % (
            wide.sum(), np.argwhere(wide)[:3].tolist())
    err_theta = rel_l2(rep["theta64"], o.theta)
    assert err_theta <= theta_tol, "theta relative L2 error %.3e > %.1e" % (err_theta, theta_tol)
    assert rep["uploads_total"][0] == o.uploads_total
    assert np.array_equal(rep["tau"], o.tau)
    if lhs_rtol is not None:
        scale = np.maximum(tr["lhs"], 1e-30)
        big = tr["lhs"] > 1e-12 * max(tr["lhs"].max(), 1e-300)
        rel = np.abs(rep["trace_lhs"] - tr["lhs"]) / scale
        assert rel[big].max() <= lhs_rtol, "LHS relative error %.3e" % rel[big].max()
        # (a systematic error would show in the bulk; of a few hundred values the 99 % quantile is the second largest,
        # which the bound on the maximum already covers)
        assert np.quantile(rel[big], 0.9) <= lhs_rtol / 10, "LHS relative error, 90%% quantile %.3e" % np.quantile(rel[big], 0.9)
        rr = np.abs(rep["trace_rhs"] - tr["rhs"]) / np.maximum(tr["rhs"], 1e-300)
        assert rr[tr["rhs"] > 0].max() <= lhs_rtol, "RHS relative error %.3e" % rr[tr["rhs"] > 0].max()
    stats = {"K": K, "first_free_disagreement": first_bad,
             "first_free_disagreement_margin": None if first_bad is None else float(mg[first_bad][diff[first_bad]].max()), "own_disagreements": int(own_diff.sum()),
             "own_disagreements_outside_margin": int(wide.sum()), "theta_rel_l2": err_theta,
             "h_rel_l2": rel_l2(rep["h"], o.h), "vhat_rel_l2": rel_l2(rep["vhat"], o.vhat),
             "nabla_rel_l2": rel_l2(rep["nabla"], o.nabla), "ring_rel": rel_l2(rep["ring"], o.ring),
             "stored_rel_l2": rel_l2(rep["stored"], o.G), "uploads": int(o.uploads_total)}
    if report is not None:
        report.update(stats)
    return stats, o, tr, rep


def split64(a):
    """float64 array -> (hi, lo) float32 device tensors with hi + lo = a to ~2^-48 relative."""
    a = np.asarray(a, dtype=np.float64)
    hi = a.astype(np.float32)
    lo = (a - hi.astype(np.float64)).astype(np.float32)
    return to_dev(hi), to_dev(lo)


def inject_oracle_state(eng, o):
    """Hands the oracle's whole state (before its iteration o.k) to the library through
    cada_set_state: the library then continues Algorithm 1 from the oracle's own trajectory."""
    th, tl = split64(o.theta)
    kw = dict(k=int(o.k), theta=th, theta_lo=tl, h=to_dev(o.h, torch.float32), vhat=to_dev(o.vhat, torch.float32),
              stored_gradients=to_dev(o.G, torch.float32), tau=to_dev(o.tau, torch.int32),
              ring=to_dev(o.ring, torch.float32), uploads_total=int(o.uploads_total))
    if o.rule == 2:
        kw["reference"], kw["reference_lo"] = split64(o.theta_hat)
    elif o.rule == 1:
        kw["reference"], kw["reference_lo"] = split64(o.theta_snap)
        kw["stored_innovations"] = to_dev(o.delta_stored, torch.float32)
    eng.set_state(**kw)


def library_state(eng):
    torch.cuda.synchronize()
    st = eng.state()
    torch.cuda.synchronize()
    out = {k: (v.cpu().numpy().copy() if isinstance(v, torch.Tensor) else v) for k, v in st.items()}
    out["theta64"] = out["theta"].astype(np.float64) + out["theta_lo"].astype(np.float64)
    return out
