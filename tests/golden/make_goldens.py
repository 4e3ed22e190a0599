#!/usr/bin/env python3
"""Writes the stored expected values of the full-size parity cases.

Calls only the CPU oracle (oracle/) and the seeded input generators (cada_synth/); nothing
here touches the GPU library.  Each .npz holds the oracle's trace (mask, lhs, rhs, tau),
the final iterate (all of it up to 2^16 coordinates, else every `stride`-th coordinate plus
its norm) and a fingerprint of the inputs so that a test can tell a stale file.

    python tests/golden/make_goldens.py [case ...]
"""
from __future__ import annotations

import os
import sys
import time
import zlib

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from cada_synth import configs, generators  # noqa: E402
from oracle.driver import oracle_for        # noqa: E402

# name -> (config, steps).  Every horizon passes the maximum delay D of its workload, so that the
# forced upload of Algorithm 1 (tau_m >= D), the wrap of the D+1 retained iterates (CADA2) and the
# snapshot refresh at k = D (CADA1) are all crossed at full size.
CASES = {
    "cfg3_full_c0.3": (configs.CFG3, 104),                      # with c = 0.3 nobody uploads before the forced upload at k = 100
    "cfg3_full_c1e-4": (configs.CFG3.scaled(c=1e-4), 104),      # rule-driven uploads and skips mix
    "cfg4_full": (configs.CFG4, 104),
    "cfg5_full": (configs.CFG5, 204),
    # larger c than the workloads' 0.5, with which every worker uploads in the first steps
    "cfg4_full_c3": (configs.CFG4.scaled(c=3.0), 104),
    "cfg5_full_c20": (configs.CFG5.scaled(c=20.0), 204),
}
# iterates are also kept after these many steps (sampled like the final one, at most 2^14 coordinates)
CHECKPOINTS = (2, 8, 25, 50, 99, 101, 150, 199, 201)


def fingerprint(cfg, prob, sched) -> int:
    """CRC of the schedule, the initial iterate and the first minibatch of worker 0."""
    X0, y0 = prob.rows(0, sched[0, 0])
    h = zlib.crc32(np.ascontiguousarray(sched).tobytes())
    h = zlib.crc32(np.ascontiguousarray(prob.theta0).tobytes(), h)
    h = zlib.crc32(np.ascontiguousarray(X0).tobytes(), h)
    h = zlib.crc32(np.ascontiguousarray(y0).tobytes(), h)
    return h


def theta_sample(theta, most=1 << 16):
    stride = 1 if theta.size <= most else int(np.ceil(theta.size / most))
    return theta[::stride].copy(), stride


def make(name):
    cfg, K = CASES[name]
    t0 = time.time()
    prob = generators.make_problem(cfg)
    sched = generators.make_schedule(cfg, K)
    o = oracle_for(cfg, prob)
    first = {}
    ck_steps, ck_theta, ck_stride, ck_full = [], [], 1, {}
    for k in range(K):
        o.step(sched[k])
        if k + 1 in CHECKPOINTS and k + 1 < K:
            th_k, ck_stride = theta_sample(o.theta, 1 << 14)
            ck_steps.append(k + 1)
            ck_theta.append(th_k)
            if cfg.model == "mlp":
                ck_full[k + 1] = o.theta.copy()
        if k == 0:   # every worker uploads at step 0: the stored gradients are the gradients at theta0
            first = dict(G0_first=theta_sample(o.G[0])[0], G0_last=theta_sample(o.G[-1])[0],
                         G0_norms=np.linalg.norm(o.G, axis=1))
        print("  %s step %d/%d  %.0fs" % (name, k + 1, K, time.time() - t0), flush=True)
    tr = o.trace_arrays()
    probe = {}
    if cfg.model == "mlp":
        # How far the fp64 oracle itself moves when its initial iterate is perturbed by 1e-6 relative
        # (same decisions replayed): a ReLU network's trajectory is only piecewise smooth, and this is
        # the yardstick for the drift of any finite-precision implementation over the same horizon.
        rng = np.random.default_rng(cfg.seed + 1)
        th0 = prob.theta0.astype(np.float64) * (1.0 + 1e-6 * rng.uniform(-1.0, 1.0, prob.theta0.size))
        o2 = oracle_for(cfg, prob, theta0=th0)
        drift = []
        k_list = list(ck_steps) + [K]
        for k in range(K):
            o2.step(sched[k], tr["mask"][k])
            if k + 1 in k_list:
                drift.append(np.linalg.norm(o2.theta - (ck_full[k + 1] if k + 1 < K else o.theta)) / np.linalg.norm(o.theta))
            if (k + 1) % 10 == 0:
                print("  %s probe step %d/%d  %.0fs" % (name, k + 1, K, time.time() - t0), flush=True)
        probe = dict(probe_steps=np.asarray(k_list, dtype=np.int64), probe_drift=np.asarray(drift))
    th, stride = theta_sample(o.theta)
    # stored gradient of the first and the last worker, sampled like the iterate, and every
    # worker's stored-gradient norm: a direct check of the gradient kernels at full size
    G_first, _ = theta_sample(o.G[0])
    G_last, _ = theta_sample(o.G[-1])
    np.savez_compressed(os.path.join(HERE, name + ".npz"), mask=tr["mask"], own_mask=tr["own_mask"], lhs=tr["lhs"],
                        rhs=tr["rhs"], tau=tr["tau"], tau_final=o.tau, theta=th, theta_stride=stride,
                        G_first=G_first, G_last=G_last, G_norms=np.linalg.norm(o.G, axis=1), **first,
                        theta_norm=np.linalg.norm(o.theta), h_norm=np.linalg.norm(o.h),
                        vhat_norm=np.linalg.norm(o.vhat), ring=o.ring, uploads_total=o.uploads_total,
                        ckpt_steps=np.asarray(ck_steps, dtype=np.int64), ckpt_theta=np.asarray(ck_theta), ckpt_stride=ck_stride,
                        fingerprint=fingerprint(cfg, prob, sched), K=K, **probe)


if __name__ == "__main__":
    for n in (sys.argv[1:] or list(CASES)):
        make(n)
