#!/usr/bin/env python3
"""Throughput of the CADA hot path on one MI355X: worker-iterations/s.

A step is one call of cada_step(): both minibatch gradients of all M workers, the
communication rule, the masked refresh, the aggregate, the AMSGrad-type update and the
ring push.  Inputs (features, labels, the whole index schedule) are resident in HBM before
the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_per_step(cfg) -> float:
    """Bytes the method itself must move per step for the logistic models: the B gathered
    rows of every worker once (4 B p), the reference iterate read (4p) and the fresh
    gradient write (4p) per worker (CADA1: stored innovation read + fresh innovation write
    instead of the reference read), and the server's pass over the M stored gradients
    plus the five p-vectors it reads/writes (32p)."""
    M, p, B = cfg.M, cfg.p, cfg.B
    per_worker = 4.0 * B * p + 4.0 * p + 4.0 * p
    if cfg.rule == 1:
        per_worker += 4.0 * p
    return M * per_worker + 4.0 * M * p + 32.0 * p


def algorithmic_flops_per_step(cfg) -> float:
    """MLP: two gradient evaluations per worker-iteration, each = forward 2 B sum(in*out),
    weight gradients (the same) and activation gradients for layers >= 2."""
    d = cfg.layer_dims
    fwd = sum(2.0 * cfg.B * d[i] * d[i + 1] for i in range(len(d) - 1))
    dact = sum(2.0 * cfg.B * d[i] * d[i + 1] for i in range(1, len(d) - 1))
    return cfg.M * 2.0 * (2.0 * fwd + dact)


MFMA_BF16_PEAK_TFLOPS = 2500.0


def stored_traffic(workload: str):
    """HBM bytes per launch of the single-pass kernel from the committed rocprofv3 --pmc
    summary, or None when there is none or the kernel's source changed since it was taken."""
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(here, "profiles", "k_fused_%s_traffic.json" % workload)
    src = os.path.join(here, "paper_2012_15469_amd", "csrc", "cada_logreg_fused.hip")
    try:
        rec = json.load(open(path))
        # the kernel is everything above the host-side planning code of that file
        text = open(src).read().split("// Chooses the cluster geometry")[0]
        if rec["kernel_source_sha256"] != hashlib.sha256(text.encode()).hexdigest():
            return None
        return rec["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def bench_replicas(args, cfg, dev) -> int:
    """R independent runs of a small logistic workload in one launch per call."""
    import json as _json
    import numpy as np
    import torch
    from cada_synth import generators
    from paper_2012_15469_amd.binding import Cada
    if cfg.model != "logreg" or cfg.p >= 8192:
        print("--replicas serves the small logistic workloads (1 and 2)", file=sys.stderr)
        return 2
    R, K, W = args.replicas, args.steps, args.warmup
    engines, scheds = [], []
    for r in range(R):
        c = cfg.scaled(seed=cfg.seed + 17 * r)
        prob = generators.make_problem(c)
        X, y = torch.from_numpy(prob.X).to(dev), torch.from_numpy(prob.y).to(dev)
        engines.append(Cada.from_config(c, X, y, torch.from_numpy(prob.theta0).to(dev), whole_steps=True))
        scheds.append(torch.from_numpy(generators.make_schedule(c, W + K)).to(dev))
    Cada.run_replicas(engines, [s[:W].contiguous() for s in scheds])
    timed = [s[W:].contiguous() for s in scheds]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    Cada.run_replicas(engines, timed)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    uploads = 0
    for e in engines:
        st = e.state()
        torch.cuda.synchronize()
        assert int(st["error_flags"].item()) == 0 and bool(torch.isfinite(st["theta"]).all())
        uploads += int(st["uploads_total"].item())
    out = {"metric": "worker-iterations/sec (grads+CADA rule+AMSGrad)", "value": R * cfg.M * K / dt, "unit": "worker-iterations/s",
           "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": 1e3 * dt / K, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "%s x %d independent runs in one launch" % (cfg.name, R), "replicas": R, "M": cfg.M, "p": cfg.p,
                      "B": cfg.B, "N_m": cfg.N_m, "rule": "CADA%d" % cfg.rule, "D": cfg.D, "d_max": cfg.d_max, "c": cfg.c,
                      "uploads_per_worker_step": uploads / float(R * cfg.M * (W + K))}}
    print(_json.dumps(out))
    return 0


def kernel_bytes_per_launch(cfg) -> float:
    """Algorithmic bytes of ONE launch of the logistic gradient kernel(s): the B gathered rows of every
    worker once, the reference iterate (CADA1: the stored innovation) read and the fresh gradient
    written (CADA1: plus the fresh innovation written): M (4 B p + 8 p), CADA1 M (4 B p + 12 p)."""
    per_worker = 4.0 * cfg.B * cfg.p + 8.0 * cfg.p + (4.0 * cfg.p if cfg.rule == 1 else 0.0)
    return cfg.M * per_worker


def measure(cfg, K: int, W: int, plain_launch: bool = False, bf16_store: bool = False, path: str = "auto"):
    """W warm-up steps, K timed steps (no events inside the loop), then K more steps with an event
    around every kernel phase.  Returns (record for the JSON line, problem, seconds of set-up).
    bf16_store: the MLP workloads with the stored gradients kept as bf16 (CADA_STORE_BF16)."""
    import torch
    from cada_synth import generators, native
    from paper_2012_15469_amd import binding
    from paper_2012_15469_amd.binding import Cada
    dev = torch.device("cuda:0")
    t0 = time.time()
    prob = generators.make_problem(cfg)
    if prob.X is None:                  # counter-based recipe: generated in HBM
        shift = torch.from_numpy(prob.shift).to(dev)
        X = torch.empty((cfg.M * cfg.N_m, cfg.p), dtype=torch.float32, device=dev)
        y = torch.empty(cfg.M * cfg.N_m, dtype=torch.float32, device=dev)
        native.fill_device(cfg, shift, X, y)
    else:
        X, y = torch.from_numpy(prob.X).to(dev), torch.from_numpy(prob.y).to(dev)
    theta0 = torch.from_numpy(prob.theta0).to(dev)
    sched = torch.from_numpy(generators.make_schedule(cfg, W + 2 * K)).to(dev)
    torch.cuda.synchronize()
    t_setup = time.time() - t0

    paths = {"auto": binding.PATH_AUTO, "two_pass": binding.PATH_TWO_PASS, "single_pass": binding.PATH_SINGLE_PASS,
             "whole_steps": binding.PATH_WHOLE_STEPS}
    eng = Cada.from_config(cfg, X, y, theta0, trace_steps=0, plain_launch=plain_launch, path=paths[path],
                           gradient_store=binding.STORE_BF16 if bf16_store else binding.STORE_F32)
    # small logistic workloads run whole iterations inside one kernel: the K timed steps are one
    # cada_run call (one launch); everything else is one cada_step call per step
    whole = binding.cada_profile_phase_names(eng.ctx) == ["logreg_whole_steps"]

    def advance(k0, k1):
        if whole:
            eng.run(sched[k0:k1])
        else:
            for k in range(k0, k1):
                eng.step(sched[k])

    advance(0, W)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    advance(W, W + K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    uploads_timed = int(eng.state()["uploads_total"].item())
    binding.cada_profile_begin(eng.ctx, K)
    advance(W + K, W + 2 * K)
    torch.cuda.synchronize()
    prof = binding.cada_profile_end(eng.ctx)
    if whole:       # one profiled launch covered K steps
        prof = {k: (v / K if k != "steps" else K) for k, v in prof.items()}
    st = eng.state()
    torch.cuda.synchronize()
    assert int(st["error_flags"].item()) == 0
    assert bool(torch.isfinite(st["theta"]).all())

    rec = {"value": cfg.M * K / dt, "unit": "worker-iterations/s", "steps": K, "warmup": W, "ms_per_step": 1e3 * dt / K,
           "dtype": "f32" if cfg.gemm_dtype == "fp32" else "bf16",
           "config": {"workload": cfg.name, "M": cfg.M, "p": cfg.p, "B": cfg.B, "N_m": cfg.N_m,
                      "rule": "CADA%d" % cfg.rule, "D": cfg.D, "d_max": cfg.d_max, "c": cfg.c,
                      "gradient_store": "bf16" if bf16_store else "f32",
                      "uploads_per_worker_step": uploads_timed / float(cfg.M * (W + K)), "setup_s": round(t_setup, 1)},
           "kernel_ms": {k: v for k, v in prof.items() if k != "steps"}}
    if cfg.model == "logreg":
        # the gradient phase is one launch of the single-pass kernel (p >= 8192), the two streaming
        # passes over the gathered rows, or (tiny workloads) whole iterations in one kernel
        single = "logreg_single_pass" in prof
        # (single pass: the kernel's own launches; the few microseconds of "logreg_split_round_sum" are listed beside it)
        grad_ms = prof["logreg_single_pass"] if single else sum(v for k, v in prof.items() if k.startswith("logreg_"))
        alg = kernel_bytes_per_launch(cfg) if not whole else algorithmic_bytes_per_step(cfg)
        achieved = alg / (grad_ms * 1e-3) / 1e9
        name = "k_fused" if single else ("k_small (whole iterations; latency-bound)" if whole else "k_dots+k_grad")
        rec["roofline"] = {"bound": "hbm", "kernel": name, "achieved": achieved,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "traffic": stored_traffic(cfg.name) if single else None,
                           "algorithmic_bytes_per_launch": alg, "avg_launch_ms": grad_ms,
                           "whole_step_bytes": algorithmic_bytes_per_step(cfg)}
    else:
        fl = algorithmic_flops_per_step(cfg)
        ms = prof["mlp_gradients"]
        achieved = fl / (ms * 1e-3) / 1e12
        rec["roofline"] = {"bound": "mfma", "kernel": "mlp_gradients (all contraction and elementwise kernels of S1+S2)",
                           "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                           "algorithmic_flops_per_launch": fl, "avg_launch_ms": ms}
    eng.close()
    del X, y, eng, sched
    torch.cuda.empty_cache()
    return rec, prob, t_setup


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=120,
                    help="timed steps of the headline workload (the default passes the forced upload at k = D = 100)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="headline workload 1..5 (default 3: the HBM-bound logistic workload)")
    ap.add_argument("--others", type=str, default="1,2,4,5,4b,5b",
                    help="workloads also measured in this process and reported under \"other_workloads\" ('' = none); "
                         "4b, 5b: the MLP workloads with the bf16 gradient store")
    ap.add_argument("--other-steps", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replicas", type=int, default=1,
                    help="workloads 1-2 only: R independent runs (seeds seed, seed+17, ...) advanced side by side in one "
                         "launch per call (cada_run_replicas); value counts the worker-iterations of all of them")
    ap.add_argument("--bf16-gradient-store", action="store_true",
                    help="workloads 4-5 as the headline workload with the stored gradients kept as bf16 (CADA_STORE_BF16)")
    ap.add_argument("--path", choices=["auto", "two_pass", "single_pass", "whole_steps"], default="auto",
                    help="logistic workloads: the kernels of the headline workload (cada_config.path); auto = the library's choice")
    ap.add_argument("--plain-launch", action="store_true",
                    help="launch the single-pass kernel without the cooperative-launch API (rocprofv3 on this "
                         "image crashes at exit after tracing a cooperative dispatch); same grid, same kernel")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one elementwise pass over 1 GiB (reads 1 GiB, writes 1 GiB): the kernel of known "
                         "size that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: every box here has one, and the path uses no collectives "
              "(--gpus %d refused)" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from cada_synth import configs, generators

    cfg = configs.ALL[args.config]
    dev = torch.device("cuda:0")
    if args.replicas > 1:
        return bench_replicas(args, cfg, dev)
    K, W = args.steps, args.warmup
    rec, prob, _ = measure(cfg, K, W, args.plain_launch, bf16_store=args.bf16_gradient_store, path=args.path)
    out = {"metric": "worker-iterations/sec (grads+CADA rule+AMSGrad)", "value": rec["value"], "unit": rec["unit"],
           "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": rec["ms_per_step"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": rec["dtype"], "data": "synthetic",
           "config": rec["config"], "kernel_ms": rec["kernel_ms"], "roofline": rec["roofline"]}

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    others = [x.strip() for x in args.others.split(",") if x.strip() and x.strip() != str(args.config)]
    if others:
        out["other_workloads"] = {}
        for x in others:
            n, b16 = int(x.rstrip("b")), x.endswith("b")
            r, _, _ = measure(configs.ALL[n], args.other_steps, W, bf16_store=b16)
            out["other_workloads"][configs.ALL[n].name + ("+bf16_gradient_store" if b16 else "")] = r

    if not args.no_cpu_baseline:
        from oracle.driver import oracle_for
        # bounded sample: a few steps of the first Ms workers of the same workload
        Ms = min(cfg.M, 8 if cfg.p >= 4096 else cfg.M)
        sub = cfg.scaled(M=Ms)
        sprob = generators.Problem(sub, None if prob.X is None else prob.X[:Ms * cfg.N_m],
                                   None if prob.y is None else prob.y[:Ms * cfg.N_m], prob.theta0,
                                   None if prob.shift is None else prob.shift[:Ms])
        ssched = generators.make_schedule(sub, 64)
        o = oracle_for(sub, sprob)
        tc = time.perf_counter()
        n = 0
        while n < 64 and (n < 2 or time.perf_counter() - tc < 10.0):
            o.step(ssched[n])
            n += 1
        dtc = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": Ms * n / dtc, "unit": "worker-iterations/s",
                               "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
                               "sample": "%d steps of the first %d of %d workers, same p/B/N_m, fp64 numpy" % (n, Ms, cfg.M)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
