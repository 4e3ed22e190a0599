"""Host-side logic of bench.py: the figures its roofline divides by, the refusal of more than one GPU,
and that the stored HBM traffic is offered only while the kernel it was measured on is unchanged."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_algorithmic_work_of_the_workloads():
    import bench
    from cada_synth import configs
    c3 = configs.CFG3
    # M (4 B p + 8 p): the sampled rows once, the reference iterate read, the fresh gradient written
    assert bench.kernel_bytes_per_launch(c3) == 100 * (4.0 * 256 * 65536 + 8.0 * 65536) == 6763315200.0
    # the whole step adds the server's pass over the stored gradients and its p-vectors
    assert bench.algorithmic_bytes_per_step(c3) == 6763315200.0 + 4.0 * 100 * 65536 + 32.0 * 65536
    # CADA1: stored innovation read and fresh innovation written instead of the reference read
    c2 = configs.CFG2
    assert bench.kernel_bytes_per_launch(c2) == 20 * (4.0 * 32 * 784 + 12.0 * 784)
    # two gradient evaluations: forward + weight gradients (2 x forward) + activation gradients of layers >= 2
    c5 = configs.CFG5
    fwd = 2.0 * 256 * (3072 * 1024 + 1024 * 1024 + 1024 * 10)
    dact = 2.0 * 256 * (1024 * 1024 + 1024 * 10)
    assert bench.algorithmic_flops_per_step(c5) == 16 * 2.0 * (2.0 * fwd + dact)


def test_more_than_one_gpu_is_refused_before_anything_is_imported():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_stored_traffic_belongs_to_the_present_kernel(tmp_path, monkeypatch):
    import bench
    path = os.path.join(ROOT, "profiles", "k_fused_cfg3_logreg_p65536_cada2_traffic.json")
    rec = json.load(open(path))
    t = bench.stored_traffic("cfg3_logreg_p65536_cada2")
    # the committed summary was taken on the committed kernel: offered, and close to the algorithmic bytes
    assert t == rec["hbm_bytes_per_launch"] and 1.0 <= t / 6763315200.0 < 1.1
    assert bench.stored_traffic("no_such_workload") is None
