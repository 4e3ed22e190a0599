"""Builds the HIP libraries in-tree for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]

LIBCADA = os.path.join(HERE, "libcada.so")
LIBCADA_SRC = [os.path.join(HERE, "csrc", f) for f in
               ("cada_api.hip", "cada_logreg.hip", "cada_logreg_fused.hip", "cada_logreg_small.hip", "cada_server.hip",
                "cada_mlp.hip")]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build_libcada() -> str:
    """Compiles the translation units side by side (objects in a temporary folder), then links."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    compile_flags = [f for f in HIP_FLAGS if f != "-shared"] + ["-c", "-I", os.path.join(ROOT, "include")]
    with tempfile.TemporaryDirectory(prefix="libcada_build_") as tmp:
        objs = [os.path.join(tmp, os.path.basename(src) + ".o") for src in LIBCADA_SRC]
        with ThreadPoolExecutor(max_workers=min(len(objs), os.cpu_count() or 1)) as pool:
            list(pool.map(lambda so: _run([HIPCC, *compile_flags, "-o", so[1], so[0]]), zip(LIBCADA_SRC, objs)))
        _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIBCADA, *objs])
    return LIBCADA


def build_all() -> None:
    build_libcada()


if __name__ == "__main__":
    build_all()
    print("built", LIBCADA)
    sys.exit(0)
