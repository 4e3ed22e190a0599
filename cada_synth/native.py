"""Native twins of the counter-based row generator: a C one for host rows and a HIP
one that fills HBM directly.  Both implement the function defined in philox.py."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

from . import philox

HERE = os.path.dirname(os.path.abspath(__file__))
CPU_LIB = os.path.join(HERE, "libcada_rowgen_cpu.so")
HIP_LIB = os.path.join(HERE, "libcada_rowgen_hip.so")


def build() -> None:
    subprocess.run(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", CPU_LIB,
                    os.path.join(HERE, "csrc", "rowgen_cpu.c")], check=True)
    r = subprocess.run([os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "-O3", "--offload-arch=gfx950", "-std=c++17",
                        "-shared", "-fPIC", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-o", HIP_LIB, os.path.join(HERE, "csrc", "rowgen.hip")],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stdout)


_cpu = None
_hip = None


def have_cpu() -> bool:
    return os.path.exists(CPU_LIB)


def rows_cpu(seed: int, m: int, rows, p: int, shift_m: np.ndarray):
    """Features float32 [R, p] and labels float32 [R] of worker m's samples ``rows``."""
    global _cpu
    if _cpu is None:
        _cpu = C.CDLL(CPU_LIB)
        _cpu.cada_synth_rows_cpu.restype = C.c_int
        _cpu.cada_synth_rows_cpu.argtypes = [C.c_uint32, C.c_int32, C.c_void_p, C.c_int64, C.c_int64, C.c_float,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    shift_m = np.ascontiguousarray(shift_m, dtype=np.float32)
    X = np.empty((rows.size, p), dtype=np.float32)
    y = np.empty(rows.size, dtype=np.float32)
    rc = _cpu.cada_synth_rows_cpu(seed & 0xFFFFFFFF, m, rows.ctypes.data, rows.size, p, float(philox.scale_for(p)),
                                  shift_m.ctypes.data, X.ctypes.data, y.ctypes.data)
    if rc != 0:
        raise MemoryError("cada_synth_rows_cpu failed")
    return X, y


def fill_device(cfg, shift_dev, X_dev, y_dev, stream_ptr: int = 0, rows_per_call: int = 1 << 20):
    """Generates all M*N_m rows of ``cfg`` into the torch CUDA tensors X_dev [M*N_m, p] and
    y_dev [M*N_m] (float32).  ``shift_dev`` is the float32 [M, p] mean shift on the device."""
    import torch
    global _hip
    if _hip is None:
        _hip = C.CDLL(HIP_LIB)
        _hip.cada_synth_counter_rows.restype = C.c_int
        _hip.cada_synth_counter_rows.argtypes = [C.c_uint32, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_float,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    p, total = cfg.d0, cfg.M * cfg.N_m
    assert X_dev.shape == (total, p) and X_dev.dtype == torch.float32 and X_dev.is_contiguous()
    assert y_dev.shape == (total,) and y_dev.dtype == torch.float32
    assert shift_dev.shape == (cfg.M, p) and shift_dev.dtype == torch.float32 and shift_dev.is_contiguous()
    tdir = torch.empty(p, dtype=torch.int32, device=X_dev.device)
    for r0 in range(0, total, rows_per_call):
        n = min(rows_per_call, total - r0)
        rc = _hip.cada_synth_counter_rows(cfg.seed & 0xFFFFFFFF, cfg.N_m, p, r0, n, float(philox.scale_for(p)),
                                          shift_dev.data_ptr(), tdir.data_ptr(), X_dev.data_ptr(), y_dev.data_ptr(),
                                          stream_ptr)
        if rc != 0:
            raise RuntimeError("cada_synth_counter_rows failed with hipError %d" % rc)
    return tdir
