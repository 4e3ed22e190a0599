"""ctypes binding of libcada.so: argument marshalling only.

The functions carry the names of the C ABI (include/cada.h).  PyTorch supplies
device memory and the stream; every step of the path runs in the library's HIP
kernels.  There is no fallback: if the library is missing, importing this
module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcada.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libcada.so is not built: run `python -m paper_2012_15469_amd.build` "
                      "(no CPU fallback exists)")
_lib = C.CDLL(LIB_PATH)

RULE_CADA1, RULE_CADA2 = 1, 2
MODEL_LOGREG, MODEL_MLP = 0, 1
GEMM_FP32, GEMM_BF16 = 0, 1
REPLAY_FREE = 255
EVAL_NOALLOC_MAX_M = 256
PATH_AUTO, PATH_TWO_PASS, PATH_SINGLE_PASS, PATH_WHOLE_STEPS = 0, 1, 2, 3
STORE_F32, STORE_BF16 = 0, 1


class cada_config(C.Structure):
    _fields_ = [("M", C.c_int32), ("p", C.c_int64), ("model", C.c_int32), ("n_layers", C.c_int32),
                ("layer_dims", C.POINTER(C.c_int32)), ("B", C.c_int32),
                ("n_samples", C.POINTER(C.c_int64)), ("X", C.c_void_p), ("y", C.c_void_p),
                ("alpha", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("lambda_l2", C.c_double), ("c", C.c_double), ("d_max", C.c_int32), ("D", C.c_int32),
                ("rule", C.c_int32), ("gemm_dtype", C.c_int32), ("server", C.c_int32), ("alpha_K0", C.c_int64), ("trace_steps", C.c_int64),
                ("path", C.c_int32), ("single_pass_rows", C.c_int32), ("single_pass_clusters", C.c_int32),
                ("plain_launch", C.c_int32), ("two_pass_group", C.c_int32), ("gradient_store", C.c_int32),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p)]


class cada_state(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("theta", "h", "v", "vhat", "nabla", "theta_lo", "tau", "ring", "mask", "lhs",
                                           "uploads_total", "error_flags")] + \
               [("k", C.c_int64), ("trace_steps", C.c_int64)] + \
               [(n, C.c_void_p) for n in ("trace_mask", "trace_own_mask", "trace_lhs", "trace_rhs", "trace_tau")]


_lib.cada_workspace_bytes.restype = C.c_size_t
_lib.cada_workspace_bytes.argtypes = [C.POINTER(cada_config)]
_lib.cada_init.restype = C.c_int
_lib.cada_init.argtypes = [C.POINTER(cada_config), C.c_void_p, C.POINTER(C.c_void_p)]
_lib.cada_step.restype = C.c_int
_lib.cada_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
_lib.cada_run.restype = C.c_int
_lib.cada_run.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
_lib.cada_run_replicas.restype = C.c_int
_lib.cada_run_replicas.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int64]
_lib.cada_get_state.restype = C.c_int
_lib.cada_get_state.argtypes = [C.c_void_p, C.POINTER(cada_state)]
_lib.cada_copy_stored_gradients.restype = C.c_int
_lib.cada_copy_stored_gradients.argtypes = [C.c_void_p, C.c_void_p]
class cada_state_in(C.Structure):
    _fields_ = [("k", C.c_int64)] + \
               [(n, C.c_void_p) for n in ("theta", "theta_lo", "h", "vhat", "stored_gradients", "reference", "reference_lo",
                                           "stored_innovations", "tau", "ring")] + \
               [("uploads_total", C.c_uint64)]


_lib.cada_set_state.restype = C.c_int
_lib.cada_set_state.argtypes = [C.c_void_p, C.POINTER(cada_state_in)]
_lib.cada_eval.restype = C.c_int
_lib.cada_eval.argtypes = [C.c_void_p, C.c_void_p]
_lib.cada_eval_noalloc.restype = C.c_int
_lib.cada_eval_noalloc.argtypes = [C.c_void_p, C.c_void_p]
_lib.cada_checkpoint_bytes.restype = C.c_size_t
_lib.cada_checkpoint_bytes.argtypes = [C.c_void_p]
_lib.cada_checkpoint_save.restype = C.c_int
_lib.cada_checkpoint_save.argtypes = [C.c_void_p, C.c_void_p]
_lib.cada_checkpoint_load.restype = C.c_int
_lib.cada_checkpoint_load.argtypes = [C.c_void_p, C.c_void_p]
_lib.cada_profile_phases.restype = C.c_int
_lib.cada_profile_phases.argtypes = [C.c_void_p]
_lib.cada_profile_phase_name.restype = C.c_char_p
_lib.cada_profile_phase_name.argtypes = [C.c_void_p, C.c_int]
_lib.cada_profile_begin.restype = C.c_int
_lib.cada_profile_begin.argtypes = [C.c_void_p, C.c_int64]
_lib.cada_profile_end.restype = C.c_int
_lib.cada_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.c_int, C.POINTER(C.c_int64)]
_lib.cada_destroy.restype = None
_lib.cada_destroy.argtypes = [C.c_void_p]
_lib.cada_last_error.restype = C.c_char_p
_lib.cada_last_error.argtypes = []


class CadaError(RuntimeError):
    pass


def cada_last_error() -> str:
    return _lib.cada_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise CadaError("libcada error %d: %s" % (rc, cada_last_error()))


def cada_workspace_bytes(cfg: cada_config) -> int:
    n = _lib.cada_workspace_bytes(C.byref(cfg))
    if n == 0:
        raise CadaError("libcada: %s" % cada_last_error())
    return n


def cada_init(cfg: cada_config, theta0_ptr: int) -> int:
    out = C.c_void_p()
    _check(_lib.cada_init(C.byref(cfg), theta0_ptr, C.byref(out)))
    return out.value


def cada_step(ctx: int, idx_ptr: int, replay_ptr: Optional[int]):
    _check(_lib.cada_step(ctx, idx_ptr, replay_ptr))


def cada_run(ctx: int, idx_sched_ptr: int, replay_sched_ptr: Optional[int], n_steps: int):
    _check(_lib.cada_run(ctx, idx_sched_ptr, replay_sched_ptr, n_steps))


def cada_get_state(ctx: int) -> cada_state:
    st = cada_state()
    _check(_lib.cada_get_state(ctx, C.byref(st)))
    return st


def cada_copy_stored_gradients(ctx: int, out_ptr: int):
    _check(_lib.cada_copy_stored_gradients(ctx, out_ptr))


def cada_set_state(ctx: int, st: cada_state_in):
    _check(_lib.cada_set_state(ctx, C.byref(st)))


def cada_profile_begin(ctx: int, max_steps: int):
    _check(_lib.cada_profile_begin(ctx, max_steps))


def cada_eval(ctx: int, out_ptr: int):
    _check(_lib.cada_eval(ctx, out_ptr))


def cada_eval_noalloc(ctx: int, out_ptr: int):
    _check(_lib.cada_eval_noalloc(ctx, out_ptr))


def cada_checkpoint_bytes(ctx: int) -> int:
    return int(_lib.cada_checkpoint_bytes(ctx))


def cada_checkpoint_save(ctx: int, dst_ptr: int):
    _check(_lib.cada_checkpoint_save(ctx, dst_ptr))


def cada_checkpoint_load(ctx: int, src_ptr: int):
    _check(_lib.cada_checkpoint_load(ctx, src_ptr))


def cada_profile_phase_names(ctx: int) -> list:
    return [_lib.cada_profile_phase_name(ctx, i).decode() for i in range(_lib.cada_profile_phases(ctx))]


def cada_profile_end(ctx: int) -> dict:
    """{phase name: mean milliseconds per step} over the profiled steps, plus "steps"."""
    n = _lib.cada_profile_phases(ctx)
    ms = (C.c_double * max(n, 1))()
    steps = C.c_int64()
    _check(_lib.cada_profile_end(ctx, ms, n, C.byref(steps)))
    out = {_lib.cada_profile_phase_name(ctx, i).decode(): (ms[i] / max(steps.value, 1)) for i in range(n)}
    out["steps"] = steps.value
    return out


def cada_run_replicas(ctxs: Sequence[int], idx_sched_ptrs: Sequence[int], replay_sched_ptrs: Optional[Sequence[Optional[int]]],
                      n_steps: int):
    n = len(ctxs)
    a_ctx = (C.c_void_p * n)(*ctxs)
    a_idx = (C.c_void_p * n)(*idx_sched_ptrs)
    a_rep = None if replay_sched_ptrs is None else (C.c_void_p * n)(*replay_sched_ptrs)
    _check(_lib.cada_run_replicas(a_ctx, n, a_idx, a_rep, n_steps))


def cada_destroy(ctx: int):
    _lib.cada_destroy(ctx)


class Cada:
    """Owns the torch-allocated workspace and the library context for one run."""

    def __init__(self, *, model: str, layer_dims: Sequence[int], M: int, B: int, n_samples: Sequence[int],
                 X: torch.Tensor, y: torch.Tensor, theta0: torch.Tensor, rule: int, D: int, d_max: int,
                 c: float, alpha: float, beta1: float, beta2: float, eps: float, lam: float = 0.0,
                 gemm_dtype: str = "fp32", trace_steps: int = 0, stream: Optional[torch.cuda.Stream] = None,
                 server: int = 0, alpha_K0: int = 0, whole_steps: bool = False, path: int = PATH_AUTO,
                 single_pass_rows: int = 0, single_pass_clusters: int = 0, plain_launch: bool = False, two_pass_group: int = 0,
                 gradient_store: int = STORE_F32):
        assert X.is_cuda and y.is_cuda and theta0.is_cuda
        assert X.dtype == torch.float32 and X.is_contiguous() and theta0.dtype == torch.float32
        assert y.dtype == (torch.float32 if model == "logreg" else torch.int32) and y.is_contiguous()
        self.M, self.B, self.p = M, B, int(theta0.numel())
        self.d_max = d_max
        self.stream = stream or torch.cuda.current_stream(X.device)
        self._keep = (X, y)
        dims = list(layer_dims) if model == "mlp" else [int(layer_dims[0]), 1]
        n_layers = len(dims) - 1
        self._dims = (C.c_int32 * len(dims))(*dims)
        self._ns = (C.c_int64 * M)(*[int(n) for n in n_samples])
        cfg = cada_config()
        cfg.M, cfg.p, cfg.model, cfg.n_layers = M, self.p, MODEL_LOGREG if model == "logreg" else MODEL_MLP, n_layers
        cfg.layer_dims, cfg.B, cfg.n_samples = self._dims, B, self._ns
        cfg.X, cfg.y = X.data_ptr(), y.data_ptr()
        cfg.alpha, cfg.beta1, cfg.beta2, cfg.eps, cfg.lambda_l2, cfg.c = alpha, beta1, beta2, eps, lam, c
        cfg.d_max, cfg.D, cfg.rule = d_max, D, rule
        cfg.gemm_dtype = GEMM_BF16 if gemm_dtype == "bf16" else GEMM_FP32
        cfg.server = server
        cfg.alpha_K0 = alpha_K0
        cfg.trace_steps = trace_steps
        cfg.path = PATH_WHOLE_STEPS if whole_steps else path
        cfg.single_pass_rows, cfg.single_pass_clusters = single_pass_rows, single_pass_clusters
        cfg.plain_launch, cfg.two_pass_group = (1 if plain_launch else 0), two_pass_group
        cfg.gradient_store = gradient_store
        cfg.stream = self.stream.cuda_stream
        nbytes = cada_workspace_bytes(cfg)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=X.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self._ws_off = base - self.workspace.data_ptr()
        cfg.workspace, cfg.workspace_bytes = base, nbytes
        self.cfg = cfg
        self.ctx = cada_init(cfg, theta0.contiguous().data_ptr())
        self.k = 0

    @classmethod
    def from_config(cls, cfg, X, y, theta0, **kw):
        args = dict(model=cfg.model, layer_dims=cfg.layer_dims, M=cfg.M, B=cfg.B, n_samples=[cfg.N_m] * cfg.M,
                    X=X, y=y, theta0=theta0, rule=cfg.rule, D=cfg.D, d_max=cfg.d_max, c=cfg.c, alpha=cfg.alpha,
                    beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, lam=cfg.lam, gemm_dtype=cfg.gemm_dtype,
                    server=getattr(cfg, "server", 0), alpha_K0=getattr(cfg, "alpha_K0", 0))
        args.update(kw)
        return cls(**args)

    def step(self, idx: torch.Tensor, replay: Optional[torch.Tensor] = None):
        assert idx.dtype == torch.int32 and idx.is_cuda and idx.is_contiguous() and idx.numel() == self.M * self.B
        if replay is not None:
            assert replay.dtype == torch.uint8 and replay.is_cuda and replay.numel() == self.M
        cada_step(self.ctx, idx.data_ptr(), None if replay is None else replay.data_ptr())
        self.k += 1

    def run(self, idx_sched: torch.Tensor, replay_sched: Optional[torch.Tensor] = None):
        n = idx_sched.shape[0]
        assert idx_sched.dtype == torch.int32 and idx_sched.is_cuda and idx_sched.is_contiguous()
        assert idx_sched.numel() == n * self.M * self.B
        if replay_sched is not None:
            assert replay_sched.dtype == torch.uint8 and replay_sched.is_contiguous() and replay_sched.numel() == n * self.M
        cada_run(self.ctx, idx_sched.data_ptr(), None if replay_sched is None else replay_sched.data_ptr(), n)
        self.k += n

    @staticmethod
    def run_replicas(engines: Sequence["Cada"], idx_scheds: Sequence[torch.Tensor],
                     replay_scheds: Optional[Sequence[Optional[torch.Tensor]]] = None):
        """Independent runs (same shapes, created with whole_steps=True) advanced together in one launch."""
        n = idx_scheds[0].shape[0]
        for e, s in zip(engines, idx_scheds):
            assert s.dtype == torch.int32 and s.is_cuda and s.is_contiguous() and s.numel() == n * e.M * e.B
        reps = None
        if replay_scheds is not None:
            for e, r in zip(engines, replay_scheds):
                assert r is None or (r.dtype == torch.uint8 and r.is_contiguous() and r.numel() == n * e.M)
            reps = [None if r is None else r.data_ptr() for r in replay_scheds]
        cada_run_replicas([e.ctx for e in engines], [s.data_ptr() for s in idx_scheds], reps, n)
        for e in engines:
            e.k += n

    def _view(self, ptr: int, n: int, dtype: torch.dtype) -> torch.Tensor:
        off = ptr - self.workspace.data_ptr()
        nb = n * torch.empty((), dtype=dtype).element_size()
        return self.workspace[off:off + nb].view(dtype)

    def state(self) -> dict:
        """Views into the workspace (no copies).  Synchronise the stream before reading."""
        st = cada_get_state(self.ctx)
        M, p, T = self.M, self.p, min(int(st.trace_steps), int(st.k))
        f32, i32, u8 = torch.float32, torch.int32, torch.uint8
        out = {n: self._view(getattr(st, n), p, f32) for n in ("theta", "theta_lo", "h", "v", "vhat", "nabla")}
        out["tau"] = self._view(st.tau, M, i32)
        out["ring"] = self._view(st.ring, self.d_max, f32)
        out["mask"] = self._view(st.mask, M, u8)
        out["lhs"] = self._view(st.lhs, M, f32)
        out["uploads_total"] = self._view(st.uploads_total, 1, torch.int64)
        out["error_flags"] = self._view(st.error_flags, 1, i32)
        out["k"] = int(st.k)
        if T > 0:
            out["trace_mask"] = self._view(st.trace_mask, T * M, u8).view(T, M)
            out["trace_own_mask"] = self._view(st.trace_own_mask, T * M, u8).view(T, M)
            out["trace_lhs"] = self._view(st.trace_lhs, T * M, f32).view(T, M)
            out["trace_rhs"] = self._view(st.trace_rhs, T, f32)
            out["trace_tau"] = self._view(st.trace_tau, T * M, i32).view(T, M)
        return out

    def stored_gradients(self) -> torch.Tensor:
        out = torch.empty(self.M, self.p, dtype=torch.float32, device=self.workspace.device)
        cada_copy_stored_gradients(self.ctx, out.data_ptr())
        return out

    def set_state(self, *, k: int, theta, h, vhat, stored_gradients, tau, ring, uploads_total: int = 0, theta_lo=None,
                  reference=None, reference_lo=None, stored_innovations=None):
        """Replaces the state by explicit device arrays (see cada_set_state): float32 tensors of the
        shapes documented in cada.h, tau int32."""
        M, p = self.M, self.p
        def ptr(t, n, dtype=torch.float32):
            if t is None:
                return None
            assert t.is_cuda and t.dtype == dtype and t.is_contiguous() and t.numel() == n, (t.shape, t.dtype, n)
            return t.data_ptr()
        st = cada_state_in()
        st.k = k
        st.theta, st.theta_lo, st.h, st.vhat = ptr(theta, p), ptr(theta_lo, p), ptr(h, p), ptr(vhat, p)
        st.stored_gradients = ptr(stored_gradients, M * p)
        nref = M * p if self.cfg.rule == RULE_CADA2 else p
        st.reference, st.reference_lo = ptr(reference, nref), ptr(reference_lo, nref)
        st.stored_innovations = ptr(stored_innovations, M * p)
        st.tau, st.ring = ptr(tau, M, torch.int32), ptr(ring, self.d_max)
        st.uploads_total = uploads_total
        cada_set_state(self.ctx, st)
        self.k = k

    def evaluate(self) -> torch.Tensor:
        """DEVICE float64 [2]: objective L(theta) and accuracy on all the data (see cada_eval)."""
        out = torch.empty(2, dtype=torch.float64, device=self.workspace.device)
        cada_eval(self.ctx, out.data_ptr())
        return out

    def checkpoint(self) -> torch.Tensor:
        """The whole state as one opaque device block (see cada_checkpoint_save)."""
        out = torch.empty(cada_checkpoint_bytes(self.ctx), dtype=torch.uint8, device=self.workspace.device)
        cada_checkpoint_save(self.ctx, out.data_ptr())
        return out

    def restore(self, block: torch.Tensor):
        assert block.is_cuda and block.dtype == torch.uint8 and block.is_contiguous()
        assert block.numel() == cada_checkpoint_bytes(self.ctx)
        cada_checkpoint_load(self.ctx, block.data_ptr())
        st = cada_state()
        _check(_lib.cada_get_state(self.ctx, C.byref(st)))
        self.k = int(st.k)

    def close(self):
        if self.ctx:
            cada_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
