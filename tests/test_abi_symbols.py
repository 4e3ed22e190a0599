"""The C-ABI library loads without a GPU and exports every function the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header_text):
    text = re.sub(r"/\*.*?\*/", "", header_text, flags=re.S)
    return sorted(set(re.findall(r"\b(cada_[a-z_0-9]+)\s*\(", text)))


def test_libcada_exports_every_declared_symbol():
    names = []
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            names += declared_functions(open(os.path.join(inc, f)).read())
    assert {"cada_init", "cada_step", "cada_get_state"} <= set(names)
    lib_path = os.path.join(ROOT, "paper_2012_15469_amd", "libcada.so")
    if not os.path.exists(lib_path):
        from paper_2012_15469_amd import build
        build.build_all()
    lib = ctypes.CDLL(lib_path)
    for n in names:
        assert hasattr(lib, n), "libcada.so does not export %s" % n


def test_argument_errors_without_gpu():
    """Validation happens on the host before anything touches a device."""
    from paper_2012_15469_amd import binding as b
    cfg = b.cada_config()
    cfg.M = 0
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0
    assert "M must be" in b.cada_last_error()
    dims = (ctypes.c_int32 * 2)(54, 1)
    ns = (ctypes.c_int64 * 2)(10, 10)
    cfg.M, cfg.p, cfg.model, cfg.n_layers, cfg.layer_dims, cfg.B, cfg.n_samples = 2, 54, 0, 1, dims, 4, ns
    cfg.d_max, cfg.D, cfg.rule = 10, 5, 2
    n = b._lib.cada_workspace_bytes(ctypes.byref(cfg))
    assert n > 4 * 54 * (5 + 2 * 2 + 6)
    cfg.p = 55
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "does not match" in b.cada_last_error()
    cfg.p = 54
    cfg.path = 7
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "path must be" in b.cada_last_error()
    cfg.path = b.PATH_AUTO
    cfg.single_pass_clusters = -1
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "tuning" in b.cada_last_error()
    cfg.single_pass_clusters = 0
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) > 0
    out = ctypes.c_void_p()
    assert b._lib.cada_init(ctypes.byref(cfg), None, ctypes.byref(out)) == -1     # theta0 NULL
    assert b._lib.cada_set_state(None, None) == -1 and b._lib.cada_eval_noalloc(None, None) == -1
    assert b._lib.cada_step(None, None, None) == -1


def _mlp_cfg(b, dims, M, B, N_m, rule):
    cfg = b.cada_config()
    d = (ctypes.c_int32 * len(dims))(*dims)
    ns = (ctypes.c_int64 * M)(*([N_m] * M))
    p = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
    cfg.M, cfg.p, cfg.model, cfg.n_layers, cfg.layer_dims, cfg.B, cfg.n_samples = M, p, b.MODEL_MLP, len(dims) - 1, d, B, ns
    cfg.d_max, cfg.D, cfg.rule, cfg.gemm_dtype = 10, 20, rule, b.GEMM_BF16
    cfg._keep = (d, ns)
    return cfg, p


def test_mlp_workspace_sizing_without_gpu():
    """Workspace of the MLP path: at least the state the method keeps (two gradient rows per worker,
    the server vectors, CADA1's stored innovations or CADA2's iterate history), growing with the
    number of workers; shapes the kernels do not cover are refused on the host."""
    from paper_2012_15469_amd import binding as b
    sizes = {}
    for rule in (1, 2):
        for M in (4, 8):
            cfg, p = _mlp_cfg(b, (784, 512, 10), M, 128, 600, rule)
            n = b._lib.cada_workspace_bytes(ctypes.byref(cfg))
            assert n > 0, b.cada_last_error()
            state = 4 * p * (2 * M + 6) + (4 * p * 2 * M if rule == 1 else 4 * p * 2 * (cfg.D + 1))
            assert n > state
            assert n < 4 * state + (1 << 28)           # and not absurdly more
            sizes[rule, M] = n
        assert sizes[rule, 8] > sizes[rule, 4]
    cfg, p = _mlp_cfg(b, (784, 512, 40), 4, 128, 600, 2)
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "32 classes" in b.cada_last_error()
    cfg, p = _mlp_cfg(b, (784, 512, 10), 4, 128, 600, 2)
    cfg.gemm_dtype = b.GEMM_FP32
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "bf16" in b.cada_last_error()
    cfg, p = _mlp_cfg(b, (784, 512, 10), 4, 128, 600, 2)
    cfg.p = p + 1
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "does not match" in b.cada_last_error()


def test_gradient_store_choices_without_gpu():
    """The bf16 gradient store: two bytes instead of four for each of the 2 M p stored values, refused where
    no kernel writes it (logistic model) or where the rule reads the stored gradients (stochastic LAG)."""
    from paper_2012_15469_amd import binding as b
    for rule in (0, 1, 2):
        cfg, p = _mlp_cfg(b, (784, 512, 10), 8, 128, 600, rule)
        n32 = b._lib.cada_workspace_bytes(ctypes.byref(cfg))
        cfg.gradient_store = b.STORE_BF16
        n16 = b._lib.cada_workspace_bytes(ctypes.byref(cfg))
        assert 0 < n16 < n32, b.cada_last_error()
        assert abs((n32 - n16) - 2 * 8 * p * 2) < 2 * 8 * 64 + 4096          # (rows are padded to 16 bytes)
    cfg, p = _mlp_cfg(b, (784, 512, 10), 8, 128, 600, 3)
    cfg.gradient_store = b.STORE_BF16
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "LAG" in b.cada_last_error()
    out = ctypes.c_void_p()
    assert b._lib.cada_init(ctypes.byref(cfg), None, ctypes.byref(out)) == -4          # CADA_EUNSUPPORTED, before any pointer is looked at
    cfg.gradient_store = 7
    assert b._lib.cada_workspace_bytes(ctypes.byref(cfg)) == 0 and "gradient_store must be" in b.cada_last_error()
    lr = b.cada_config()
    dims = (ctypes.c_int32 * 2)(54, 1)
    ns = (ctypes.c_int64 * 2)(10, 10)
    lr.M, lr.p, lr.model, lr.n_layers, lr.layer_dims, lr.B, lr.n_samples = 2, 54, 0, 1, dims, 4, ns
    lr.d_max, lr.D, lr.rule = 10, 5, 2
    assert b._lib.cada_workspace_bytes(ctypes.byref(lr)) > 0
    lr.gradient_store = b.STORE_BF16
    assert b._lib.cada_workspace_bytes(ctypes.byref(lr)) == 0 and "MLP model only" in b.cada_last_error()
