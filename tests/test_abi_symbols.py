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
    out = ctypes.c_void_p()
    cfg.p = 54
    assert b._lib.cada_init(ctypes.byref(cfg), None, ctypes.byref(out)) == -1     # theta0 NULL
    assert b._lib.cada_step(None, None, None) == -1
