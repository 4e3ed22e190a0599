"""Re-exports the input fingerprint used by tests/golden/make_goldens.py."""
import importlib.util
import os

_spec = importlib.util.spec_from_file_location(
    "make_goldens", os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "make_goldens.py"))
_mod = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(_mod)
fingerprint = _mod.fingerprint
CASES = _mod.CASES
