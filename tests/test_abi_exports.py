"""No GPU: the C-ABI library loads, exports every symbol include/agg.h declares, and rejects bad handles."""
import ctypes
import os
import re

import paper_2504_19442_amd as agg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "agg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_library_exports_every_declared_symbol():
    assert os.path.exists(agg.lib_path()), "build the HIP extension first"
    L = ctypes.CDLL(agg.lib_path())
    names = _declared_functions()
    assert len(names) >= 15
    assert sorted(names) == sorted(agg.EXPORTS)
    for n in names:
        assert hasattr(L, n), f"libagg.so does not export {n}"


def test_null_context_is_rejected_without_touching_the_gpu():
    L = ctypes.CDLL(agg.lib_path())
    for name in ("symm_free", "signal_reset", "agg_status"):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        args = [ctypes.c_void_p(None)] + ([ctypes.c_void_p(None)] if name == "signal_reset" else [])
        assert f(*args) == agg.ERR_INVALID_ARG
    assert agg.agg_strerror(agg.ERR_TIMEOUT).startswith("a kernel gave up")
    assert agg.agg_strerror(0) == "ok"


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2504_19442_amd", "binding.py")).read()
    assert "oracle" not in src and "numpy" not in src
