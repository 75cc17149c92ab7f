"""The C-ABI library loads and exports every symbol include/*.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if h.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
            names |= set(re.findall(r"\b(das_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    import paper_2511_13841_amd as das
    L = das.lib()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/ but not exported"


def test_error_paths_without_a_gpu_or_model():
    import paper_2511_13841_amd as das
    L = das.lib()
    assert L.das_strerror(0) == b"ok"
    assert L.das_strerror(das.DAS_ERR_NOMEM) != L.das_strerror(das.DAS_ERR_STATE)
    # null model / bad arguments are rejected before anything touches a device
    assert L.das_verify_step(None, 1, None, None, None, None, None, None, None) == das.DAS_ERR_INVALID
    assert L.das_kv_commit(None, 1, None, None, None) == das.DAS_ERR_INVALID
    assert L.das_kv_rollback(None, 0, None) == das.DAS_ERR_INVALID
    h = ctypes.c_void_p()
    assert L.das_model_load(None, 0, None, None, ctypes.byref(h)) == das.DAS_ERR_INVALID
    import das_inputs as di
    bad = das.config_for(di.MODELS["tiny"], 8, 1024, 64, 200, 64)        # (1+max_draft)*G > 256
    dummy = (ctypes.c_uint16 * 4)()
    assert L.das_model_load(ctypes.byref(bad), 0, dummy, None, ctypes.byref(h)) == das.DAS_ERR_INVALID
    bad = das.config_for(di.MODELS["tiny"].replace(head_dim=96), 8, 1024, 64, 4, 64)
    assert L.das_model_load(ctypes.byref(bad), 0, dummy, None, ctypes.byref(h)) == das.DAS_ERR_INVALID
    assert "attention" in das.kernel_classes()


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_13841_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f"{f} mentions the oracle"
