"""Host-side checks of the C ABI: the shared library loads without a GPU and exports
every function include/knm.h declares (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "knm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:int|size_t|const char \*)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_declares_the_named_entry_points():
    names = _declared()
    for required in ("knm_prod", "knm_t_y", "precond_build", "falkon_fit", "falkon_predict"):
        assert required in names


def test_library_exports_every_declared_symbol():
    import paper_2006_10350_amd as pkg

    if not os.path.exists(pkg.LIB_PATH):
        pytest.fail("libknm.so is not built: run python paper_2006_10350_amd/build.py")
    lib = ctypes.CDLL(pkg.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in knm.h but not exported"
    assert sorted(pkg.SIGNATURES) == _declared()


def test_static_queries_need_no_gpu():
    import paper_2006_10350_amd as pkg

    lib = pkg.load_library()
    assert lib.knm_max_d() >= 28 and lib.knm_max_t() >= 10
    assert lib.knm_strerror(0) == b"ok"
    assert b"positive definite" in lib.knm_strerror(-5)
    assert lib.knm_workspace_bytes(20000, 1000, 8, 1) >= 20000 * 4
    assert lib.knm_workspace_bytes(0, 1000, 8, 1) == 0
    # null context is rejected, not dereferenced
    assert lib.knm_destroy(None) == -1
    assert lib.knm_set_timing(None, 1) == -1


def test_no_cpu_fallback_without_gpu():
    import torch

    import paper_2006_10350_amd as pkg

    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        pkg.Context()
