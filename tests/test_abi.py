"""Host-side checks of the C ABI that need no GPU: the library loads and exports what include/idkm.h declares."""
import ctypes
import os
import re

import pytest

from paper_2312_07759_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "idkm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(idkm_[a-zA-Z_0-9]+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    names = _declared()
    for must in ("idkm_create", "idkm_destroy", "idkm_forward", "idkm_backward", "idkm_last_error"):
        assert must in names


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.load_library()
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_version_limits_and_status_strings_need_no_device():
    lib = binding.load_library()
    assert lib.idkm_version() >= 100
    lim = binding.limits()
    assert lim["max_k"] >= 256 and lim["max_d"] >= 4 and lim["max_kd"] >= 1024
    assert lib.idkm_status_string(0) == b"ok"
    assert lib.idkm_status_string(5) == b"no forward state"


def test_null_arguments_are_rejected_without_touching_a_device():
    lib = binding.load_library()
    assert lib.idkm_create(None, 0) == 1
    assert lib.idkm_destroy(None) == 1
    assert lib.idkm_set_path(None, 0) == 1
    assert lib.idkm_last_error(None) == b"null context"
    info = binding.IdkmInfo()
    assert lib.idkm_forward(None, None, 1, 1, None, 1, 1.0, 0.0, 1, 0, None, None, None, None,
                            ctypes.byref(info), None) == 1
    assert lib.idkm_backward(None, None, 0, 0.0, 1, 1.0, None, None, None) == 1


def test_create_without_a_gpu_reports_a_device_error():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = binding.load_library()
    h = ctypes.c_void_p()
    st = lib.idkm_create(ctypes.byref(h), 0)
    assert st == 3 and not h.value
    with pytest.raises(binding.IdkmError):
        binding.Context(0)
