"""The C-ABI library loads and exports every symbol include/hla.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hla_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_core_calls():
    names = _declared_functions()
    for n in ("hla_create", "hla_forward", "hla_backward", "hla_destroy"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2602_12128_amd import binding
    assert os.path.exists(binding.LIB_PATH), "build libhla.so first (python -m paper_2602_12128_amd.build)"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} declared in hla.h but not exported"
    assert set(binding.EXPORTS) == set(_declared_functions())


def test_status_strings_and_null_handling_without_gpu():
    from paper_2602_12128_amd import binding
    lib = binding.load_library()
    assert binding.status_string(0) == "HLA_OK"
    assert binding.status_string(2) == "HLA_ERR_UNSUPPORTED"
    assert lib.hla_destroy(None) == 0
    assert lib.hla_active_path(None) == -1
    # argument errors are caught before any device call
    assert lib.hla_create(None, None) == 1
    h = ctypes.c_void_p()
    cfg = binding.hla_config(48, 6, 3, 1e-6, 1, 0, 0, 1, 1, 1)  # head_dim 48: no kernel
    assert lib.hla_create(ctypes.byref(cfg), ctypes.byref(h)) == 2 and not h
    cfg = binding.hla_config(128, 6, 3, 1e-6, 7, 0, 0, 1, 1, 1)  # bad dtype
    assert lib.hla_create(ctypes.byref(cfg), ctypes.byref(h)) == 1 and not h
    cfg = binding.hla_config(128, 7, 3, 1e-6, 1, 0, 0, 1, 1, 1)  # 7^3 > 256
    assert lib.hla_create(ctypes.byref(cfg), ctypes.byref(h)) == 2 and not h
