"""The C-ABI library loads and exports every function include/adaptra.h declares.
No compute call is made here (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "adaptra.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adaptra_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def binding():
    from paper_2504_19232_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2504_19232_amd import build
        build.build_library()
    return b


def test_header_declares_the_entry_points():
    names = declared_functions()
    for n in ("adaptra_eval", "adaptra_best", "adaptra_check_inputs", "adaptra_workspace_bytes"):
        assert n in names


def test_library_exports_every_declared_symbol(binding):
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in adaptra.h but not exported"
    assert set(binding.EXPORTS) == set(declared_functions())


def test_host_only_calls(binding):
    assert binding.adaptra_version() >= 1
    n = binding.adaptra_workspace_bytes(8, 32, 16384, 64)
    assert n > 0 and n % 256 == 0
    assert binding.adaptra_workspace_bytes(0, 32, 10, 10) == 0       # S out of range
    assert binding.adaptra_workspace_bytes(65, 32, 10, 10) == 0
    assert binding.adaptra_workspace_bytes(8, 0, 10, 10) == 0
    assert binding.adaptra_workspace_bytes(8, 32, 0, 10) == 0
    assert binding.adaptra_workspace_bytes(8, 32, 2 ** 31, 10) == 0
    prev = binding.adaptra_set_kernel_mode(1)
    assert binding.adaptra_set_kernel_mode(prev) == 1
    assert binding.adaptra_set_kernel_mode(7) == -1


def test_null_arguments_are_rejected_without_touching_the_gpu(binding):
    lib = binding.load()
    assert lib.adaptra_eval(None, None, None, None, None, None, None, 0, None) == binding.EINVAL
    assert lib.adaptra_best(None, None, None, None, None, None, None, None, 0, None) == binding.EINVAL
    p = binding.Params(4, 8, 1, 1, None, 0, 0)                        # non-null dummies, never dereferenced
    c = binding.Candidates(10, 1, -1)
    s = binding.Scenarios(10, 1, 1, None, None)
    rc = lib.adaptra_eval(ctypes.byref(p), ctypes.byref(c), ctypes.byref(s), 1, None, 1, None, 0, None)
    assert rc == binding.EWORKSPACE


def test_zb_and_search_reject_bad_arguments_without_touching_the_gpu(binding):
    lib = binding.load()
    assert lib.adaptra_zb_eval(None, None, None, None, 0, None, None, None, 0, None) == binding.EINVAL
    p = binding.Params(4, 8, 1, 1, None, 0, 0)                        # non-null dummies, never dereferenced
    c = binding.Candidates(10, 1, -1)
    s = binding.Scenarios(6, 1, 1, None, None)
    args = (ctypes.byref(p), 1, ctypes.byref(c), ctypes.byref(s))
    assert lib.adaptra_zb_eval(*args, 6, 1, None, 256, 1 << 30, None) == binding.EINVAL      # plan scenario out of range
    assert lib.adaptra_zb_eval(*args, -2, 1, None, 256, 1 << 30, None) == binding.EINVAL
    assert lib.adaptra_zb_eval(*args, -1, 1, None, 256, 64, None) == binding.EWORKSPACE      # too small
    assert lib.adaptra_zb_eval(*args, -1, 1, None, 257, 1 << 30, None) == binding.EWORKSPACE  # misaligned
    big = binding.Params(65, 8, 1, 1, None, 0, 0)
    assert lib.adaptra_zb_workspace_bytes(ctypes.byref(big), 10, 6) == 0                      # more than 64 stages
    assert lib.adaptra_zb_workspace_bytes(ctypes.byref(p), 10, 6) > 0
    assert lib.adaptra_search_workspace_bytes(ctypes.byref(p), 6, 2) == 0                     # unknown neighbourhood
    assert lib.adaptra_search(ctypes.byref(p), ctypes.byref(s), 1, 0, 0, 1, 1, None, None, 256, 1 << 30, None) == binding.EINVAL

