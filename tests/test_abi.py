"""The C-ABI library loads and exports every function include/*.h declares.
No compute call is made here (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="adaptra.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
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
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert headers == ["adaptra.h", "adaptra_testing.h"]
    for header in headers:
        for name in declared_functions(header):
            assert hasattr(lib, name), f"{name} is declared in {header} but not exported"
    assert set(binding.EXPORTS) == set(declared_functions("adaptra.h"))
    assert set(binding.TESTING_EXPORTS) == set(declared_functions("adaptra_testing.h"))
    # the product header carries no test switch or probe
    assert not set(binding.TESTING_EXPORTS) & set(declared_functions("adaptra.h"))


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
    assert lib.adaptra_zb_check_inputs(None, None, None, None, None, 0, None) == binding.EINVAL
    assert lib.adaptra_zb_check_inputs(*args, 256, 64, None) == binding.EWORKSPACE


def test_static_entry_point_rejects_sizes_beyond_its_limits_without_touching_the_gpu(binding):
    lib = binding.load()
    p = binding.Params(4, 8, 1, 1, None, 0, 0)
    s = binding.Scenarios(6, 1, 1, None, None)
    too_many = binding.Candidates(binding.STATIC_MAX_CANDIDATES + 1, 1, -1)
    assert lib.adaptra_best_static(ctypes.byref(p), ctypes.byref(too_many), ctypes.byref(s), 1, 1, None, None, None) == binding.ELIMIT
    c = binding.Candidates(10, 1, -1)
    wide = binding.Scenarios(binding.STATIC_MAX_SCENARIOS + 1, 1, 1, None, None)
    assert lib.adaptra_best_static(ctypes.byref(p), ctypes.byref(c), ctypes.byref(wide), 1, 1, None, None, None) == binding.ELIMIT
    long_ = binding.Params(4, binding.STATIC_MAX_MICROBATCHES + 1, 1, 1, None, 0, 0)
    assert lib.adaptra_best_static(ctypes.byref(long_), ctypes.byref(c), ctypes.byref(s), 1, 1, None, None, None) == binding.ELIMIT
    assert lib.adaptra_best_static(None, None, None, None, None, None, None, None) == binding.EINVAL


def test_grid_limits_are_checked_before_anything_is_enqueued(binding):
    """2^31 - 1 candidates x 2^31 - 1 scenarios make more 64 x 64 tiles than a grid holds: EINVAL
    from the planning, ahead of the workspace test and of every launch."""
    lib = binding.load()
    p = binding.Params(4, 8, 1, 1, None, 0, 0)
    c = binding.Candidates(2 ** 31 - 1, 1, -1)
    s = binding.Scenarios(2 ** 31 - 1, 1, 1, None, None)
    assert lib.adaptra_best(ctypes.byref(p), ctypes.byref(c), ctypes.byref(s), 1, 1, None, None, 256, 1 << 62, None) == binding.EINVAL

