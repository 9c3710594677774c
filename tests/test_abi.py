"""Host-side checks of the C ABI: the library loads and exports every function that
include/gcaps_rta.h declares; argument errors are reported without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    lib = os.path.join(ROOT, "paper_2406_05221_amd", "libgcaps_rta.so")
    if not os.path.exists(lib):
        from paper_2406_05221_amd import build
        build.build_hip()
    from paper_2406_05221_amd import binding as B
    return B


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gcaps_rta.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gcaps_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported(binding):
    names = declared_functions()
    assert names == sorted(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name


def test_strerror_covers_every_code(binding):
    seen = {binding.gcaps_strerror(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and "unknown" in binding.gcaps_strerror(-99)


def test_argument_errors_need_no_device(binding):
    lib = ctypes.CDLL(binding.LIB_PATH)
    lib.gcaps_create.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    assert lib.gcaps_create(None, 0, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_rta_batch(None, None, 3, 0, None, None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_rta_batch_device(None, None, 3, 0, None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_status(None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_set_binning(None, 1) == binding.GCAPS_EINVAL
    assert lib.gcaps_set_continue_after_miss(None, 1) == binding.GCAPS_EINVAL
    assert lib.gcaps_last_wide_count(None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_gprio_assign_batch(None, None, 0, None, None, None, None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_gprio_assign_batch_device(None, None, 0, None, None, None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_gprio_rta_batch(None, None, 0, None, None, None, None) == binding.GCAPS_EINVAL
    assert lib.gcaps_gprio_rta_batch_device(None, None, 0, None, None, None) == binding.GCAPS_EINVAL
    lib.gcaps_destroy.argtypes = [ctypes.c_void_p]
    lib.gcaps_destroy(None)


def test_create_fails_cleanly_without_a_gpu(binding):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(binding.GcapsError) as e:
        binding.gcaps_create(0)
    assert e.value.code == binding.GCAPS_EDEVICE
