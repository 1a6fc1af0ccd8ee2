"""The C-ABI library loads without a GPU and exports every function include/estimator.h declares;
argument errors that are caught before any device work are reported as error codes."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1812_01776_amd import estimator as binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "estimator.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(estimator_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load_library()


def test_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert len(names) >= 9
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == names


def test_exports_nothing_the_header_does_not_declare():
    """Every dynamic function symbol the library defines with C linkage is declared in include/estimator.h."""
    import subprocess
    out = subprocess.check_output(["nm", "-D", "--defined-only", binding.LIB_PATH], text=True)
    exported = sorted(parts[2] for parts in (l.split() for l in out.splitlines())
                      if len(parts) == 3 and parts[1] in "TW" and not parts[2].startswith("_"))
    assert exported == _declared_functions(), exported


def test_create_rejects_bad_arguments_before_touching_the_device(lib):
    h = ctypes.c_void_p()
    assert lib.estimator_create(None, None, ctypes.byref(h)) == binding.EST_EINVAL
    assert lib.estimator_create(None, None, None) == binding.EST_EINVAL
    lat = np.ones((2, 1, 4), np.uint32)
    cost = np.ones((2, 1), np.uint64)

    def create(S, off, idx, lat=lat, H=1, Bmax=4):
        off = np.asarray(off, np.uint32); idx = np.asarray(idx, np.uint32)
        dag = binding._Dag(S, off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
        prof = binding._Profiles(H, Bmax, lat.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                                 cost.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
        hh = ctypes.c_void_p()
        rc = lib.estimator_create(ctypes.byref(dag), ctypes.byref(prof), ctypes.byref(hh))
        if rc == 0:
            lib.estimator_destroy(hh)
        return rc

    assert create(0, [0], [0]) == binding.EST_EINVAL                 # no stages
    assert create(33, [0] * 34, [0]) == binding.EST_EINVAL           # too many stages
    assert create(2, [0, 0, 1], [1]) == binding.EST_EINVAL           # parent index >= child
    assert create(2, [0, 1, 1], [0]) == binding.EST_EINVAL           # a root with a parent entry
    assert create(2, [0, 0, 1], [0], Bmax=65) == binding.EST_EINVAL  # Bmax out of range
    assert create(2, [0, 0, 1], [0], H=0) == binding.EST_EINVAL
    zero = lat.copy(); zero[1, 0, 2] = 0
    assert create(2, [0, 0, 1], [0], lat=zero) == binding.EST_EINVAL  # a zero latency entry
    lib.estimator_destroy(None)                                       # no-op
    assert lib.estimator_last_error(None) == b"invalid handle"
    assert lib.estimator_workspace_bytes(None, ctypes.c_uint64(10), ctypes.c_uint64(10)) == 0


def test_no_fallback_without_a_gpu(lib):
    """On a machine without a GPU a valid create must fail with EST_EDEVICE, not fall back."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lat = np.ones((1, 1, 1), np.uint32)
    with pytest.raises(binding.EstimatorError) as ei:
        binding.Estimator([[]], lat, np.ones((1, 1), np.uint64))
    assert ei.value.code == binding.EST_EDEVICE
