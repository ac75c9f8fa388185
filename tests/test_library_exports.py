"""CPU-side checks of the C-ABI library: it loads and exports every symbol the header
declares; host-side validation returns error codes without touching a GPU."""
import ctypes
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dyspec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dyspec_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_host_validation_without_gpu():
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    assert binding.status_string(0) == "ok"
    b = binding.Batch.from_sizes([10, 70, 129])
    assert b.mask_words == 3
    c = b._c()
    # the tree builder's workspace: per row 16*512 segment sums, 16 totals, the maximum (padded
    # to 8 doubles) and 32768 drawn-token bits
    assert lib.dyspec_workspace_bytes(0, ctypes.byref(c), 32000, 64, 8, 128) == 209 * (16 * 512 + 16 + 8 + 512) * 8
    assert lib.dyspec_workspace_bytes(1, ctypes.byref(c), 32000, 64, 8, 128) == 0
    assert lib.dyspec_workspace_bytes(2, ctypes.byref(c), 32000, 64, 8, 128) == 0
    # null pointers are refused before any launch
    st = lib.dyspec_build_tree(None, 100, ctypes.byref(c), None, 0, None, None, None, None, None, 0, None)
    assert st == -1
    too_many = binding.Batch.from_sizes([1] * 65)
    assert too_many.mask_words == 0           # invalid batch
    bad = binding.Batch(np.array([0, 5, 3], np.int32), np.zeros(2, np.int32), np.zeros(3, np.int64))
    cb = bad._c()
    assert lib.dyspec_build_tree(None, 100, ctypes.byref(cb), None, 0, None, None, None, None, None, 0, None) == -2
