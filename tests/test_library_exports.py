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
    # the tree builder's workspace: per row 16 segment totals, the maximum (padded to 8 doubles)
    # and 32768 drawn-token bits
    assert lib.dyspec_workspace_bytes(0, ctypes.byref(c), 32000, 64, 8, 128) == 209 * (16 + 8 + 512) * 8
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


def test_misaligned_pointers_are_refused_before_any_launch():
    """Addresses that are not aligned as the header states give DYSPEC_BAD_ARG from the host-side
    validation (nothing is launched, so fake addresses are enough and no GPU is needed)."""
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    b = binding.Batch.from_sizes([40, 9], [100, 64])
    c = b._c()
    F = ctypes.c_float
    temps = (F * 2)(1.0, 1.0)
    A = 0x7f0000001000                                     # a well-aligned fake device address
    tree = binding._Tree(*[A + 0x100 * k for k in range(6)])

    def attn(q=A, kp=A, vp=A, kt=A, vt=A, mask=A, out=A, ws=None, dtype=binding.BF16):
        return lib.dyspec_tree_attn(q, kp, vp, kt, vt, mask, ctypes.byref(c), 8, 2, 128, dtype, 0.1, out, ws, 0, None)

    for name in ("q", "kp", "vp", "kt", "vt", "out", "ws"):
        assert attn(**{name: A + 8}) == -1, name           # tensors and workspace: 16 bytes
    assert attn(mask=A + 4) == -1                           # mask words: 8 bytes
    assert attn(q=A + 8, dtype=binding.F32) == -1
    # more query heads than the kernels' 32-bit row offsets reach: a shape error, not a wrong address
    assert lib.dyspec_tree_attn(A, A, A, A, A, A, ctypes.byref(c), 4096, 2, 128, binding.BF16, 0.1, A, None, 0, None) == -2
    # the fp32 / odd-size kernel reads rows four values at a time
    for hd, dt in ((66, binding.F32), (2, binding.F32), (260, binding.F32), (70, binding.BF16_WAVE)):
        assert lib.dyspec_tree_attn(A, A, A, A, A, A, ctypes.byref(c), 8, 2, hd, dt, 0.1, A, None, 0, None) == -3, hd
    assert lib.dyspec_tree_attn_layers(A, A, A + 2, A, A, A, ctypes.byref(c), 3, 1 << 20, 1 << 20, 1 << 20, 8, 2, 128,
                                       binding.BF16, 0.1, A, None, 0, None) == -1

    outs = [A] * 6

    def verify(fn, d=A, t=A, tr=tree, outs=outs):
        return fn(d, t, 1000, ctypes.byref(c), ctypes.byref(tr), temps, temps, 0, 1, *outs, None, 0, None)

    for fn in (lib.dyspec_verify, lib.dyspec_verify_bf16):
        assert verify(fn, d=A + 4) == -1 and verify(fn, t=A + 8) == -1            # logit tables: 16 bytes
        assert verify(fn, outs=[A + 8] + [A] * 5) == -1                           # row_stats: 16 bytes
        assert verify(fn, outs=[A, A + 2] + [A] * 4) == -1                        # float / int arrays: 4 bytes
        assert verify(fn, tr=binding._Tree(A, A + 2, A, A, A, A)) == -1

    def build(d=A, tr=tree, est=A, mask=A, nb=A, ws=None):
        return lib.dyspec_build_tree(d, 1000, ctypes.byref(c), temps, 0, ctypes.byref(tr), est, mask, nb, ws, 0, None)

    assert build(d=A + 4) == -1 and build(mask=A + 4) == -1 and build(est=A + 2) == -1 and build(ws=A + 4) == -1
    thr = (ctypes.c_double * 2)(0.1, 0.1)
    assert lib.dyspec_build_tree_threshold(A + 4, 1000, ctypes.byref(c), temps, thr, 0, ctypes.byref(tree), A, A, A,
                                           None, A, 1 << 30, None) == -1
    tree2 = binding._Tree(*[A + 0x1000 + 0x100 * k for k in range(6)])
    assert lib.dyspec_dfs_reorder(ctypes.byref(c), ctypes.byref(tree), ctypes.byref(tree2), A + 2, A, None) == -1
    assert lib.dyspec_dfs_reorder(ctypes.byref(c), ctypes.byref(tree), ctypes.byref(tree2), A, A + 4, None) == -1


def test_static_scratch_entry_point_refuses_oversized_batches_on_the_host():
    """The size check of dyspec_tree_attn_static_scratch comes before anything touches a GPU."""
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    b = binding.Batch.from_sizes([128], [4096])
    c = b._c()
    A = 0x7f0000001000
    assert lib.dyspec_workspace_bytes(1, ctypes.byref(c), 0, 32, 32, 128) > (8 << 20)
    st = lib.dyspec_tree_attn_static_scratch(A, A, A, A, A, A, ctypes.byref(c), 32, 32, 128, binding.BF16, 0.1, A, None)
    assert st == -4


def test_row_limits_per_entry_point():
    """Attention, reorder and verification take trees of up to 2048 rows; the builders 1024."""
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    A = 0x7f0000001000
    F = ctypes.c_float
    temps = (F * 1)(1.0)
    tree = binding._Tree(*[A + 0x100 * k for k in range(6)])
    ok, over = binding.Batch.from_sizes([2048], [10]), binding.Batch.from_sizes([2049], [10])
    assert ok.mask_words == 32 and over.mask_words == 0
    c = over._c()
    assert lib.dyspec_tree_attn(A, A, A, A, A, A, ctypes.byref(c), 8, 2, 128, binding.BF16, 0.1, A, None, 0, None) == -2
    assert lib.dyspec_verify(A, A, 100, ctypes.byref(c), ctypes.byref(tree), temps, temps, 0, 1, *([A] * 6), None, 0, None) == -2
    c = binding.Batch.from_sizes([1025])._c()
    assert lib.dyspec_build_tree(A, 100, ctypes.byref(c), temps, 0, ctypes.byref(tree), A, A, A, None, 0, None) == -2
    assert lib.dyspec_workspace_bytes(0, ctypes.byref(c), 100, 8, 2, 128) == 0
    assert lib.dyspec_build_tree_threshold_workspace_bytes(ctypes.byref(c)) == 0


def test_tree_attention_cut_by_shape():
    """How many partial results per (row tile, KV head) the workspace is sized for: the prefix splits
    that fill the chip once, plus one for the tree when that shortens the longest walk."""
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    part = 4 * 64 * (128 // 4 + 2) * 4
    for nodes, prefix, Hq, Hkv, groups, parts in [((128,), (1024,), 32, 32, 32, 5),      # four prefix splits + the tree's own
                                                 ((256,), (2048,), 40, 40, 80, 3),      # no room for a fourth workgroup per group
                                                 ((32,), (4096,), 64, 8, 16, 8),        # one tree tile: it stays with the last split
                                                 ((128, 64), (1024, 640), 8, 8, 16, 3)]:
        c = binding.Batch.from_sizes(nodes, prefix)._c()
        assert lib.dyspec_workspace_bytes(1, ctypes.byref(c), 0, Hq, Hkv, 128) == 4096 + groups * parts * part
    c = binding.Batch.from_sizes((512,), (4096,))._c()
    assert lib.dyspec_workspace_bytes(1, ctypes.byref(c), 0, 64, 8, 128) == 0           # 256 workgroups: no split


def test_prepared_call_reports_the_status_of_every_issue():
    """A prepared call is the C call with its arguments kept: each issue returns `out` or raises
    with the library's status (here a misaligned fake address: nothing is launched, no GPU needed)."""
    import pytest
    from paper_2410_11744_amd import binding
    lib = binding.load_library()
    c = binding.Batch.from_sizes([40, 9], [100, 64])._c()
    A = 0x7f0000001000
    args = (A + 8, A, A, A, A, A, ctypes.byref(c), 8, 2, 128, binding.BF16, ctypes.c_float(0.1), A, None, ctypes.c_size_t(0), None)
    call = binding.PreparedCall(lib.dyspec_tree_attn, args, (c,), "dyspec_tree_attn", "the output")
    for _ in range(2):
        with pytest.raises(binding.DyspecError) as e:
            call()
        assert e.value.status == -1
