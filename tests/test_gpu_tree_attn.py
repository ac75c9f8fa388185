"""GPU parity: dyspec_tree_attn against the fp64 oracle (through the C ABI)."""
import math

import numpy as np
import pytest

import oracle
from helpers import ATTN_TOL, oracle_attention_rows

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


def random_parents(n, rng, chain=False, shallow=False):
    if chain:
        return np.arange(-1, n - 1, dtype=np.int32)
    par = np.full(n, -1, np.int32)
    if shallow:                                   # every node hangs below one of the first few
        for i in range(1, n):
            par[i] = int(rng.integers(0, min(i, 6)))
        return par
    for i in range(1, n):
        par[i] = int(rng.integers(max(0, i - 12), i)) if rng.random() < 0.7 else int(rng.integers(0, i))
    return par


def make_case(nodes, prefix, Hq, Hkv, d, dtype, seed, chain=False, shallow=False, qscale=1.0, ramp=0.0):
    rng = np.random.default_rng(seed)
    g = torch.Generator().manual_seed(seed)
    dt = torch.float32 if dtype == "f32" else torch.bfloat16
    tn, tp = sum(nodes), sum(prefix)
    mk = lambda *sh: torch.randn(sh, generator=g, dtype=torch.float32).to(dt)
    q, kp, vp, kt, vt = mk(tn, Hq, d), mk(tp, Hkv, d), mk(tp, Hkv, d), mk(tn, Hkv, d), mk(tn, Hkv, d)
    if qscale != 1.0:
        q = (q.float() * qscale).to(dt)
    if ramp and tp:                               # later prefix keys score higher and higher
        f = 1.0 + ramp * torch.arange(tp, dtype=torch.float32) / tp
        kp = (kp.float() * f[:, None, None]).to(dt)
    words = (max(nodes) + 63) // 64
    mask = np.zeros((tn, words), np.uint64)
    off = 0
    for n in nodes:
        m = oracle.ancestor_mask(random_parents(n, rng, chain, shallow))
        mask[off:off + n, :m.shape[1]] = m
        off += n
    return q, kp, vp, kt, vt, mask


def run_and_compare(dy, nodes, prefix, Hq, Hkv, d, dtype, seed, chain=False, api_dtype=None, max_rows=4000,
                    shallow=False, qscale=1.0, ramp=0.0):
    print(f"attn case nodes={nodes} prefix={prefix} H={Hq}/{Hkv} d={d} {dtype} seed={seed}", flush=True)
    batch = dy.Batch.from_sizes(nodes, prefix)
    q, kp, vp, kt, vt, mask = make_case(nodes, prefix, Hq, Hkv, d, dtype, seed, chain, shallow, qscale, ramp)
    scale = 1.0 / math.sqrt(d)
    dev = lambda t: t.cuda() if t.numel() else torch.empty(t.shape, dtype=t.dtype, device="cuda")
    mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
    out = dy.tree_attn(dev(q), dev(kp), dev(vp), dev(kt), dev(vt), mask_dev, batch, scale, dtype=api_dtype)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    host = [t.float().numpy() for t in (q, kp, vp, kt, vt)]
    rng = np.random.default_rng(seed + 1)
    worst = 0.0
    for s, n in enumerate(nodes):
        total = n * Hq
        if total <= max_rows:
            rj, rh = np.divmod(np.arange(total), Hq)
        else:
            pick = rng.choice(total, max_rows, replace=False)
            rj, rh = np.divmod(pick, Hq)
        want = oracle_attention_rows(*host, mask, batch, s, scale, rj, rh)
        a = int(batch.node_offset[s])
        err = np.abs(got[a + rj, rh] - want).max()
        worst = max(worst, float(err))
    assert np.isfinite(got).all()
    assert worst <= ATTN_TOL[dtype], f"max abs error {worst}"
    return worst


def test_tiny_fp32_config(dy):
    run_and_compare(dy, (32,), (128,), 8, 8, 64, "f32", 0)


@pytest.mark.parametrize("nodes,prefix,Hq,Hkv,d,seed", [
    ((32,), (128,), 8, 8, 64, 1),            # one 128-row tile per 4 heads... G=1, partial tiles
    ((128,), (1024,), 4, 4, 128, 2),         # 7B-shaped slice (4 of 32 heads)
    ((100,), (1000,), 8, 2, 128, 3),         # GQA 4, ragged prefix tile and ragged tree tile
    ((512,), (333,), 16, 2, 128, 4),         # 70B-shaped GQA 8, many row tiles, odd prefix
    ((70,), (0,), 4, 2, 128, 5),             # no prefix at all
    ((1,), (65,), 8, 8, 128, 6),             # root only
    ((64, 7, 200, 1), (100, 1, 513, 64), 8, 2, 128, 7),   # ragged batch
    ((300,), (64,), 6, 2, 64, 8),            # head_dim 64, G = 3 (rows of a node split across blocks)
    ((768,), (129,), 8, 1, 128, 9),          # widest supported tree slice: 12 mask words
])
def test_bf16_matrix_core_kernel(dy, nodes, prefix, Hq, Hkv, d, seed):
    run_and_compare(dy, nodes, prefix, Hq, Hkv, d, "bf16", seed)


def test_bf16_long_prefix_wide_tree(dy):
    # nine whole prefix tiles and a ragged one, a tree of sixteen key tiles
    run_and_compare(dy, (1024,), (64 * 9 + 5,), 8, 1, 128, "bf16", 12)


def test_bf16_shallow_tree_leaves_tiles_out(dy):
    # ancestors all sit in the first key tile: most tree tiles hold no visible key for a row tile
    run_and_compare(dy, (1024, 300), (512, 700), 8, 2, 128, "bf16", 13, shallow=True)


def test_bf16_rising_scores_raise_the_reference(dy):
    # large scores that keep growing along the prefix: the running maximum is raised many times
    run_and_compare(dy, (96,), (2048,), 8, 2, 128, "bf16", 14, qscale=3.0, ramp=3.0)
    run_and_compare(dy, (200,), (640,), 4, 4, 64, "bf16", 15, qscale=4.0, ramp=2.0)


@pytest.mark.parametrize("nodes,prefix,Hq,Hkv,groups,parts", [
    ((32,), (4096,), 64, 8, 16, 8),               # 70B shape, narrow tree: 16 workgroups become 128
    ((128,), (1024 + 37,), 8, 8, 8, 4),           # ragged last prefix tile; the last split holds the tree alone already
    ((40, 9), (64 * 22, 64 * 17 + 1), 4, 2, 4, 4),   # shares of uneven size, ragged batch
    ((128,), (1024,), 32, 32, 32, 5),             # 7B shape: four prefix splits and one for the two tree tiles
    ((128, 64), (1024, 640), 8, 8, 16, 3),        # ragged batch with a split for the trees: two, one tree tiles
])
def test_bf16_prefix_split_matches_unsplit_and_oracle(dy, nodes, prefix, Hq, Hkv, groups, parts):
    batch = dy.Batch.from_sizes(nodes, prefix)
    q, kp, vp, kt, vt, mask = make_case(nodes, prefix, Hq, Hkv, 128, "bf16", 21)
    scale = 1.0 / math.sqrt(128)
    mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
    args = [t.cuda() for t in (q, kp, vp, kt, vt)]
    need = dy.load_library().dyspec_workspace_bytes(1, __import__("ctypes").byref(batch._c()), 0, Hq, Hkv, 128)
    # arrival counters, then per (row tile, KV head) and part 4 x 64 lanes x (32 + 2) words
    assert need == 4096 + groups * parts * 4 * 64 * 34 * 4, "the cut this case is meant to exercise"
    split = dy.tree_attn(*args, mask_dev, batch, scale)
    whole = dy.tree_attn(*args, mask_dev, batch, scale, use_workspace=False)
    torch.cuda.synchronize()
    # same products; every split's share of a row is rounded to bf16 before the merge
    assert float((split.float() - whole.float()).abs().max()) <= 2.0 ** -6
    # the merge sums the parts in split order whoever performs it: the same bits on every launch
    for _ in range(3):
        again = dy.tree_attn(*args, mask_dev, batch, scale)
        assert torch.equal(again.view(torch.int16), split.view(torch.int16))
    # and the arrival counters at the head of the workspace are zero again for the next call
    from paper_2410_11744_amd import binding
    torch.cuda.synchronize()
    ws = binding._scratch_cache[str(args[0].device)]
    assert int(ws[:1024].view(torch.int32).abs().max().item()) == 0
    run_and_compare(dy, nodes, prefix, Hq, Hkv, 128, "bf16", 21)


def test_bf16_prefix_split_head_dim_64(dy):
    """The split walk and its merged, staged rows at head_dim 64 (half rows of 64 bytes), with a ragged
    last row tile and a tree that gets a split of its own."""
    import ctypes
    for nodes, prefix, Hq, Hkv, seed in (((70,), (2048 + 5,), 8, 8, 31), ((128, 33), (1024, 700), 4, 4, 32)):
        batch = dy.Batch.from_sizes(nodes, prefix)
        assert dy.load_library().dyspec_workspace_bytes(1, ctypes.byref(batch._c()), 0, Hq, Hkv, 64) > 0, "meant to be split"
        run_and_compare(dy, nodes, prefix, Hq, Hkv, 64, "bf16", seed)
        q, kp, vp, kt, vt, mask = make_case(nodes, prefix, Hq, Hkv, 64, "bf16", seed)
        args = [t.cuda() for t in (q, kp, vp, kt, vt)]
        mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
        split = dy.tree_attn(*args, mask_dev, batch, 0.125)
        whole = dy.tree_attn(*args, mask_dev, batch, 0.125, use_workspace=False)
        torch.cuda.synchronize()
        assert float((split.float() - whole.float()).abs().max()) <= 2.0 ** -6


def test_split_needs_zeroed_counters_only_once(dy):
    """A caller's own workspace: cleared once after allocation, then used for calls of different shapes
    and split counts in a row, never cleared again; results equal to the unsplit call's within the
    bf16 rounding of the parts."""
    import ctypes
    lib = dy.load_library()
    ws = torch.zeros(3 << 20, dtype=torch.float32, device="cuda")            # 12 MB, zero-filled once
    for k, (nodes, prefix, Hq, Hkv) in enumerate([((32,), (4096,), 64, 8), ((128,), (1024,), 8, 8), ((40, 9), (64 * 22, 64 * 17 + 1), 4, 2),
                                                  ((32,), (4096,), 64, 8)]):
        batch = dy.Batch.from_sizes(nodes, prefix)
        q, kp, vp, kt, vt, mask = make_case(nodes, prefix, Hq, Hkv, 128, "bf16", 40 + k)
        args = [t.cuda() for t in (q, kp, vp, kt, vt)]
        mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
        cb = batch._c()
        need = lib.dyspec_workspace_bytes(1, ctypes.byref(cb), 0, Hq, Hkv, 128)
        assert 0 < need <= ws.numel() * 4
        out = torch.empty_like(args[0])
        st = lib.dyspec_tree_attn(*[t.data_ptr() for t in args], mask_dev.data_ptr(), ctypes.byref(cb), Hq, Hkv, 128, dy.BF16,
                                  ctypes.c_float(1.0 / math.sqrt(128)), out.data_ptr(), ws.data_ptr(), ctypes.c_size_t(need),
                                  torch.cuda.current_stream().cuda_stream)
        assert st == 0
        whole = dy.tree_attn(*args, mask_dev, batch, 1.0 / math.sqrt(128), use_workspace=False)
        torch.cuda.synchronize()
        assert float((out.float() - whole.float()).abs().max()) <= 2.0 ** -6
        assert int(ws[:1024].view(torch.int32).abs().max().item()) == 0


def test_bf16_tree_only_large_trees(dy):
    # no prefix and a short one ahead of sixteen tree tiles: the tile set is agreed on before the first loads
    run_and_compare(dy, (1024,), (0,), 8, 1, 128, "bf16", 16)
    run_and_compare(dy, (1024, 640), (0, 100), 4, 4, 128, "bf16", 17, shallow=True)
    run_and_compare(dy, (900,), (130,), 8, 8, 64, "bf16", 18, shallow=True)


def test_bf16_chain_tree_is_causal(dy):
    run_and_compare(dy, (130,), (70,), 4, 2, 128, "bf16", 11, chain=True)


@pytest.mark.parametrize("dtype,api", [("f32", None), ("bf16", 0x101)])
def test_per_wave_kernel_odd_head_dim(dy, dtype, api):
    run_and_compare(dy, (40, 9), (77, 3), 6, 3, 80, dtype, 12, api_dtype=api)


@pytest.mark.parametrize("nodes,prefix,Hq,Hkv,d,dtype,api,seed", [
    ((7, 130), (0, 300), 2, 1, 4, "f32", None, 40),          # one 16-byte piece per row; a sequence without prefix
    ((65,), (1000,), 3, 3, 64, "f32", None, 41),            # several trips per wavefront, 64 keys each
    ((33, 1), (257, 5), 4, 2, 192, "f32", None, 42),        # three pieces per lane
    ((20, 70), (129, 64), 2, 2, 256, "f32", None, 43),      # four pieces per lane
    ((50,), (90,), 4, 1, 252, "bf16", 0x101, 44),           # last piece of the lane missing for lanes 15 of 16
    ((300,), (17,), 2, 2, 128, "bf16", 0x101, 45),          # more tree keys than prefix keys, five mask words
    ((1, 1, 1), (0, 1, 3), 2, 2, 8, "f32", None, 46),       # roots only: wavefronts and groups without any key
])
def test_per_row_kernel_piece_counts_and_key_splits(dy, nodes, prefix, Hq, Hkv, d, dtype, api, seed):
    """The fp32 / odd-size kernel over its four piece counts, head sizes that leave lanes without
    a piece, walks shorter than one wavefront's run and walks of many runs."""
    run_and_compare(dy, nodes, prefix, Hq, Hkv, d, dtype, seed, api_dtype=api)


def test_unsupported_head_dim_is_rejected(dy):
    batch = dy.Batch.from_sizes([4], [4])
    z = lambda *sh: torch.zeros(sh, dtype=torch.bfloat16, device="cuda")
    mask = torch.zeros((4, 1), dtype=torch.int64, device="cuda")
    with pytest.raises(dy.DyspecError) as e:
        dy.tree_attn(z(4, 2, 96), z(4, 2, 96), z(4, 2, 96), z(4, 2, 96), z(4, 2, 96), mask, batch, 0.1)
    assert e.value.status == -3


def test_widest_batch_of_sequences(dy):
    """64 sequences (the batch limit) of a few rows each, ragged prefixes, some without prefix."""
    rng = np.random.default_rng(640)
    nodes = tuple(int(x) for x in rng.integers(1, 24, 64))
    prefix = tuple(int(x) for x in rng.choice([0, 1, 63, 64, 65, 130], 64))
    run_and_compare(dy, nodes, prefix, 8, 2, 128, "bf16", 64)
    run_and_compare(dy, nodes, prefix, 4, 4, 64, "f32", 65)
