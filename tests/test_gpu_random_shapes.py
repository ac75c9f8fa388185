"""GPU parity on seeded random shapes: ragged batches, odd sizes and mixed options drawn from the
ranges the library accepts, each checked against the oracle like the hand-picked cases."""
import math

import numpy as np
import pytest

import oracle
from helpers import build_in_full, next_seed, verify_in_full
from test_gpu_tree_attn import run_and_compare
from test_gpu_tree_attn_layers import check_layers, stacked_case
from test_gpu_threshold import compare_threshold_trees

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


def threshold_in_full(dy, draft_dev, draft_host, batch, temps, thr, seed, tries=8):
    """dyspec_build_tree_threshold against the oracle; a seed at which the oracle took a decision at a
    margin below the bar is followed by the next one until every sequence was compared row by row."""
    for k in range(tries):
        sd = next_seed(seed, k)
        built, _ = dy.build_tree_threshold(draft_dev, batch, temps, thr, sd)
        torch.cuda.synchronize()
        if compare_threshold_trees(built, batch, draft_host, temps, thr, sd) == batch.n_seq:
            return built
    raise AssertionError("no seed gave threshold-builder margins above the bar in every sequence")


HEADS = [(8, 8), (8, 2), (4, 1), (6, 2), (16, 4), (12, 12), (5, 5)]


@pytest.mark.parametrize("seed", range(16))
def test_attention_random_shapes(dy, seed):
    rng = np.random.default_rng(9000 + seed)
    n_seq = int(rng.integers(1, 6))
    nodes = tuple(int(x) for x in rng.integers(1, 260, n_seq))
    prefix = tuple(int(x) for x in rng.choice([0, 1, 17, 64, 65, 127, 128, 300, 513, 700], n_seq))
    Hq, Hkv = HEADS[int(rng.integers(0, len(HEADS)))]
    d = int(rng.choice([64, 128]))
    run_and_compare(dy, nodes, prefix, Hq, Hkv, d, "bf16", 9100 + seed, max_rows=1200,
                    shallow=bool(rng.integers(0, 2)))
    if seed % 4 == 0:                                   # the stacked call on the same kind of shape
        L = int(rng.integers(2, 4))
        batch = dy.Batch.from_sizes(nodes, prefix)
        stack, mask = stacked_case(L, nodes, prefix, Hq, Hkv, d, "bf16", 9200 + seed)
        dev = [t.cuda() if t.numel() else torch.empty(t.shape, dtype=t.dtype, device="cuda") for t in stack]
        out = dy.tree_attn_layers(*dev, torch.from_numpy(mask.view(np.int64)).cuda(), batch, 1.0 / math.sqrt(d))
        torch.cuda.synchronize()
        check_layers(dy, out, stack, mask, batch, nodes, Hq, "bf16", 1.0 / math.sqrt(d), seed, max_rows=600)


@pytest.mark.parametrize("seed", range(12))
def test_build_and_verify_random_shapes(dy, seed):
    rng = np.random.default_rng(9500 + seed)
    n_seq = int(rng.integers(1, 6))
    nodes = tuple(int(x) for x in rng.integers(1, 130, n_seq))
    V = int(rng.choice([5, 77, 1000, 4096, 5003, 12000]))
    td = tuple(float(x) for x in rng.choice([0.5, 0.7, 1.0, 1.3], n_seq))
    tt = tuple(float(x) for x in rng.choice([0.0, 0.6, 1.0], n_seq))
    sigma, tsigma = float(rng.choice([1.0, 2.5, 4.0])), float(rng.choice([0.3, 1.0, 2.0]))
    print(f"random build/verify nodes={nodes} V={V} td={td} tt={tt}", flush=True)
    d = (rng.standard_normal((sum(nodes), V)) * sigma).astype(np.float32)
    t = (d + rng.standard_normal((sum(nodes), V)) * tsigma).astype(np.float32)
    bf16 = seed % 3 == 2
    batch = dy.Batch.from_sizes(nodes)
    dd, tg = torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda()
    # the builder reads the fp32 table (values rounded to bf16 tie often, and a tie between two open
    # positions is a decision of margin 0); verification below reads the rounded tables
    built, _, _ = build_in_full(dy, dd, d, batch, nodes, td, seed)
    g = {k: getattr(built.tree, k).cpu().numpy() for k in ("token", "first_child", "next_sibling")}
    trees = [tuple(g[k][int(batch.node_offset[s]):int(batch.node_offset[s + 1])] for k in ("token", "first_child", "next_sibling"))
             for s in range(n_seq)]
    if bf16:                                            # bf16 tables for verification: both sides read the rounded values
        vd, vt = dd.to(torch.bfloat16), tg.to(torch.bfloat16)
        d, t = vd.float().cpu().numpy(), vt.float().cpu().numpy()
    else:
        vd, vt = dd, tg
    for bonus in (True, False):
        verify_in_full(lambda sd: dy.verify(vd, vt, batch, built.tree, td, tt, sd, emit_bonus=bonus),
                       batch, trees, d, t, td, tt, 77 + seed, emit_bonus=bonus)


@pytest.mark.parametrize("seed", range(8))
def test_threshold_builder_random_shapes(dy, seed):
    rng = np.random.default_rng(9800 + seed)
    n_seq = int(rng.integers(1, 5))
    nodes = tuple(int(x) for x in rng.integers(1, 200, n_seq))
    V = int(rng.choice([9, 130, 1000, 4096, 5003]))
    temps = tuple(float(x) for x in rng.choice([0.5, 0.7, 1.0], n_seq))
    thr = tuple(float(x) for x in rng.choice([0.3, 0.1, 0.03, 0.01, 0.003], n_seq))
    print(f"random threshold nodes={nodes} V={V} t={thr}", flush=True)
    d = (rng.standard_normal((sum(nodes), V)) * float(rng.choice([2.0, 4.0]))).astype(np.float32)
    batch = dy.Batch.from_sizes(nodes)
    built = threshold_in_full(dy, torch.from_numpy(d).cuda(), d, batch, temps, thr, seed)
    # and a depth-first renaming of whatever was built keeps verification's outcome
    re = dy.dfs_reorder(built.tree, batch)
    torch.cuda.synchronize()
    par = built.tree.parent.cpu().numpy()
    fc, ns = built.tree.first_child.cpu().numpy(), built.tree.next_sibling.cpu().numpy()
    order = re.order.cpu().numpy()
    for s in range(n_seq):
        a, b = int(batch.node_offset[s]), int(batch.node_offset[s + 1])
        np.testing.assert_array_equal(order[a:b], oracle.dfs_order(par[a:b], fc[a:b], ns[a:b]))


@pytest.mark.parametrize("seed", range(4))
def test_builders_large_random_shapes(dy, seed):
    """Trees of 300 to 1024 rows over large vocabularies: the greedy builder against the oracle and
    against its own form without a workspace (bit for bit), the threshold builder against the oracle."""
    rng = np.random.default_rng(77000 + seed)
    n_seq = int(rng.integers(1, 4))
    nodes = tuple(int(x) for x in rng.integers(300, 1025, n_seq))
    V = int(rng.choice([32000, 32768, 5003, 9001]))
    td = tuple(float(x) for x in rng.choice([0.5, 0.7, 1.0], n_seq))
    print(f"large builders nodes={nodes} V={V} td={td}", flush=True)
    d = (rng.standard_normal((sum(nodes), V)) * float(rng.choice([1.0, 2.5, 4.0]))).astype(np.float32)
    batch = dy.Batch.from_sizes(nodes)
    dd = torch.from_numpy(d).cuda()
    built, _, seed = build_in_full(dy, dd, d, batch, nodes, td, seed)
    plain = dy.build_tree(dd, batch, td, seed, use_workspace=False)
    torch.cuda.synchronize()
    for k in ("parent", "token", "sib_rank", "first_child", "next_sibling", "depth"):
        assert torch.equal(getattr(built.tree, k), getattr(plain.tree, k)), k
    assert torch.equal(built.anc_mask, plain.anc_mask)
    thr = tuple(float(x) for x in rng.choice([0.02, 0.005, 0.002], n_seq))
    threshold_in_full(dy, dd, d, batch, td, thr, seed)
