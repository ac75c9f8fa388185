"""GPU parity at the library's largest tree, 2048 rows (the last row of the paper's random-tree table
in its appendix on token order): dyspec_dfs_reorder bit for bit against the oracle, tree attention on
the tree in creation order and renamed depth-first (tree-only as in that table, and behind a
prefix) against the fp64 oracle, verification of a hand-linked 2048-row tree; the builders stop at
their own limit."""
import math

import numpy as np
import pytest

import oracle
from helpers import ATTN_TOL, compare_verify, oracle_attention_rows
from test_gpu_reorder import check_against_oracle, device_tree

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


def random_tree(n, rng, near=0.0):
    """Parent of node i uniform among the earlier nodes (the paper's random tree), or among the last
    few with probability `near`; children linked in index order."""
    par = np.full(n, -1, np.int32)
    for i in range(1, n):
        par[i] = int(rng.integers(max(0, i - 8), i)) if rng.random() < near else int(rng.integers(0, i))
    fc, ns, dep = oracle.links_from_parent(par)
    rk = np.zeros(n, np.int32)
    cnt = np.zeros(n, np.int32)
    for i in range(1, n):
        rk[i] = cnt[par[i]]
        cnt[par[i]] += 1
    return par, fc, ns, dep, rk


@pytest.mark.parametrize("n,prefix,Hq,Hkv,near,seed", [
    (2048, 0, 8, 2, 0.0, 1),          # tree-only, as the paper's table measures it
    (2048, 200, 4, 1, 0.6, 2),        # behind a ragged prefix, deeper tree
    (1999, 64, 8, 8, 0.3, 3),         # ragged last tree tile, no query grouping
])
def test_wide_tree_reorder_and_attention(dy, n, prefix, Hq, Hkv, near, seed):
    print(f"wide tree n={n} prefix={prefix} H={Hq}/{Hkv} seed={seed}", flush=True)
    rng = np.random.default_rng(seed)
    d = 128
    par, fc, ns, dep, rk = random_tree(n, rng, near)
    batch = dy.Batch.from_sizes([n], [prefix])
    assert batch.mask_words == (n + 63) // 64
    tree = device_tree(dy, par, fc, ns, dep, rk, np.arange(n, dtype=np.int32))
    re = dy.dfs_reorder(tree, batch)
    torch.cuda.synchronize()
    check_against_oracle(dy, batch, tree, re)
    mask = oracle.ancestor_mask(par)
    b0, b1 = oracle.mask_block_count(mask, n), oracle.mask_block_count(re.anc_mask.cpu().numpy().view(np.uint64), n)
    print(f"  non-empty 32x32 blocks: {b0} in creation order, {b1} depth-first", flush=True)
    assert b1 < b0

    g = torch.Generator().manual_seed(seed)
    mk = lambda *sh: torch.randn(sh, generator=g, dtype=torch.float32).to(torch.bfloat16)
    q, kp, vp, kt, vt = mk(n, Hq, d), mk(prefix, Hkv, d), mk(prefix, Hkv, d), mk(n, Hkv, d), mk(n, Hkv, d)
    dev = lambda t: t.cuda() if t.numel() else torch.empty(t.shape, dtype=t.dtype, device="cuda")
    scale = 1.0 / math.sqrt(d)
    mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
    out = dy.tree_attn(dev(q), dev(kp), dev(vp), dev(kt), dev(vt), mask_dev, batch, scale)
    idx = re.gather_index(batch)
    out_dfs = dy.tree_attn(dev(q)[idx], dev(kp), dev(vp), dev(kt)[idx], dev(vt)[idx], re.anc_mask, batch, scale)
    torch.cuda.synchronize()
    host = [t.float().numpy() for t in (q, kp, vp, kt, vt)]
    pick = np.unique(np.concatenate([rng.choice(n * Hq, 3000, replace=False), np.arange(Hq), n * Hq - 1 - np.arange(Hq)]))
    rj, rh = np.divmod(pick, Hq)
    want = oracle_attention_rows(*host, mask, batch, 0, scale, rj, rh)
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()
    err = float(np.abs(got[rj, rh] - want).max())
    # row `new` of the renamed tree is row order[new] of the original
    order = re.order.cpu().numpy()
    rank = np.empty(n, np.int64)
    rank[order] = np.arange(n)
    got_dfs = out_dfs.float().cpu().numpy()
    err_dfs = float(np.abs(got_dfs[rank[rj], rh] - want).max())
    print(f"  attention max abs error {err:.2e} (creation order), {err_dfs:.2e} (depth-first)", flush=True)
    assert err <= ATTN_TOL["bf16"] and err_dfs <= ATTN_TOL["bf16"]


def test_wide_tree_verification(dy):
    """Algorithm 3 on a hand-linked tree of 2048 rows (a random tree whose tokens are distinct among
    siblings), against the oracle."""
    n, V = 2048, 1000
    rng = np.random.default_rng(9)
    par, fc, ns, dep, rk = random_tree(n, rng, 0.5)
    d = (rng.standard_normal((n, V)) * 3.0).astype(np.float32)
    t = (d + rng.standard_normal((n, V)) * 0.5).astype(np.float32)
    tok = np.full(n, -1, np.int32)
    for i in range(1, n):                         # the rk-th likeliest token of the parent's draft row
        tok[i] = int(np.argsort(-d[par[i]])[rk[i]])
    batch = dy.Batch.from_sizes([n])
    tree = device_tree(dy, par, fc, ns, dep, rk, tok)
    dd, tt = torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda()
    paths = 0
    for seed in range(8):
        out = dy.verify(dd, tt, batch, tree, (0.7,), (0.9,), seed)
        torch.cuda.synchronize()
        paths += compare_verify(out, batch, [(tok, fc, ns)], d, t, (0.7,), (0.9,), seed)[0]
    assert paths >= 7


def test_builders_stop_at_their_own_limit(dy):
    d = torch.zeros((1025, 64), device="cuda")
    batch = dy.Batch.from_sizes([1025])
    with pytest.raises(dy.DyspecError) as e:
        dy.build_tree(d, batch, (1.0,), 0)
    assert e.value.status == -2
    with pytest.raises(dy.DyspecError) as e:
        dy.build_tree_threshold(d, batch, (1.0,), (0.1,), 0)
    assert e.value.status == -2
