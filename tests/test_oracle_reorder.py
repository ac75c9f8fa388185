"""Pins for the oracle's depth-first renaming of a token tree (Appendix "Block-Sparsity
Friendly Token Order"): checked against a recursive definition on small trees, against the
invariants any pre-order numbering has, and against the permuted mask of the original tree."""
import itertools

import numpy as np
import pytest

import oracle


def recursive_preorder(parent, children_order):
    out = []

    def visit(v):
        out.append(v)
        for c in children_order[v]:
            visit(c)
    visit(0)
    return out


def all_parent_arrays(n):
    """Every rooted tree on nodes 0..n-1 whose parents precede children."""
    for tail in itertools.product(*[range(i) for i in range(1, n)]):
        yield np.array((-1,) + tail, dtype=np.int32)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_order_equals_recursive_preorder_on_every_small_tree(n):
    for par in all_parent_arrays(n):
        fc, ns, dep = oracle.links_from_parent(par)
        kids = {v: [c for c in range(n) if par[c] == v] for v in range(n)}
        assert oracle.dfs_order(par, fc, ns).tolist() == recursive_preorder(par, kids)


def random_tree(n, rng, sampling_order_shuffled=True):
    par = np.full(n, -1, np.int32)
    for i in range(1, n):
        par[i] = rng.integers(0, i)
    fc, ns, dep = oracle.links_from_parent(par)
    if sampling_order_shuffled:            # sibling lists in an order other than by index
        fc[:] = -1
        ns[:] = -1
        for v in range(n):
            kids = [c for c in range(n) if par[c] == v]
            rng.shuffle(kids)
            for a, b in zip(kids, kids[1:]):
                ns[a] = b
            if kids:
                fc[v] = kids[0]
    rk = np.zeros(n, np.int32)
    for v in range(n):
        c, r = fc[v], 0
        while c >= 0:
            rk[c] = r
            r += 1
            c = ns[c]
    return par, fc, ns, dep, rk


@pytest.mark.parametrize("seed", range(6))
def test_preorder_invariants_and_permuted_mask(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 200))
    par, fc, ns, dep, rk = random_tree(n, rng)
    tok = rng.integers(0, 1000, n).astype(np.int32)
    order = oracle.dfs_order(par, fc, ns)
    assert sorted(order.tolist()) == list(range(n)) and order[0] == 0
    par_n, tok_n, rk_n, fc_n, ns_n, dep_n, mask_n = oracle.relabel_tree(order, par, tok, rk, fc, ns, dep)
    # parents precede children; every subtree is a contiguous run that starts at its root
    assert all(par_n[j] < j for j in range(1, n))
    size = np.ones(n, np.int64)
    for j in range(n - 1, 0, -1):
        size[par_n[j]] += size[j]
    for j in range(n):
        inside = [a for a in range(n) if (mask_n[a, j // 64] >> np.uint64(j % 64)) & np.uint64(1)]
        assert inside == list(range(j, j + size[j]))
    # the first child is the next node; siblings keep their sampling order
    for j in range(n):
        if fc_n[j] >= 0:
            assert fc_n[j] == j + 1
        if ns_n[j] >= 0:
            assert ns_n[j] == j + size[j] and rk_n[ns_n[j]] == rk_n[j] + 1
    assert np.array_equal(tok_n, tok[order]) and np.array_equal(dep_n, dep[order])
    # the mask of the renamed tree is the original mask with rows and columns permuted
    m = oracle.ancestor_mask(par)
    for jn in range(n):
        for an in range(n):
            bit_new = (mask_n[jn, an // 64] >> np.uint64(an % 64)) & np.uint64(1)
            j, a = order[jn], order[an]
            assert bit_new == ((m[j, a // 64] >> np.uint64(a % 64)) & np.uint64(1))
    assert np.array_equal(oracle.ancestor_mask(par_n), mask_n)


def test_chain_and_star_keep_their_order():
    n = 70
    chain = np.arange(-1, n - 1, dtype=np.int32)
    fc, ns, dep = oracle.links_from_parent(chain)
    assert oracle.dfs_order(chain, fc, ns).tolist() == list(range(n))
    star = np.array([-1] + [0] * (n - 1), dtype=np.int32)
    fc, ns, dep = oracle.links_from_parent(star)
    assert oracle.dfs_order(star, fc, ns).tolist() == list(range(n))


def test_rows_outside_the_tree_go_last():
    par = np.array([-1, 0, 0, 1, -1, -1], dtype=np.int32)      # rows 4, 5 were never built
    fc = np.array([1, 3, -1, -1, -1, -1], np.int32)
    ns = np.array([-1, 2, -1, -1, -1, -1], np.int32)
    order = oracle.dfs_order(par, fc, ns)
    assert order.tolist() == [0, 1, 3, 2, 4, 5]
    z = np.zeros(6, np.int32)
    par_n, *_rest, mask_n = oracle.relabel_tree(order, par, z, z, fc, ns, z)
    assert par_n.tolist() == [-1, 0, 1, 0, -1, -1]
    assert mask_n[:, 0].tolist() == [0b1, 0b11, 0b111, 0b1001, 0b10000, 0b100000]


def test_block_count_closed_forms():
    n = 128
    chain = np.arange(-1, n - 1, dtype=np.int32)               # lower triangle: 4 block rows -> 1+2+3+4
    assert oracle.mask_block_count(oracle.ancestor_mask(chain), n, 32) == 10
    star = np.array([-1] + [0] * (n - 1), dtype=np.int32)      # diagonal blocks plus the first block column
    assert oracle.mask_block_count(oracle.ancestor_mask(star), n, 32) == 4 + 3
    assert oracle.mask_block_count(oracle.ancestor_mask(star), 100, 32) == 4 + 3
