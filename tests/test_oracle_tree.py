"""Pins for the oracle's greedy tree construction (Algorithm 1) and ancestor mask."""
import itertools

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle


def make_logits(n, V, sigma, seed):
    return (np.random.default_rng(seed).standard_normal((n, V)) * sigma).astype(np.float32)


def probs(logits, temp):
    return sp_softmax(logits.astype(np.float64) / temp, axis=-1)


# ----------------------------------------------------------------- inverse CDF by hand

def test_inverse_cdf_hand_example():
    """V=4, d=(0.1,0.2,0.3,0.4): token = smallest y with cumulative mass > u (strict)."""
    d = np.array([0.1, 0.2, 0.3, 0.4])
    logits = np.log(d)[None, :].repeat(2, 0).astype(np.float32)
    for u, want in [(0.0, 0), (0.05, 0), (0.11, 1), (0.29, 1), (0.31, 2), (0.59, 2), (0.61, 3), (0.999, 3)]:
        t = oracle.build_tree_explicit(logits, 2, 1.0, [0.0, u])
        assert t.n_built == 2 and t.token[1] == want and t.parent[1] == 0


def test_second_sibling_uses_renormalised_residual():
    """After token 3 (d=0.4) is taken the residual is (1,2,3)/6 over tokens 0..2
    (Appendix D: draft_k = d_k / (1 - sum of earlier siblings))."""
    d = np.array([0.1, 0.2, 0.3, 0.4])
    logits = np.log(d)[None, :].repeat(3, 0).astype(np.float32)
    # node 1 = token 3 (v0 = 0.4, v1 = 0.6): next pop is the sibling slot (0.6 > 0.4)
    for u2, want in [(0.1, 0), (0.2, 1), (0.49, 1), (0.51, 2), (0.99, 2)]:
        t = oracle.build_tree_explicit(logits, 3, 1.0, [0.0, 0.9, u2])
        assert list(t.parent[:3]) == [-1, 0, 0]
        assert t.token[1] == 3 and t.token[2] == want
        assert t.est_value[2] == pytest.approx(0.6, rel=1e-6)


# ----------------------------------------------------------------- closed form of values

def closed_form_value(tree, P, i):
    """Appendix D: value of the sampling that produced node i = product of ORIGINAL draft
    probabilities of its ancestors' tokens times (1 - sum of original probabilities of its
    earlier siblings)."""
    v = 1.0
    a = tree.parent[i]
    while a > 0:
        v *= P[tree.parent[a], tree.token[a]]
        a = tree.parent[a]
    p = tree.parent[i]
    earlier = [c for c in range(1, i) if tree.parent[c] == p]
    return v * (1.0 - sum(P[p, tree.token[c]] for c in earlier))


@pytest.mark.parametrize("V,N,sigma,temp,seed", [(50, 24, 2.0, 1.0, 0), (1000, 32, 2.0, 1.0, 0),
                                                   (300, 64, 3.0, 0.6, 3), (20, 40, 1.0, 1.0, 7)])
def test_values_match_closed_form_and_pops_decrease(V, N, sigma, temp, seed):
    logits = make_logits(N, V, sigma, seed)
    P = probs(logits, temp)
    t = oracle.build_tree(logits, N, temp, seed)
    assert t.n_built == N
    assert t.est_value[0] == 1.0
    for i in range(1, N):
        assert t.est_value[i] == pytest.approx(closed_form_value(t, P, i), rel=1e-9, abs=1e-15)
    ev = t.est_value[1:N]
    assert np.all(ev[1:] <= ev[:-1] * (1 + 1e-12))          # popped values never increase
    assert ev[0] == 1.0


def test_structure_invariants():
    V, N = 200, 96
    logits = make_logits(N, V, 3.0, 11)
    t = oracle.build_tree(logits, N, 0.6, 11)
    assert t.parent[0] == -1 and t.depth[0] == 0
    for i in range(1, N):
        p = t.parent[i]
        assert 0 <= p < i
        assert t.depth[i] == t.depth[p] + 1
    for p in range(N):
        kids = [c for c in range(1, N) if t.parent[c] == p]
        # sampling order == creation order; ranks contiguous; tokens distinct
        assert [t.sib_rank[c] for c in kids] == list(range(len(kids)))
        assert len({int(t.token[c]) for c in kids}) == len(kids)
        chain, c = [], t.first_child[p]
        while c >= 0:
            chain.append(int(c))
            c = t.next_sibling[c]
        assert chain == kids


def test_mask_is_ancestor_relation():
    V, N = 100, 130                    # three mask words, ragged last word
    logits = make_logits(N, V, 2.0, 5)
    t = oracle.build_tree(logits, N, 1.0, 5)
    dense = np.zeros((N, N), dtype=bool)
    for j in range(N):
        for i in range(N):
            dense[j, i] = bool((int(t.mask[j, i // 64]) >> (i % 64)) & 1)
    for j in range(N):
        anc, a = set(), j
        while a >= 0:
            anc.add(a)
            a = t.parent[a]
        assert set(np.nonzero(dense[j])[0]) == anc
        assert dense[j].sum() == t.depth[j] + 1
        assert not dense[j, j + 1:].any()
    assert np.array_equal(oracle.ancestor_mask(t.parent), t.mask)


def test_chain_mask_is_lower_triangular():
    N = 70
    parent = np.arange(-1, N - 1, dtype=np.int32)
    m = oracle.ancestor_mask(parent)
    for j in range(N):
        bits = sum(int(m[j, w]) << (64 * w) for w in range(m.shape[1]))
        assert bits == (1 << (j + 1)) - 1


# ----------------------------------------------------------------- greedy optimality

def test_greedy_is_max_weight_connected_subtree():
    """Appendix D.1: the first n nodes the greedy rule creates carry the largest total
    estimated value among all sets of n samplings that are reachable (a sampling exists
    only after its parent node and its previous sibling).  Draws are named by path, so a
    larger budget extends the same tree and reveals the competing candidates."""
    V, big, n = 3, 13, 6
    for seed in range(6):
        logits = make_logits(big, V, 1.0, 100 + seed)
        T = oracle.build_tree(logits, big, 1.0, seed)
        small = oracle.build_tree(logits, n, 1.0, seed)
        assert np.array_equal(small.parent, T.parent[:n]) and np.array_equal(small.token, T.token[:n])
        nb = T.n_built
        prev_sib = {}
        for p in range(nb):
            kids = [c for c in range(1, nb) if T.parent[c] == p]
            for a, b in zip(kids[:-1], kids[1:]):
                prev_sib[b] = a
        best = -1.0
        for sub in itertools.combinations(range(1, nb), n - 1):
            s = set(sub) | {0}
            if all(T.parent[c] in s and prev_sib.get(c, 0) in s for c in sub):
                best = max(best, sum(T.est_value[c] for c in sub))
        greedy = sum(T.est_value[c] for c in range(1, n))
        assert greedy == pytest.approx(best, rel=1e-12)


# ----------------------------------------------------------------- sampling law

def test_first_child_token_follows_draft_distribution():
    V, temp = 8, 0.8
    logits = make_logits(2, V, 1.5, 42)
    p = probs(logits, temp)[0]
    counts = np.zeros(V)
    n = 20000
    for seed in range(n):
        counts[oracle.build_tree(logits, 2, temp, seed).token[1]] += 1
    chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 29.9              # 7 dof, p ~ 1e-4


def test_frontier_exhausts_when_vocabulary_is_smaller_than_budget():
    """V=2, rows all the same: each node can have at most 2 children; with a huge logit gap
    the values of the unlikely branches underflow to 0 and are never opened."""
    logits = np.array([[0.0, -2000.0]] * 6, dtype=np.float32)
    t = oracle.build_tree(logits, 6, 1.0, 0)
    # only the chain of token-0 nodes has positive value: sibling slots have v = 0
    assert t.n_built == 6
    assert list(t.token[1:6]) == [0] * 5 and list(t.parent[1:6]) == [0, 1, 2, 3, 4]
    one = np.array([[0.0]] * 4, dtype=np.float32)        # V = 1: a single chain, no siblings
    t1 = oracle.build_tree(one, 4, 1.0, 0)
    assert t1.n_built == 4 and list(t1.parent[:4]) == [-1, 0, 1, 2]


def test_path_keyed_draws_do_not_depend_on_sequence_of_other_paths():
    """Different seq index gives a different, independent stream; same (seed, seq) repeats."""
    logits = make_logits(16, 64, 2.0, 9)
    a = oracle.build_tree(logits, 16, 1.0, 3, seq=0)
    b = oracle.build_tree(logits, 16, 1.0, 3, seq=0)
    c = oracle.build_tree(logits, 16, 1.0, 3, seq=1)
    assert np.array_equal(a.token, b.token) and np.array_equal(a.parent, b.parent)
    assert not np.array_equal(a.token, c.token)


def test_zero_weight_tokens_are_never_drawn_and_ties_pop_earliest_slot():
    """u = 0 must skip leading zero-probability tokens (strict inequality in the inverse
    CDF).  With d = (.5,.5) the two slots opened by node 1 tie at 0.5: the sibling slot was
    opened first, so node 2 hangs off the root."""
    z = np.array([[-3000.0, 0.0, 0.0]] * 2, dtype=np.float32)
    assert oracle.build_tree_explicit(z, 2, 1.0, [0.0, 0.0]).token[1] == 1
    half = np.zeros((3, 2), dtype=np.float32)
    t = oracle.build_tree_explicit(half, 3, 1.0, [0.0, 0.25, 0.25])
    assert list(t.parent[:3]) == [-1, 0, 0] and list(t.token[1:3]) == [0, 1]
    assert t.margin_pop[2] == 0.0
