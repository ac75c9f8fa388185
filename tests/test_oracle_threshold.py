"""Pins for the oracle's threshold construction (Algorithm 2, Section 4.4, Appendix A.2)."""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle


def paths_of(parent, sib_rank, n):
    out = [()]
    for i in range(1, n):
        out.append(out[parent[i]] + (int(sib_rank[i]),))
    return out


@pytest.mark.parametrize("V,N,temp,seed", [(50, 24, 1.0, 0), (50, 40, 0.7, 1), (1000, 64, 0.6, 2), (7, 30, 1.3, 3),
                                          (300, 48, 1.0, 4), (1000, 33, 0.8, 5)])
def test_threshold_of_last_greedy_pick_rebuilds_the_greedy_tree(V, N, temp, seed):
    """Appendix A.1, last paragraph: with the threshold set to the estimated value of the last
    node the greedy construction added, the level-by-level construction yields the same tree.
    Rows are handed out by path so both constructions give a node the same draft row."""
    rng = np.random.default_rng(seed)
    draft = (rng.standard_normal((N + 16, V)) * 2.0).astype(np.float32)
    g = oracle.build_tree(draft, N, temp, seed=seed, seq=3)
    assert g.n_built == N
    gp = paths_of(g.parent, g.sib_rank, N)
    index_of = {p: i for i, p in enumerate(gp)}
    t = float(g.est_value[:N].min())
    # a slot the greedy run left unopened may tie with t only by accident; the test needs a gap
    th = oracle.threshold_tree(draft, N + 16, temp, t * (1.0 - 1e-12), seed=seed, seq=3,
                               row_of=lambda path, i: index_of.get(path, 0))
    assert th.n_built == N, "another slot lies within 1e-12 of the threshold: pick another seed"
    tp = th.paths[:N]
    assert sorted(tp) == sorted(gp)
    for i, p in enumerate(tp):
        j = index_of[p]
        assert th.token[i] == g.token[j]
        assert th.depth[i] == g.depth[j]
        assert th.est_value[i] == pytest.approx(g.est_value[j], rel=1e-12)
    # same ancestor sets, up to the renaming of nodes
    for i, p in enumerate(tp):
        anc_t = {tp[k] for k in range(N) if (int(th.mask[i, k // 64]) >> (k % 64)) & 1}
        j = index_of[p]
        anc_g = {gp[k] for k in range(N) if (int(g.mask[j, k // 64]) >> (k % 64)) & 1}
        assert anc_t == anc_g


@pytest.mark.parametrize("seed", range(4))
def test_values_follow_the_closed_form_and_the_threshold_rule(seed):
    """Appendix D: a node's estimated value is the product of the original draft probabilities
    along its path times (1 - the original probabilities of its earlier siblings).  Every
    created node was drawn at a value >= t; every position left unopened has a value < t."""
    V, cap, temp, t = 40, 400, 0.9, 0.02
    rng = np.random.default_rng(10 + seed)
    draft = (rng.standard_normal((cap, V)) * 1.5).astype(np.float32)
    th = oracle.threshold_tree(draft, cap, temp, t, seed=seed)
    n = th.n_built
    assert 10 < n < cap
    P = sp_softmax(draft.astype(np.float64) / temp, axis=1)          # row i: distribution after node i
    path_prob = np.ones(n)                                            # product of original probabilities down to i
    for i in range(1, n):
        p = th.parent[i]
        path_prob[i] = path_prob[p] * P[p, th.token[i]]
    for p in range(n):
        kids = [i for i in range(n) if th.parent[i] == p]
        kids.sort(key=lambda i: th.sib_rank[i])
        assert [th.sib_rank[i] for i in kids] == list(range(len(kids)))
        assert len({int(th.token[i]) for i in kids}) == len(kids)     # drawn without replacement
        gone = 0.0
        for i in kids:
            want = path_prob[p] * (1.0 - gone)
            assert th.est_value[i] == pytest.approx(want, rel=1e-9)
            assert th.est_value[i] >= t
            gone += P[p, th.token[i]]
        assert path_prob[p] * (1.0 - gone) < t                        # the position after the last child
    assert np.all(np.diff(th.depth[:n]) >= 0)                         # created level by level


def test_uniform_three_tokens_by_hand():
    """V = 3, uniform rows, t = 0.3.  Root: draws at values 1, 2/3, 1/3 (then nothing is left);
    each child's own first draw is at 1/3 >= t and its second at 2/9 < t; the grandchildren's
    first draws would be at 1/9.  Seven nodes whatever the uniforms are."""
    draft = np.zeros((16, 3), np.float32)
    for seed in range(5):
        th = oracle.threshold_tree(draft, 16, 1.0, 0.3, seed=seed)
        assert th.n_built == 7 and th.n_levels == 3
        np.testing.assert_array_equal(th.parent[:7], [-1, 0, 0, 0, 1, 2, 3])
        np.testing.assert_allclose(th.est_value[:7], [1, 1, 2 / 3, 1 / 3, 1 / 3, 1 / 3, 1 / 3], rtol=1e-15)
        np.testing.assert_allclose(th.child_value[1:7], [1 / 3] * 3 + [1 / 9] * 3, rtol=1e-15)
        assert sorted(th.token[1:4]) == [0, 1, 2]
        np.testing.assert_array_equal(th.first_child[:7], [1, 4, 5, 6, -1, -1, -1])
        np.testing.assert_array_equal(th.next_sibling[:7], [-1, 2, 3, -1, -1, -1, -1])
        np.testing.assert_array_equal(th.mask[:7, 0], [1, 3, 5, 9, 0b10011, 0b100101, 0b1001001])


def test_certain_token_gives_a_chain_up_to_the_cap():
    draft = np.full((12, 5), -np.inf, np.float32)
    draft[:, 2] = 0.0
    th = oracle.threshold_tree(draft, 12, 1.0, 0.5, seed=1)
    assert th.n_built == 12
    np.testing.assert_array_equal(th.parent, np.arange(-1, 11))
    np.testing.assert_array_equal(th.token[1:], 2)
    np.testing.assert_array_equal(th.est_value, 1.0)


def test_cap_keeps_a_prefix_of_the_uncapped_tree():
    V, temp, t = 30, 1.0, 0.01
    rng = np.random.default_rng(5)
    draft = (rng.standard_normal((300, V)) * 1.5).astype(np.float32)
    full = oracle.threshold_tree(draft, 300, temp, t, seed=9)
    assert 40 < full.n_built < 300
    cut = oracle.threshold_tree(draft, 25, temp, t, seed=9)
    assert cut.n_built == 25
    for name in ("parent", "token", "sib_rank", "depth", "est_value"):
        np.testing.assert_array_equal(getattr(cut, name)[:25], getattr(full, name)[:25])
    # links inside the kept rows agree; links to rows that were cut are absent
    fc = np.where(full.first_child[:25] < 25, full.first_child[:25], -1)
    ns = np.where(full.next_sibling[:25] < 25, full.next_sibling[:25], -1)
    np.testing.assert_array_equal(cut.first_child[:25], fc)
    np.testing.assert_array_equal(cut.next_sibling[:25], ns)


def test_threshold_above_one_builds_nothing():
    draft = np.zeros((4, 6), np.float32)
    th = oracle.threshold_tree(draft, 4, 1.0, 1.5, seed=0)
    assert th.n_built == 1 and th.first_child[0] == -1
