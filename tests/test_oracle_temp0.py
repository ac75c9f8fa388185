"""Pins for the oracle's temperature-0 target (Section 5, the temperature-0 rows of the
result tables): the target row is all mass on its largest logit, so Algorithm 3 must emit
exactly the greedy decoding of the target model, whatever the tree and the draws."""
import numpy as np
import pytest

import oracle
from test_oracle_verify import exact_law, make_step


def greedy_walk(target, token, first_child, next_sibling, emit_bonus=True):
    """Follow the target's argmax token down the tree: written from the definition of greedy
    decoding, with none of Algorithm 3's residual arithmetic."""
    cur, path = 0, []
    while True:
        want = int(np.argmax(target[cur]))
        c, nxt = int(first_child[cur]), -1
        if c < 0:
            return path, (want if emit_bonus else -1), cur
        while c >= 0:
            if int(token[c]) == want:
                nxt = c
                break
            c = int(next_sibling[c])
        if nxt < 0:
            return path, want, cur
        path.append(nxt)
        cur = nxt


def test_softmax_at_temperature_zero_is_one_hot_first_argmax():
    x = np.array([0.5, 3.0, -1.0, 3.0, 2.9999], dtype=np.float32)
    p = oracle.softmax(x, 0.0)
    np.testing.assert_array_equal(p, [0, 1, 0, 0, 0])
    # and it is the limit of small temperatures (3.0 and 2.9999 separate only below 1e-5)
    p_small = oracle.softmax(np.array([0.5, 3.0, -1.0, 2.0], dtype=np.float32), 1e-2)
    np.testing.assert_allclose(p_small, [0, 1, 0, 0], atol=1e-40)
    st = oracle.softmax_stats(x[None], x[None], 1.0, 0.0)
    assert st[0, 2] == 3.0 and st[0, 3] == 1.0
    # the draft half of the statistics is untouched
    assert st[0, 0] == 3.0 and st[0, 1] == pytest.approx(np.exp(np.float64(x) - 3.0).sum(), rel=1e-15)


@pytest.mark.parametrize("n_budget,V,seed", [(1, 4, 0), (2, 4, 1), (3, 4, 2), (4, 4, 3), (4, 3, 4)])
def test_exact_output_law_is_greedy_decoding(n_budget, V, seed):
    """Integrating over every draw of the builder and the verifier: with probability one the
    emitted tokens are the target's argmax chain (all non-root rows share one target row)."""
    rng = np.random.default_rng(100 + seed)
    draft = (rng.standard_normal((n_budget, V)) * 1.5).astype(np.float32)
    target = (draft + rng.standard_normal((n_budget, V))).astype(np.float32)
    target[1:] = target[1] if n_budget > 1 else 0
    a0 = int(np.argmax(target[0]))
    a1 = int(np.argmax(target[1])) if n_budget > 1 else None
    law = exact_law(make_step(draft, target, n_budget, 0.7, 0.0, emit_bonus=True))
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-10)
    multi = 0.0
    for out, pr in law.items():
        if pr < 1e-12:
            continue
        assert out[0] == a0, (out, pr)
        assert all(t == a1 for t in out[1:]), (out, pr)
        multi += pr if len(out) > 1 else 0.0
    if n_budget > 1:
        assert multi > 0.0            # some trees do contain the argmax token as a child


@pytest.mark.parametrize("seed", range(6))
def test_walk_equals_following_the_argmax_token(seed):
    """Built trees of 48 nodes over V = 50: accepted path, stop node and last token equal the
    plain argmax walk for any verification seed; a boosted argmax makes accepted paths long."""
    V, N, td = 50, 48, 0.8
    rng = np.random.default_rng(seed)
    draft = (rng.standard_normal((N, V)) * 2.0).astype(np.float32)
    target = (draft + 0.3 * rng.standard_normal((N, V))).astype(np.float32)
    t = oracle.build_tree(draft, N, td, seed=seed, seq=0)
    lengths = []
    for vseed in range(4):
        for bonus in (True, False):
            r = oracle.verify(draft, target, t.token, t.first_child, t.next_sibling, td, 0.0,
                              seed=1000 + vseed, emit_bonus=bonus)
            path, fin, stop = greedy_walk(target, t.token, t.first_child, t.next_sibling, bonus)
            assert list(r.accepted_nodes) == path
            assert r.final_token == fin and r.stop_node == stop
            lengths.append(len(path))
    # nothing random is left in the outcome
    assert len(set(lengths)) == 1


def test_limit_of_small_target_temperatures():
    """Where every visited target row has a clear winner, a tiny positive temperature walks
    the same path and emits the same token as temperature 0."""
    V, N, td = 40, 32, 1.0
    agree = 0
    for seed in range(8):
        rng = np.random.default_rng(50 + seed)
        draft = (rng.standard_normal((N, V)) * 2.0).astype(np.float32)
        target = (draft + 0.5 * rng.standard_normal((N, V))).astype(np.float32)
        srt = np.sort(target, axis=1)
        if (srt[:, -1] - srt[:, -2]).min() < 0.02:
            continue
        t = oracle.build_tree(draft, N, td, seed=seed)
        r0 = oracle.verify(draft, target, t.token, t.first_child, t.next_sibling, td, 0.0, seed=7)
        r1 = oracle.verify(draft, target, t.token, t.first_child, t.next_sibling, td, 1e-4, seed=7)
        assert list(r0.accepted_nodes) == list(r1.accepted_nodes)
        assert r0.final_token == r1.final_token
        agree += 1
    assert agree >= 4


def test_accept_ratio_at_temperature_zero():
    """Children of the root in sampling order, none accepted before: the matching child sees
    1 / (its draft probability renormalised over what is left), every other child sees 0."""
    V, td = 12, 0.9
    rng = np.random.default_rng(3)
    draft = (rng.standard_normal((5, V)) * 1.2).astype(np.float32)
    target = draft.copy()
    tok = np.array([-1, 4, 7, 2, 9], dtype=np.int32)
    target[0, 2] = 50.0                                    # argmax of the root's target row
    fc = np.array([1, -1, -1, -1, -1], dtype=np.int32)
    ns = np.array([-1, 2, 3, 4, -1], dtype=np.int32)
    ratio = oracle.accept_ratio_all(draft, target, tok, fc, ns, td, 0.0)
    d = np.exp(np.float64(draft[0]) / td)
    d /= d.sum()
    left = 1.0 - d[4] - d[7]
    assert ratio[1] == 0.0 and ratio[2] == 0.0
    assert ratio[3] == pytest.approx(left / d[2], rel=1e-12)
    # after the argmax token itself was rejected the residual keeps its mass there:
    # relu(R - D) = (1 - d)[argmax], one-hot again, and token 9 sees 0
    assert ratio[4] == 0.0
