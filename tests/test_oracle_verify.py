"""Pins for the oracle's tree verification (Algorithm 3) and its coupling with the tree
builder: the emitted tokens must follow the target model's distribution exactly."""
import math

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle

TOP = 1.0 - 2.0 ** -53


def probs(logits, temp):
    return sp_softmax(np.asarray(logits, dtype=np.float64) / temp, axis=-1)


# ---------------------------------------------------------------------------------------
# Exact integration of a black-box procedure over its uniforms.
#
# run(u) -> (trace, output): `trace` is the ordered list of (variable, outcome) decisions
# the procedure took when every uniform comes from the dict `u` (missing ones default to
# 0.5).  Decision k depends only on the variables of decisions <= k, and each outcome is
# monotone (piecewise constant on consecutive intervals) in its own variable.  The
# integrator fixes variables one at a time, finds the interval boundaries by bisection on
# the oracle itself, and returns {output: probability}.
# ---------------------------------------------------------------------------------------

def _outcome(run, u, var, val, pos):
    u2 = dict(u)
    u2[var] = val
    trace, _ = run(u2)
    assert trace[pos][0] == var
    return trace[pos][1]


def _pieces(run, u, var, pos):
    a, out = 0.0, []
    while a < 1.0:
        o = _outcome(run, u, var, a, pos)
        if _outcome(run, u, var, TOP, pos) == o:
            b = 1.0
        else:
            lo, hi = a, TOP
            for _ in range(60):
                mid = 0.5 * (lo + hi)
                if _outcome(run, u, var, mid, pos) == o:
                    lo = mid
                else:
                    hi = mid
            b = hi
        out.append((a, b))
        if b <= a:
            b = np.nextafter(a, 2.0)
        a = b
    return out


def exact_law(run):
    law = {}

    def rec(u, weight):
        trace, output = run(u)
        for pos, (var, _) in enumerate(trace):
            if var not in u:
                for a, b in _pieces(run, u, var, pos):
                    if b > a:
                        u2 = dict(u)
                        u2[var] = 0.5 * (a + b)
                        rec(u2, weight * (b - a))
                return
        law[output] = law.get(output, 0.0) + weight

    rec({}, 1.0)
    return law


def make_step(draft, target, n_budget, temp_d, temp_t, emit_bonus=True, fixed_tree=None):
    """One speculative step (build + verify) as a function of its uniforms."""
    N = n_budget

    def run(u):
        trace = []
        if fixed_tree is None:
            ub = [u.get(("b", i), 0.5) for i in range(N)]
            t = oracle.build_tree_explicit(draft, N, temp_d, ub)
            for i in range(1, t.n_built):
                trace.append((("b", i), (int(t.parent[i]), int(t.token[i]))))
            token, fc, ns = t.token, t.first_child, t.next_sibling
        else:
            token, fc, ns = fixed_tree
        ua = [u.get(("a", i), 0.5) for i in range(N)]
        ur = [u.get(("r", i), 0.5) for i in range(N)]
        r = oracle.verify_explicit(draft, target, token, fc, ns, temp_d, temp_t, ua, ur, emit_bonus)
        acc = set(int(x) for x in r.accepted_nodes)
        tested = [i for i in range(N) if math.isfinite(r.tested_margin[i]) or i in acc]
        # tested nodes in walk order: by (depth along accepted path, sibling order) == the
        # order the walk met them; reconstruct it by following the links
        cur, order = 0, []
        while True:
            c, nxt = fc[cur], -1
            while c >= 0:
                if c in tested:
                    order.append(int(c))
                if c in acc:
                    nxt = int(c)
                    break
                c = ns[c]
            if nxt < 0:
                break
            cur = nxt
        for i in order:
            trace.append((("a", i), i in acc))
        if r.final_token >= 0:
            trace.append((("r", r.stop_node), r.final_token))
        emitted = tuple(int(token[i]) for i in r.accepted_nodes) + ((r.final_token,) if r.final_token >= 0 else ())
        return trace, emitted

    return run


def marginals(law, V):
    first = np.zeros(V)
    pair = np.zeros((V, V))
    for out, w in law.items():
        first[out[0]] += w
        if len(out) > 1:
            pair[out[0], out[1]] += w
    return first, pair


# ----------------------------------------------------------------- single child (Section 2)

def test_one_child_is_plain_speculative_sampling():
    """Token x ~ D accepted with probability min(1, T[x]/D[x]), otherwise a token from
    norm(relu(T-D)): acceptance probability is sum_x min(D,T) and the output follows T."""
    V, td, tt = 8, 0.6, 0.9
    rng = np.random.default_rng(3)
    draft = (rng.standard_normal((2, V)) * 2).astype(np.float32)
    target = (draft + rng.standard_normal((2, V))).astype(np.float32)
    D, T = probs(draft, td), probs(target, tt)
    law = exact_law(make_step(draft, target, 2, td, tt, emit_bonus=False))
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-12)
    # without the bonus token every outcome is one token: accepted child or residual sample
    first, _ = marginals(law, V)
    np.testing.assert_allclose(first, T[0], rtol=0, atol=1e-11)
    # acceptance probability through the explicit draws: accepted iff c < T[x]/D[x]
    acc = 0.0
    for x in range(V):
        edges = np.concatenate([[0.0], np.cumsum(D[0])])
        u_tok = 0.5 * (edges[x] + edges[x + 1]) / edges[-1]
        t = oracle.build_tree_explicit(draft, 2, td, [0.0, u_tok])
        assert t.token[1] == x
        ratio = oracle.accept_ratio_all(draft, target, t.token, t.first_child, t.next_sibling, td, tt)[1]
        assert ratio == pytest.approx(T[0, x] / D[0, x], rel=1e-12)
        for c, want in [(min(ratio, 1.0) * (1 - 1e-9), True), (min(ratio * (1 + 1e-9), TOP), ratio >= 1.0)]:
            r = oracle.verify_explicit(draft, target, t.token, t.first_child, t.next_sibling, td, tt,
                                       [0.0, c], [0.5, 0.5], emit_bonus=False)
            assert (r.n_accepted == 1) == want
        acc += D[0, x] * min(1.0, ratio)
    assert acc == pytest.approx(np.minimum(D[0], T[0]).sum(), rel=1e-12)


def test_one_child_residual_distribution():
    """On a reject the emitted token follows norm(relu(T-D)) (inverse CDF, ascending index)."""
    V = 8
    rng = np.random.default_rng(5)
    draft = (rng.standard_normal((2, V)) * 2).astype(np.float32)
    target = (draft + rng.standard_normal((2, V))).astype(np.float32)
    D, T = probs(draft, 1.0), probs(target, 1.0)
    res = np.maximum(T[0] - D[0], 0)
    res /= res.sum()
    x = int(np.argmax(D[0] - T[0]))            # a token the target likes less than the draft
    tok = np.array([-1, x], dtype=np.int32)
    fc, ns = np.array([1, -1], dtype=np.int32), np.array([-1, -1], dtype=np.int32)
    edges = np.concatenate([[0.0], np.cumsum(res)])
    for y in range(V):
        if res[y] <= 0:
            continue
        u = 0.5 * (edges[y] + edges[y + 1])
        r = oracle.verify_explicit(draft, target, tok, fc, ns, 1.0, 1.0, [0.0, TOP], [u, 0.5])
        assert r.n_accepted == 0 and r.final_token == y and r.stop_node == 0


# ----------------------------------------------------------------- trees of 1..4 nodes

@pytest.mark.parametrize("n_budget,V,seed", [(1, 4, 0), (2, 4, 1), (3, 4, 2), (4, 4, 3), (4, 3, 4)])
def test_exact_output_law_on_tiny_trees(n_budget, V, seed):
    """Enumerating every sampled tree and every verification outcome: the first emitted
    token follows Target(root) and the first two follow Target(root) x Target(next row),
    where all non-root rows share one target row so the product is well defined."""
    td, tt = 0.7, 1.0
    rng = np.random.default_rng(seed)
    draft = (rng.standard_normal((n_budget, V)) * 1.5).astype(np.float32)
    target = (draft + rng.standard_normal((n_budget, V))).astype(np.float32)
    target[1:] = target[1] if n_budget > 1 else 0
    T = probs(target, tt)
    law = exact_law(make_step(draft, target, n_budget, td, tt, emit_bonus=True))
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-10)
    first, pair = marginals(law, V)
    np.testing.assert_allclose(first, T[0], rtol=0, atol=1e-9)
    if n_budget > 1:
        # a second token exists whenever the first was an accepted node
        p_two = pair.sum()
        cond = pair / pair.sum(axis=1, keepdims=True).clip(1e-300)
        for x in range(V):
            if pair[x].sum() > 1e-9:
                np.testing.assert_allclose(cond[x], T[1], rtol=0, atol=1e-7)
        assert 0.0 < p_two <= 1.0


def test_exact_law_without_bonus_token():
    V, n_budget = 4, 3
    rng = np.random.default_rng(9)
    draft = (rng.standard_normal((n_budget, V)) * 1.5).astype(np.float32)
    target = (draft + rng.standard_normal((n_budget, V))).astype(np.float32)
    law = exact_law(make_step(draft, target, n_budget, 1.0, 0.8, emit_bonus=False))
    first, _ = marginals(law, V)
    np.testing.assert_allclose(first, probs(target, 0.8)[0], rtol=0, atol=1e-9)


def test_exact_law_fixed_two_siblings_residual_update():
    """Hand-built root with three children (tokens 2,0,3): probability that child k is the
    accepted one, by the recursive rejection rule written out with fractions of the
    residuals, against the oracle integrated over its uniforms."""
    V = 4
    D0 = np.array([0.4, 0.3, 0.2, 0.1])
    T0 = np.array([0.1, 0.2, 0.3, 0.4])
    draft = np.log(np.stack([D0] * 4)).astype(np.float32)
    target = np.log(np.stack([T0] * 4)).astype(np.float32)
    tok = np.array([-1, 2, 0, 3], dtype=np.int32)
    fc = np.array([1, -1, -1, -1], dtype=np.int32)
    ns = np.array([-1, 2, 3, -1], dtype=np.int32)
    law = exact_law(make_step(draft, target, 4, 1.0, 1.0, emit_bonus=False, fixed_tree=(tok, fc, ns)))
    # by hand: child 1 (token 2): ratio 0.3/0.2 > 1 -> always accepted
    assert law == pytest.approx({(2,): 1.0}, abs=1e-12)
    # reorder so rejections happen: children tokens 0,1,3
    tok2 = np.array([-1, 0, 1, 3], dtype=np.int32)
    law2 = exact_law(make_step(draft, target, 4, 1.0, 1.0, emit_bonus=False, fixed_tree=(tok2, fc, ns)))
    # child token 0: accept prob 0.1/0.4 = 0.25.  reject -> R=norm(relu(T-D))=(0,0,.1,.3)/.4=(0,0,.25,.75),
    # D=(0,.3,.2,.1)/.6.  child token 1: R[1]=0 -> rejected.  R=norm(relu(R-D)): R-D=(0,-.5,.25-.333,.75-.1667)
    # -> (0,0,0,1); D=(0,0,.2,.1)/.3.  child token 3: ratio 1/(1/3) > 1 -> accepted.
    assert law2 == pytest.approx({(0,): 0.25, (3,): 0.75}, abs=1e-7)


def test_sibling_order_and_residual_updates_by_hand():
    """V=2, draft (.5,.5), target (.8,.2), children tokens (1,0).  Child token 1 has ratio
    .2/.5 = .4, so c = .9 rejects it; then R = norm(relu((.8,.2)-(.5,.5))) = (1,0) and
    D = (1,0): child token 0 has ratio 1 and is accepted by any c < 1."""
    draft = np.log(np.array([[0.5, 0.5]] * 3)).astype(np.float32)
    target = np.log(np.array([[0.8, 0.2]] * 3)).astype(np.float32)
    tok = np.array([-1, 1, 0], dtype=np.int32)
    fc = np.array([1, -1, -1], dtype=np.int32)
    ns = np.array([-1, 2, -1], dtype=np.int32)
    r = oracle.verify_explicit(draft, target, tok, fc, ns, 1.0, 1.0, [0, 0.9, TOP], [0.5] * 3, emit_bonus=False)
    assert list(r.accepted_nodes) == [2]
    assert r.tested_margin[1] == pytest.approx(0.5, abs=1e-6)
    r = oracle.verify_explicit(draft, target, tok, fc, ns, 1.0, 1.0, [0, 0.39, TOP], [0.5] * 3, emit_bonus=False)
    assert list(r.accepted_nodes) == [1]
    # with child token 1 alone: after the reject the final token comes from R = (1,0)
    ns1 = np.array([-1, -1, -1], dtype=np.int32)
    for u in (0.0, 0.5, TOP):
        r = oracle.verify_explicit(draft, target, tok, fc, ns1, 1.0, 1.0, [0, 0.9, 0], [u] * 3)
        assert r.n_accepted == 0 and r.final_token == 0 and r.stop_node == 0


def test_leaf_bonus_token_and_printed_variant():
    """A walk that ends on a leaf emits one more token from the leaf's target row when
    emit_bonus is set, and nothing (as Algorithm 3 is printed) when it is not."""
    one = np.zeros((2, 1), dtype=np.float32)
    tok, fc, ns = (np.array([-1, 0], dtype=np.int32), np.array([1, -1], dtype=np.int32),
                   np.array([-1, -1], dtype=np.int32))
    r = oracle.verify_explicit(one, one, tok, fc, ns, 1.0, 1.0, [0, TOP], [0.5, 0.5], emit_bonus=True)
    assert list(r.accepted_nodes) == [1] and r.final_token == 0 and r.stop_node == 1
    r = oracle.verify_explicit(one, one, tok, fc, ns, 1.0, 1.0, [0, TOP], [0.5, 0.5], emit_bonus=False)
    assert list(r.accepted_nodes) == [1] and r.final_token == -1


def test_draft_exhausted_exit_is_taken():
    """The "D is all 0" exit of Algorithm 3 needs a reject that leaves the draft empty:
    draft one-hot on token 1 (logit gap beyond fp64 exp range), target one-hot on token 0,
    one child with token 1.  R[1] = 0 rejects for every c; D becomes all zero; the final
    token comes from the residual (1,0)."""
    draft = np.array([[-3000.0, 0.0]] * 2, dtype=np.float32)
    target = np.array([[0.0, -3000.0]] * 2, dtype=np.float32)
    tok, fc, ns = (np.array([-1, 1], dtype=np.int32), np.array([1, -1], dtype=np.int32),
                   np.array([-1, -1], dtype=np.int32))
    for c in (0.0, 0.5, TOP):
        r = oracle.verify_explicit(draft, target, tok, fc, ns, 1.0, 1.0, [0, c], [0.7, 0.7])
        assert r.n_accepted == 0 and r.final_token == 0 and r.stop_node == 0


# ----------------------------------------------------------------- statistical

def test_million_trial_marginals_match_target():
    """10^6 seeded steps at V=8 with Philox draws: first-token counts against Target(root)
    (chi-square, 7 dof) and second-token counts against the shared non-root target row."""
    V, n_budget, n = 8, 6, 1_000_000
    rng = np.random.default_rng(2024)
    draft = (rng.standard_normal((n_budget, V)) * 2).astype(np.float32)
    target = (draft + rng.standard_normal((n_budget, V)) * 0.8).astype(np.float32)
    target[1:] = target[1]
    T = probs(target, 0.9)
    c1, c2, mean_acc = oracle.monte_carlo(draft, target, n_budget, 0.6, 0.9, 12345, n)
    assert c1.sum() == n
    chi2 = ((c1 - n * T[0]) ** 2 / (n * T[0])).sum()
    assert chi2 < 29.9                       # 7 dof, p ~ 1e-4
    second = c2.sum(axis=0)
    m = second.sum()
    chi2b = ((second - m * T[1]) ** 2 / (m * T[1])).sum()
    assert chi2b < 29.9
    assert 0.5 < mean_acc < n_budget


def test_philox_and_explicit_variants_agree():
    """The Philox-driven entry points equal the explicit ones fed with the same uniforms
    (derived here from the path keys with the oracle's own u01 helper)."""
    V, N, seed, seq = 50, 12, 77, 3
    rng = np.random.default_rng(8)
    draft = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    target = (draft + rng.standard_normal((N, V))).astype(np.float32)
    t = oracle.build_tree(draft, N, 0.8, seed, seq)
    keys = {0: (seq, 0)}
    ub, ua, ur = np.zeros(N), np.zeros(N), np.zeros(N)
    for i in range(1, N):
        p, r = int(t.parent[i]), int(t.sib_rank[i])
        w = oracle.philox4x32_10([keys[p][0], keys[p][1], r, oracle.KIND_PATH], [seed, 0])
        keys[i] = (int(w[0]), int(w[1]))
        ub[i] = oracle.u01(seed, keys[p][0], keys[p][1], r, oracle.KIND_BUILD)
    for i in range(N):
        ua[i] = oracle.u01(seed, keys[i][0], keys[i][1], 0, oracle.KIND_ACCEPT)
        ur[i] = oracle.u01(seed, keys[i][0], keys[i][1], 0, oracle.KIND_RESID)
    t2 = oracle.build_tree_explicit(draft, N, 0.8, ub)
    assert np.array_equal(t.parent, t2.parent) and np.array_equal(t.token, t2.token)
    a = oracle.verify(draft, target, t.token, t.first_child, t.next_sibling, 0.8, 1.0, seed, seq)
    b = oracle.verify_explicit(draft, target, t.token, t.first_child, t.next_sibling, 0.8, 1.0, ua, ur)
    assert list(a.accepted_nodes) == list(b.accepted_nodes) and a.final_token == b.final_token


# ----------------------------------------------------------------- checkers the GPU tests lean on

@pytest.mark.parametrize("td,tt", [(0.6, 0.9), (0.9, 1.3), (1.3, 0.6)])
def test_softmax_stats_against_logsumexp_at_general_temperatures(td, tt):
    """Row statistics (max of logits/T, sum of exp(logits/T - max)) for draft and target at
    temperatures other than 1: max + log(sum) is the log-sum-exp of the scaled row, and the
    maximum is the largest scaled logit (library routines in fp64)."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(11)
    draft = (rng.standard_normal((5, 97)) * 3).astype(np.float32)
    target = (draft + rng.standard_normal((5, 97)) * 0.8).astype(np.float32)
    st = oracle.softmax_stats(draft, target, td, tt)
    for col, table, temp in ((0, draft, td), (2, target, tt)):
        z = table.astype(np.float64) / temp
        np.testing.assert_allclose(st[:, col], z.max(axis=1), rtol=1e-12, atol=0)
        np.testing.assert_allclose(st[:, col] + np.log(st[:, col + 1]), logsumexp(z, axis=1), rtol=1e-12, atol=0)
        # and the pair normalises the row: exp(z - max) / sum adds up to one
        p = np.exp(z - st[:, col, None]) / st[:, col + 1, None]
        np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-12)
    # a wrong 1/T on either half shows: the two temperatures differ, so do the halves on one table
    same = oracle.softmax_stats(draft, draft, td, tt)
    assert not np.allclose(same[:, 0], same[:, 2])


def test_accept_ratio_of_later_siblings_by_hand():
    """Draft (.4,.3,.2,.1), target (.1,.2,.3,.4), children with tokens 0, 1, 3 under the root
    (the inner loop of Algorithm 3 with every earlier sibling rejected).  By hand:
    child 0: R[0]/D[0] = .1/.4 = 0.25; then R = norm(relu(T-D)) = (0,0,.25,.75), D = (0,.3,.2,.1)/.6;
    child 1: R[1]/D[1] = 0/.5 = 0; then R-D = (0,-.5,.25-1/3,.75-1/6) -> R = (0,0,0,1), D = (0,0,2/3,1/3);
    child 3: R[3]/D[3] = 1/(1/3) = 3."""
    D0 = np.array([0.4, 0.3, 0.2, 0.1])
    T0 = np.array([0.1, 0.2, 0.3, 0.4])
    draft = np.log(np.stack([D0] * 4)).astype(np.float32)
    target = np.log(np.stack([T0] * 4)).astype(np.float32)
    tok = np.array([-1, 0, 1, 3], dtype=np.int32)
    fc = np.array([1, -1, -1, -1], dtype=np.int32)
    ns = np.array([-1, 2, 3, -1], dtype=np.int32)
    ratio = oracle.accept_ratio_all(draft, target, tok, fc, ns, 1.0, 1.0)
    np.testing.assert_allclose(ratio, [0.0, 0.25, 0.0, 3.0], rtol=0, atol=2e-7)   # logits are fp32 logs
    # with temperatures: D = softmax(log D0 / td), T = softmax(log T0 / tt), same recursion in numpy
    td, tt = 0.6, 1.3
    D, R = probs(np.log(D0).astype(np.float32), td), probs(np.log(T0).astype(np.float32), tt)
    want = {}
    for node, y in ((1, 0), (2, 1), (3, 3)):
        want[node] = R[y] / D[y]
        R = np.maximum(R - D, 0)
        R /= R.sum()
        D = D.copy()
        D[y] = 0
        D /= D.sum()
    ratio = oracle.accept_ratio_all(draft, target, tok, fc, ns, td, tt)
    np.testing.assert_allclose(ratio[1:], [want[1], want[2], want[3]], rtol=1e-12)


def test_accept_ratio_agrees_with_the_walk_on_built_trees():
    """On greedy trees over random tables: for every child the walk tests, |c - ratio| from
    accept_ratio_all equals the margin the verification walk itself recorded (residual update of
    Algorithm 3 after each rejected sibling, general target)."""
    V, N, td, tt = 16, 24, 0.8, 1.1
    later = 0
    for seed in range(6):
        rng = np.random.default_rng(40 + seed)
        draft = (rng.standard_normal((N, V)) * 1.5).astype(np.float32)
        target = (draft + rng.standard_normal((N, V)) * 1.2).astype(np.float32)
        t = oracle.build_tree(draft, N, td, seed)
        ratio = oracle.accept_ratio_all(draft, target, t.token, t.first_child, t.next_sibling, td, tt)
        for trial in range(40):
            ua = np.random.default_rng(1000 * seed + trial).random(N)
            r = oracle.verify_explicit(draft, target, t.token, t.first_child, t.next_sibling, td, tt, ua, [0.5] * N)
            tested = np.flatnonzero(np.isfinite(r.tested_margin))
            assert tested.size > 0
            for i in tested:
                assert abs(ua[i] - ratio[i]) == pytest.approx(r.tested_margin[i], rel=1e-9, abs=1e-12)
                later += int(t.sib_rank[i] > 0)
    assert later > 50          # the check reached siblings behind a residual update
