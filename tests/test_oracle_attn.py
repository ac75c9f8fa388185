"""Pins for the oracle's tree-masked attention (Section 2, "Tree Attention")."""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def causal_attention(q, k, v, n_prefix, scale):
    """Textbook causal attention over the concatenated sequence: query t (the t-th of the
    last N positions) sees positions 0..n_prefix+t.  q [N,H,d]; k,v [S,Hkv,d]."""
    N, Hq, d = q.shape
    S, Hkv = k.shape[0], k.shape[1]
    G = Hq // Hkv
    out = np.zeros((N, Hq, d))
    for h in range(Hq):
        kk = k[:, h // G].astype(np.float64)
        vv = v[:, h // G].astype(np.float64)
        s = q[:, h].astype(np.float64) @ kk.T * scale
        allowed = np.arange(S)[None, :] <= (n_prefix + np.arange(N))[:, None]
        s = np.where(allowed, s, -np.inf)
        out[:, h] = sp_softmax(s, axis=-1) @ vv
    return out


@pytest.mark.parametrize("N,P,Hq,Hkv,d", [(9, 17, 4, 4, 16), (70, 5, 4, 2, 8), (5, 0, 2, 1, 4)])
def test_chain_tree_is_causal_attention(N, P, Hq, Hkv, d):
    q, kp, vp = rnd((N, Hq, d), 1), rnd((P, Hkv, d), 2), rnd((P, Hkv, d), 3)
    kt, vt = rnd((N, Hkv, d), 4), rnd((N, Hkv, d), 5)
    mask = oracle.ancestor_mask(np.arange(-1, N - 1))
    got = oracle.tree_attn(q, kp, vp, kt, vt, mask, 0.37)
    want = causal_attention(q, np.concatenate([kp, kt]), np.concatenate([vp, vt]), P, 0.37)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_single_node_is_decode_attention():
    P, Hq, Hkv, d = 33, 6, 3, 8
    q, kp, vp, kt, vt = rnd((1, Hq, d), 1), rnd((P, Hkv, d), 2), rnd((P, Hkv, d), 3), rnd((1, Hkv, d), 4), rnd((1, Hkv, d), 5)
    got = oracle.tree_attn(q, kp, vp, kt, vt, np.array([[1]], dtype=np.uint64), 0.5)
    for h in range(Hq):
        g = h // 2
        k = np.concatenate([kp[:, g], kt[:, g]]).astype(np.float64)
        v = np.concatenate([vp[:, g], vt[:, g]]).astype(np.float64)
        w = sp_softmax(k @ q[0, h].astype(np.float64) * 0.5)
        np.testing.assert_allclose(got[0, h], w @ v, rtol=1e-11, atol=1e-13)


def test_triple_loop_on_a_branching_tree():
    """Brute force with explicit ancestor sets on a small branching tree, GQA 4/2."""
    parent = np.array([-1, 0, 0, 1, 1, 2, 5, 0], dtype=np.int32)
    N, P, Hq, Hkv, d = 8, 3, 4, 2, 5
    q, kp, vp = rnd((N, Hq, d), 11), rnd((P, Hkv, d), 12), rnd((P, Hkv, d), 13)
    kt, vt = rnd((N, Hkv, d), 14), rnd((N, Hkv, d), 15)
    got = oracle.tree_attn(q, kp, vp, kt, vt, oracle.ancestor_mask(parent), 0.8)
    for j in range(N):
        vis, a = [], j
        while a >= 0:
            vis.append(a)
            a = parent[a]
        for h in range(Hq):
            g = h // 2
            keys = [kp[k, g] for k in range(P)] + [kt[i, g] for i in vis]
            vals = [vp[k, g] for k in range(P)] + [vt[i, g] for i in vis]
            s = [0.8 * sum(float(q[j, h, c]) * float(kv[c]) for c in range(d)) for kv in keys]
            m = max(s)
            e = [np.exp(x - m) for x in s]
            z = sum(e)
            for c in range(d):
                want = sum(e[i] / z * float(vals[i][c]) for i in range(len(keys)))
                assert got[j, h, c] == pytest.approx(want, rel=1e-11, abs=1e-13)


def test_star_tree_rows_see_prefix_root_and_self_only():
    N, P, H, d = 6, 4, 2, 4
    parent = np.array([-1, 0, 0, 0, 0, 0], dtype=np.int32)
    q, kp, vp, kt, vt = rnd((N, H, d), 1), rnd((P, H, d), 2), rnd((P, H, d), 3), rnd((N, H, d), 4), rnd((N, H, d), 5)
    base = oracle.tree_attn(q, kp, vp, kt, vt, oracle.ancestor_mask(parent), 1.0)
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[3] += 10.0
    vt2[3] -= 5.0                       # perturb node 3: only row 3 may change
    pert = oracle.tree_attn(q, kp, vp, kt2, vt2, oracle.ancestor_mask(parent), 1.0)
    changed = [j for j in range(N) if not np.allclose(base[j], pert[j], rtol=0, atol=1e-14)]
    assert changed == [3]


def test_prefix_permutation_invariance_and_rows_subset():
    N, P, Hq, Hkv, d = 12, 20, 4, 2, 8
    logits = np.random.default_rng(0).standard_normal((N, 30)).astype(np.float32)
    t = oracle.build_tree(logits, N, 1.0, 0)
    q, kp, vp = rnd((N, Hq, d), 21), rnd((P, Hkv, d), 22), rnd((P, Hkv, d), 23)
    kt, vt = rnd((N, Hkv, d), 24), rnd((N, Hkv, d), 25)
    a = oracle.tree_attn(q, kp, vp, kt, vt, t.mask, 0.3)
    perm = np.random.default_rng(1).permutation(P)
    b = oracle.tree_attn(q, kp[perm], vp[perm], kt, vt, t.mask, 0.3)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    rj, rh = np.array([0, 5, 11, 7]), np.array([3, 0, 2, 1])
    rows = oracle.tree_attn_rows(q, kp, vp, kt, vt, t.mask, 0.3, rj, rh)
    np.testing.assert_array_equal(rows, a[rj, rh])
