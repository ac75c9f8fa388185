"""GPU parity of dyspec_verify with a temperature-0 target (Section 5's temperature-0 rows):
row statistics carry (largest target logit, its index), the walk follows the target's argmax
token down the tree; checked against the CPU oracle and against a plain argmax walk."""
import numpy as np
import pytest

from helpers import compare_trees, compare_verify, oracle_trees, verify_in_full
from test_oracle_temp0 import greedy_walk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


def logits(n, V, sigma, tsigma, seed):
    rng = np.random.default_rng(seed)
    d = (rng.standard_normal((n, V)) * sigma).astype(np.float32)
    t = (d + rng.standard_normal((n, V)) * tsigma).astype(np.float32)
    return d, t


CASES = [
    # (nodes per seq, V, sigma, target sigma, draft temps, target temps, seed)
    ((32,), 1000, 2.0, 0.5, (1.0,), (0.0,), 0),
    ((40,), 130, 2.0, 0.3, (0.7,), (0.0,), 1),                         # scalar-load statistics kernel
    ((13,), 3, 1.0, 1.0, (1.0,), (0.0,), 2),                           # tiny vocabulary: drafts run out
    ((128,), 32000, 3.0, 0.3, (0.6,), (0.0,), 3),                      # 7B-shaped logits, sharp agreement
    ((64, 7, 200, 1), 5000, 3.0, 0.5, (0.6, 1.0, 0.8, 1.0), (0.0, 0.7, 0.0, 0.0), 4),   # mixed batch
    ((300,), 32768, 3.0, 0.8, (0.6,), (0.0,), 5),                      # largest vocabulary
    ((2,), 8, 1.0, 1.0, (0.9,), (0.0,), 6),
    ((1,), 64, 1.0, 1.0, (1.0,), (0.0,), 7),                           # root only: bonus token = argmax
]


@pytest.mark.parametrize("nodes,V,sigma,tsigma,td,tt,seed", CASES)
def test_temperature_zero_target_matches_oracle(dy, nodes, V, sigma, tsigma, td, tt, seed):
    print(f"case nodes={nodes} V={V} seed={seed}", flush=True)
    batch = dy.Batch.from_sizes(nodes)
    d, t = logits(sum(nodes), V, sigma, tsigma, 300 + seed)
    dd, tg = torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda()
    built = dy.build_tree(dd, batch, td, seed)
    torch.cuda.synchronize()
    trees = oracle_trees(d, nodes, td, seed)
    assert compare_trees(built, batch, trees) == len(nodes)
    for bonus in (True, False):
        for vseed in (seed, seed + 91):
            out, _ = verify_in_full(lambda sd: dy.verify(dd, tg, batch, built.tree, td, tt, sd, emit_bonus=bonus),
                                    batch, trees, d, t, td, tt, vseed, emit_bonus=bonus)
            # the outcome of a temperature-0 sequence does not depend on the draws at all: it
            # is the argmax walk, low-margin draws included
            na, fin = out.n_accepted.cpu().numpy(), out.final_token.cpu().numpy()
            acc = out.accepted_nodes.cpu().numpy()
            for s, tr in enumerate(trees):
                if tt[s] != 0.0:
                    continue
                a, b = int(batch.node_offset[s]), int(batch.node_offset[s + 1])
                path, last, _ = greedy_walk(t[a:b], tr.token, tr.first_child, tr.next_sibling, bonus)
                assert list(acc[a:a + na[s]]) == path, f"seq {s}"
                assert fin[s] == last, f"seq {s}"


def test_ties_go_to_the_smallest_index(dy):
    """Target logits on a coarse grid so that every row's maximum is shared by several
    tokens, in both statistics kernels (V % 4 == 0 and not)."""
    for V, n in ((4096, 24), (4099, 24), (32000, 16)):
        rng = np.random.default_rng(V)
        d = (rng.standard_normal((n, V)) * 2.0).astype(np.float32)
        t = np.minimum(np.round(d + rng.standard_normal((n, V))), 4.0).astype(np.float32)
        assert ((t == t.max(axis=1, keepdims=True)).sum(axis=1) > 1).all()
        batch = dy.Batch.from_sizes([n])
        dd, tg = torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda()
        built = dy.build_tree(dd, batch, (1.0,), 1)
        out = dy.verify(dd, tg, batch, built.tree, (1.0,), (0.0,), 1)
        torch.cuda.synchronize()
        st = out.row_stats.cpu().numpy()
        np.testing.assert_array_equal(st[:, 3], np.argmax(t, axis=1).astype(np.float32))
        np.testing.assert_array_equal(st[:, 2], t.max(axis=1))
        trees = oracle_trees(d, (n,), (1.0,), 1)
        assert compare_verify(out, batch, trees, d, t, (1.0,), (0.0,), 1) == (1, 0)


def test_full_size_tree_long_accepted_path(dy):
    """The 70B-shaped step (512 rows of 32000 logits) with a target that mostly agrees with
    the draft: accepted paths of several tokens, equal to the oracle's and to the argmax walk."""
    from paper_2410_11744_amd import synth
    cfg = synth.CONFIGS["llama2_70b"]
    d, _ = synth.make_logits(cfg)
    rng = np.random.default_rng(11)
    t = (d + 0.25 * rng.standard_normal(d.shape, dtype=np.float32)).astype(np.float32)
    batch = dy.Batch.from_sizes(cfg.n_nodes)
    dd, tg = torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda()
    built = dy.build_tree(dd, batch, cfg.temps, cfg.seed)
    torch.cuda.synchronize()
    trees = oracle_trees(d, cfg.n_nodes, cfg.temps, cfg.seed)
    assert compare_trees(built, batch, trees) == 1
    out = dy.verify(dd, tg, batch, built.tree, cfg.temps, (0.0,), cfg.seed)
    torch.cuda.synchronize()
    assert compare_verify(out, batch, trees, d, t, cfg.temps, (0.0,), cfg.seed) == (1, 0)
    tr = trees[0]
    path, last, _ = greedy_walk(t, tr.token, tr.first_child, tr.next_sibling)
    na = int(out.n_accepted.item())
    assert list(out.accepted_nodes.cpu().numpy()[:na]) == path and out.final_token.item() == last
    assert na >= 2


def test_negative_target_temperature_is_rejected(dy):
    batch = dy.Batch.from_sizes([4])
    d = torch.zeros((4, 16), device="cuda")
    built = dy.build_tree(d, batch, (1.0,), 0)
    with pytest.raises(dy.DyspecError) as e:
        dy.verify(d, d, batch, built.tree, (1.0,), (-0.5,), 0)
    assert e.value.status == -1
    with pytest.raises(dy.DyspecError) as e:
        dy.verify(d, d, batch, built.tree, (0.0,), (1.0,), 0)        # the draft must stay a distribution to sample
    assert e.value.status == -1
