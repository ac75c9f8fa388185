"""GPU parity: dyspec_dfs_reorder against the oracle (bit-exact), and tree attention /
verification on the renamed tree against the results on the original one."""
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


def host_tree(tree, a, b):
    return {k: getattr(tree, k).cpu().numpy()[a:b] for k in ("parent", "token", "sib_rank", "first_child", "next_sibling", "depth")}


def check_against_oracle(dy, batch, tree, re):
    order = re.order.cpu().numpy()
    mask = re.anc_mask.cpu().numpy().view(np.uint64)
    for s in range(batch.n_seq):
        a, b = int(batch.node_offset[s]), int(batch.node_offset[s + 1])
        t = host_tree(tree, a, b)
        want_order = oracle.dfs_order(t["parent"], t["first_child"], t["next_sibling"])
        assert np.array_equal(order[a:b], want_order), f"sequence {s}: order"
        par, tok, rk, fc, ns, dep, m = oracle.relabel_tree(want_order, t["parent"], t["token"], t["sib_rank"],
                                                           t["first_child"], t["next_sibling"], t["depth"])
        got = host_tree(re.tree, a, b)
        for name, want in (("parent", par), ("token", tok), ("sib_rank", rk), ("first_child", fc),
                           ("next_sibling", ns), ("depth", dep)):
            assert np.array_equal(got[name], want), f"sequence {s}: {name}"
        words = m.shape[1]
        assert np.array_equal(mask[a:b, :words], m), f"sequence {s}: mask"
        assert not mask[a:b, words:].any()


@pytest.mark.parametrize("nodes,V,seed", [((32,), 1000, 0), ((300,), 5000, 1), ((64, 7, 200, 1), 3000, 2), ((1024,), 2000, 3)])
def test_reorder_of_built_trees_matches_oracle(dy, nodes, V, seed):
    rng = np.random.default_rng(seed)
    d = (rng.standard_normal((sum(nodes), V)) * 3.0).astype(np.float32)
    batch = dy.Batch.from_sizes(nodes)
    built = dy.build_tree(torch.from_numpy(d).cuda(), batch, (0.8,) * len(nodes), seed)
    re = dy.dfs_reorder(built.tree, batch)
    torch.cuda.synchronize()
    check_against_oracle(dy, batch, built.tree, re)


def device_tree(dy, parent, fc, ns, dep, rk, tok):
    mk = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    return dy.Tree(mk(parent), mk(tok), mk(rk), mk(fc), mk(ns), mk(dep))


def test_reorder_of_hand_made_trees(dy):
    # a chain, a star, a tree with rows that were never attached, all in one batch
    n = 70
    chain = np.arange(-1, n - 1, dtype=np.int32)
    star = np.array([-1] + [0] * (n - 1), dtype=np.int32)
    part = np.array([-1, 0, 0, 1, -1, -1], dtype=np.int32)
    pars, fcs, nss, deps, rks = [], [], [], [], []
    for p in (chain, star, part):
        live = p.copy()
        fc, ns, dep = oracle.links_from_parent(live)
        rk = np.zeros(len(p), np.int32)
        for v in range(len(p)):
            c, r = fc[v], 0
            while c >= 0:
                rk[c] = r
                r += 1
                c = ns[c]
        pars.append(p); fcs.append(fc); nss.append(ns); deps.append(dep); rks.append(rk)
    cat = lambda xs: np.concatenate(xs)
    batch = dy.Batch.from_sizes([n, n, len(part)])
    tok = np.arange(2 * n + len(part), dtype=np.int32)
    tree = device_tree(dy, cat(pars), cat(fcs), cat(nss), cat(deps), cat(rks), tok)
    re = dy.dfs_reorder(tree, batch)
    torch.cuda.synchronize()
    check_against_oracle(dy, batch, tree, re)
    assert re.order.cpu().numpy()[2 * n:].tolist() == [0, 1, 3, 2, 4, 5]


def test_links_that_are_no_tree_do_not_hang(dy):
    # next_sibling cycle and a parent cycle: the walk must stop, every row still gets a place
    n = 8
    parent = np.array([-1, 0, 1, 2, 3, 4, 5, 6], np.int32)
    parent[3] = 5                                   # 3 -> 5 -> 4 -> 3: a cycle above node 3
    fc = np.array([1, 2, 3, 4, 5, 6, 7, -1], np.int32)
    ns = np.array([-1, 99, -1, 3, -1, -1, -5, -1], np.int32)   # out-of-range links, a self loop
    z = np.zeros(n, np.int32)
    batch = dy.Batch.from_sizes([n])
    re = dy.dfs_reorder(device_tree(dy, parent, fc, ns, z, z, z), batch)
    torch.cuda.synchronize()
    assert sorted(re.order.cpu().tolist()) == list(range(n))


@pytest.mark.parametrize("nodes,prefix,Hq,Hkv", [((200,), (300,), 8, 2), ((96, 40), (0, 130), 4, 4)])
def test_attention_on_the_renamed_tree_is_the_permuted_result(dy, nodes, prefix, Hq, Hkv):
    rng = np.random.default_rng(5)
    V, d = 4000, 128
    batch = dy.Batch.from_sizes(nodes, prefix)
    logits = (rng.standard_normal((sum(nodes), V)) * 3.0).astype(np.float32)
    built = dy.build_tree(torch.from_numpy(logits).cuda(), batch, (0.7,) * len(nodes), 9)
    re = dy.dfs_reorder(built.tree, batch)
    g = torch.Generator().manual_seed(3)
    mk = lambda *sh: torch.randn(sh, generator=g, dtype=torch.float32).to(torch.bfloat16)
    tn, tp = sum(nodes), sum(prefix)
    q, kp, vp, kt, vt = mk(tn, Hq, d), mk(tp, Hkv, d), mk(tp, Hkv, d), mk(tn, Hkv, d), mk(tn, Hkv, d)
    scale = 1.0 / math.sqrt(d)
    dev = lambda t: t.cuda() if t.numel() else torch.empty(t.shape, dtype=t.dtype, device="cuda")
    idx = re.gather_index(batch)
    out_new = dy.tree_attn(dev(q)[idx], dev(kp), dev(vp), dev(kt)[idx], dev(vt)[idx], re.anc_mask, batch, scale)
    torch.cuda.synchronize()
    # the oracle on the ORIGINAL order, rows then permuted
    host = [t.float().numpy() for t in (q, kp, vp, kt, vt)]
    mask = built.anc_mask.cpu().numpy().view(np.uint64)
    got = out_new.float().cpu().numpy()
    order = re.order.cpu().numpy()
    for s, n in enumerate(nodes):
        a = int(batch.node_offset[s])
        rj, rh = np.divmod(np.arange(n * Hq), Hq)
        want = oracle_attention_rows(*host, mask, batch, s, scale, rj, rh).reshape(n, Hq, d)
        err = np.abs(got[a:a + n] - want[order[a:a + n]]).max()
        assert err <= ATTN_TOL["bf16"], f"sequence {s}: max abs error {err}"


def test_verification_of_the_renamed_tree_gives_the_same_tokens(dy):
    # draws are named by paths of sibling ranks and rows travel with their nodes, so the walk
    # over the renamed tree accepts the same nodes and emits the same token
    rng = np.random.default_rng(11)
    nodes, V = (150, 60), 3000
    batch = dy.Batch.from_sizes(nodes)
    d = (rng.standard_normal((sum(nodes), V)) * 3.0).astype(np.float32)
    t = (d + rng.standard_normal((sum(nodes), V)) * 0.8).astype(np.float32)
    dd, tt = torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda()
    temps = (0.7, 1.0)
    for seed in range(6):
        built = dy.build_tree(dd, batch, temps, seed)
        re = dy.dfs_reorder(built.tree, batch)
        idx = re.gather_index(batch)
        a = dy.verify(dd, tt, batch, built.tree, temps, temps, seed)
        b = dy.verify(dd[idx].contiguous(), tt[idx].contiguous(), batch, re.tree, temps, temps, seed)
        torch.cuda.synchronize()
        assert torch.equal(a.n_accepted, b.n_accepted) and torch.equal(a.final_token, b.final_token)
        order = re.order.cpu().numpy()
        acc_a, acc_b = a.accepted_nodes.cpu().numpy(), b.accepted_nodes.cpu().numpy()
        for s in range(batch.n_seq):
            off, k = int(batch.node_offset[s]), int(a.n_accepted[s])
            assert order[off + acc_b[off:off + k]].tolist() == acc_a[off:off + k].tolist()
