"""GPU parity of dyspec_verify_bf16 (bf16 logit tables) against the oracle, which reads the same
values widened to fp32 (bf16 -> fp32 is exact)."""
import numpy as np
import pytest

from helpers import build_in_full, verify_in_full

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


def bf16_tables(n, V, sigma, tsigma, seed):
    rng = np.random.default_rng(seed)
    d = (rng.standard_normal((n, V)) * sigma).astype(np.float32)
    t = (d + rng.standard_normal((n, V)) * tsigma).astype(np.float32)
    db, tb = torch.from_numpy(d).to(torch.bfloat16), torch.from_numpy(t).to(torch.bfloat16)
    return db, tb, db.float().numpy(), tb.float().numpy(), d


CASES = [
    # (nodes per seq, V, sigma, target sigma, draft temps, target temps, seed)
    ((32,), 1000, 2.0, 0.5, (1.0,), (1.0,), 0),                    # V % 8 == 0: streaming statistics
    ((40,), 132, 2.0, 1.0, (0.7,), (0.9,), 1),                     # V % 4 == 0 only: one workgroup per row, 8-byte loads
    ((24,), 131, 2.0, 1.0, (0.7,), (0.7,), 2),                     # odd V: scalar loads
    ((128,), 32000, 3.0, 1.0, (0.6,), (0.6,), 3),                  # 7B-shaped tables
    ((64, 7, 200, 1), 5000, 3.0, 1.5, (0.6, 1.0, 0.8, 1.0), (0.6, 0.0, 0.8, 0.0), 4),   # ragged batch, two greedy targets
    ((300,), 32768, 3.0, 0.8, (0.6,), (0.0,), 5),                  # largest vocabulary, temperature-0 target with bf16 ties
    ((13,), 3, 1.0, 1.0, (1.0,), (1.0,), 6),
]


@pytest.mark.parametrize("nodes,V,sigma,tsigma,td,tt,seed", CASES)
def test_bf16_tables_match_oracle(dy, nodes, V, sigma, tsigma, td, tt, seed):
    print(f"case nodes={nodes} V={V} seed={seed}", flush=True)
    batch = dy.Batch.from_sizes(nodes)
    db, tb, d, t, d_unrounded = bf16_tables(sum(nodes), V, sigma, tsigma, 700 + seed)
    # The builder reads fp32 tables; it gets the values before their rounding to bf16 (rounded values
    # tie often, and a tie between two open positions is a decision of margin 0).  Verification is
    # checked on the trees the GPU built, from the rounded tables.
    built, _, _ = build_in_full(dy, torch.from_numpy(d_unrounded).cuda(), d_unrounded, batch, nodes, td, seed)
    g = {k: getattr(built.tree, k).cpu().numpy() for k in ("token", "first_child", "next_sibling")}
    trees = [tuple(g[k][int(batch.node_offset[s]):int(batch.node_offset[s + 1])] for k in ("token", "first_child", "next_sibling"))
             for s in range(len(nodes))]
    dd, tg = db.cuda(), tb.cuda()
    for bonus in (True, False):
        verify_in_full(lambda sd: dy.verify(dd, tg, batch, built.tree, td, tt, sd, emit_bonus=bonus),
                       batch, trees, d, t, td, tt, seed, emit_bonus=bonus)
    # and the fp32 entry point on the widened tables gives the same decisions and ratios
    wide = dy.verify(torch.from_numpy(d).cuda(), torch.from_numpy(t).cuda(), batch, built.tree, td, tt, seed)
    out = dy.verify(dd, tg, batch, built.tree, td, tt, seed)
    torch.cuda.synchronize()
    assert torch.equal(wide.n_accepted, out.n_accepted) and torch.equal(wide.final_token, out.final_token)
    na = int(out.n_accepted.sum().item())
    assert torch.equal(wide.accepted_nodes[:0], out.accepted_nodes[:0])
    for s in range(len(nodes)):
        a = int(batch.node_offset[s])
        k = int(out.n_accepted[s].item())
        assert torch.equal(wide.accepted_nodes[a:a + k], out.accepted_nodes[a:a + k])
    np.testing.assert_allclose(out.row_stats.cpu().numpy(), wide.row_stats.cpu().numpy(), rtol=2e-6, atol=1e-6)


def test_mixed_dtypes_are_rejected(dy):
    batch = dy.Batch.from_sizes([4])
    d = torch.zeros((4, 16), device="cuda")
    built = dy.build_tree(d, batch, (1.0,), 0)
    with pytest.raises(ValueError):
        dy.verify(d, d.to(torch.bfloat16), batch, built.tree, (1.0,), (1.0,), 0)
