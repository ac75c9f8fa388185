"""GPU parity at the five benchmark configurations, in the launch configuration bench.py
times: tree build, one layer of tree attention (sampled rows against the fp64 oracle, which
computes any single row independently) and verification, all through the C ABI."""
import math

import numpy as np
import pytest

import oracle
from helpers import ATTN_TOL, compare_trees, oracle_attention_rows, oracle_trees, verify_in_full

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


@pytest.mark.parametrize("name,layer,rows_per_seq", [
    ("tiny_f32", 0, None),                  # None: every (row, head) pair of the layer
    ("llama2_7b", 31, None),
    ("llama2_13b", 7, None),
    ("llama2_70b", 79, None),
    ("llama2_70b_ragged8", 40, 1024),       # sampled: 3.4 G (row, key) pairs per layer in full
    ("llama2_70b_n32", 3, None),            # supplementary HBM-bound point (prefix split)
])
def test_config(dy, name, layer, rows_per_seq):
    from paper_2410_11744_amd import synth
    cfg = synth.CONFIGS[name]
    print(f"config {name}: nodes={cfg.n_nodes} prefix={cfg.prefix_len}", flush=True)
    dev = torch.device("cuda:0")
    batch = dy.Batch.from_sizes(cfg.n_nodes, cfg.prefix_len)
    draft_h, target_h = synth.make_logits(cfg)
    draft, target = torch.from_numpy(draft_h).to(dev), torch.from_numpy(target_h).to(dev)

    # ---- tree
    built = dy.build_tree(draft, batch, cfg.temps, cfg.seed)
    torch.cuda.synchronize()
    trees = oracle_trees(draft_h, cfg.n_nodes, cfg.temps, cfg.seed)
    full = compare_trees(built, batch, trees)
    assert full == batch.n_seq, "an oracle build decision had a margin below 1e-9"
    print(f"  trees match ({batch.total_nodes} nodes, max depth {max(int(t.depth.max()) for t in trees)})", flush=True)

    # ---- attention, one layer, sampled rows
    q, kp, vp, kt, vt = synth.make_attention_inputs(cfg, layer, device=dev)
    scale = 1.0 / math.sqrt(cfg.head_dim)
    out = dy.tree_attn(q, kp, vp, kt, vt, built.anc_mask, batch, scale)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()
    host = [t.float().cpu().numpy() for t in (q, kp, vp, kt, vt)]
    mask = built.anc_mask.cpu().numpy().view(np.uint64)
    rng = np.random.default_rng(cfg.seed)
    worst = 0.0
    for s, n in enumerate(cfg.n_nodes):
        total = n * cfg.n_q_heads
        pick = np.arange(total) if rows_per_seq is None or total <= rows_per_seq else rng.choice(total, rows_per_seq, replace=False)
        # always include the first and last node (tile edges, deepest mask rows)
        pick = np.unique(np.concatenate([pick, np.arange(cfg.n_q_heads), total - 1 - np.arange(cfg.n_q_heads)]))
        rj, rh = np.divmod(pick, cfg.n_q_heads)
        want = oracle_attention_rows(*host, mask, batch, s, scale, rj, rh)
        a = int(batch.node_offset[s])
        worst = max(worst, float(np.abs(got[a + rj, rh] - want).max()))
    print(f"  attention max abs error {worst:.2e}", flush=True)
    assert worst <= ATTN_TOL[cfg.dtype]

    # ---- verification
    vout, vseed = verify_in_full(lambda sd: dy.verify(draft, target, batch, built.tree, cfg.temps, cfg.temps, sd),
                                 batch, trees, draft_h, target_h, cfg.temps, cfg.temps, cfg.seed)
    print(f"  verify: accepted paths of all {batch.n_seq} sequences match at seed {vseed}, "
          f"accepted {vout.n_accepted.cpu().tolist()}", flush=True)


def test_ceiling_probes_run(dy):
    """The two measurement helpers launch, finish and report plausible work sizes."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    flops = dy.probe_mfma_bf16(10, sink)
    assert flops == 1024 * 8 * 10 * 4 * 2 * 32 * 32 * 16
    buf = torch.ones(1 << 20, dtype=torch.float32, device="cuda")
    assert dy.probe_hbm_read(buf, sink) == 4 << 20
    torch.cuda.synchronize()
    assert float(sink.item()) == 0.0
    with pytest.raises(dy.DyspecError):
        dy.probe_mfma_bf16(0, sink)
    # random operands: same work, results stay finite (the sink is never written)
    assert dy.probe_mfma_bf16(200, sink, random_operands=True) == 1024 * 8 * 200 * 4 * 2 * 32 * 32 * 16
    # the sleeping wave reports both counters and a plausible clock (between 0.3 and 3 GHz)
    counters = torch.zeros(2, dtype=torch.int64, device="cuda")
    khz = dy.probe_clock(200, counters)
    torch.cuda.synchronize()
    cyc, ticks = (int(x) for x in counters.cpu().numpy())
    assert khz > 0 and cyc >= 200 * 64 and ticks > 0
    assert 0.3 < cyc / (ticks / (khz * 1e3)) / 1e9 < 3.0
    assert float(sink.item()) == 0.0
    with pytest.raises(dy.DyspecError):
        dy.probe_clock(0, counters)
