"""GPU parity of dyspec_tree_attn_layers (all layers of one step in one call): every layer
against the fp64 oracle on its own tensors, and against the one-layer call."""
import ctypes
import math

import numpy as np
import pytest

from helpers import ATTN_TOL, oracle_attention_rows
from test_gpu_tree_attn import make_case

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    return m


def stacked_case(L, nodes, prefix, Hq, Hkv, d, dtype, seed, shallow=False):
    """L layers over one set of trees: the mask of layer 0's case, fresh tensors per layer."""
    per_layer = [make_case(nodes, prefix, Hq, Hkv, d, dtype, seed + 100 * l, shallow=shallow) for l in range(L)]
    mask = per_layer[0][5]
    stack = [torch.stack([per_layer[l][k] for l in range(L)]) for k in range(5)]
    return stack, mask


def check_layers(dy, out, stack, mask, batch, nodes, Hq, dtype, scale, seed, max_rows=1500):
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()
    rng = np.random.default_rng(seed)
    worst = 0.0
    for l in range(got.shape[0]):
        host = [t[l].float().numpy() for t in stack]
        for s, n in enumerate(nodes):
            total = n * Hq
            pick = np.arange(total) if total <= max_rows else rng.choice(total, max_rows, replace=False)
            rj, rh = np.divmod(pick, Hq)
            want = oracle_attention_rows(*host, mask, batch, s, scale, rj, rh)
            a = int(batch.node_offset[s])
            worst = max(worst, float(np.abs(got[l, a + rj, rh] - want).max()))
    assert worst <= ATTN_TOL[dtype], f"max abs error {worst}"
    return worst


@pytest.mark.parametrize("L,nodes,prefix,Hq,Hkv,d,seed", [
    (3, (70,), (1100,), 4, 4, 128, 1),                     # the one-layer call splits the prefix, the three-layer call less
    (2, (64, 7, 200, 1), (100, 1, 513, 64), 8, 2, 128, 2),  # ragged batch, GQA
    (5, (40,), (64 * 24,), 4, 2, 128, 3),                  # few workgroups per layer: split stays on, per layer
    (4, (300,), (64,), 6, 2, 64, 4),                       # head_dim 64
    (1, (128,), (1024,), 4, 4, 128, 5),                    # a single layer through the stacked call
    (2, (33,), (0,), 4, 2, 128, 6),                        # no prefix
])
def test_bf16_layers_match_oracle_and_single_layer_call(dy, L, nodes, prefix, Hq, Hkv, d, seed):
    print(f"layers case L={L} nodes={nodes} prefix={prefix} H={Hq}/{Hkv} d={d}", flush=True)
    batch = dy.Batch.from_sizes(nodes, prefix)
    stack, mask = stacked_case(L, nodes, prefix, Hq, Hkv, d, "bf16", seed)
    scale = 1.0 / math.sqrt(d)
    dev = [t.cuda() if t.numel() else torch.empty(t.shape, dtype=t.dtype, device="cuda") for t in stack]
    mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
    out = dy.tree_attn_layers(*dev, mask_dev, batch, scale)
    torch.cuda.synchronize()
    check_layers(dy, out, stack, mask, batch, nodes, Hq, "bf16", scale, seed)
    # the one-layer call on each layer: same products; the prefix may be split differently,
    # which moves one fp32 combine and a bf16 rounding point
    for l in range(L):
        one = dy.tree_attn(*[t[l] for t in dev], mask_dev, batch, scale)
        assert float((one.float() - out[l].float()).abs().max()) <= 2.0 ** -6
    # without a workspace no prefix is split: bit-identical to the unsplit one-layer call
    whole = dy.tree_attn_layers(*dev, mask_dev, batch, scale, use_workspace=False)
    for l in range(L):
        one = dy.tree_attn(*[t[l] for t in dev], mask_dev, batch, scale, use_workspace=False)
        assert torch.equal(one, whole[l])


def test_strided_layer_dimension(dy):
    """Layers taken as every second plane of a larger stack (layer stride twice the dense one)."""
    nodes, prefix, Hq, Hkv, d = (90,), (200,), 8, 2, 128
    batch = dy.Batch.from_sizes(nodes, prefix)
    stack, mask = stacked_case(6, nodes, prefix, Hq, Hkv, d, "bf16", 9)
    dev = [t.cuda() for t in stack]
    mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
    scale = 1.0 / math.sqrt(d)
    out_full = torch.zeros_like(dev[0])
    views = [t[::2] for t in dev]
    dy.tree_attn_layers(*views, mask_dev, batch, scale, out=out_full[::2])
    torch.cuda.synchronize()
    check_layers(dy, out_full[::2], [t[::2] for t in stack], mask, batch, nodes, Hq, "bf16", scale, 9)
    assert float(out_full[1::2].float().abs().max()) == 0.0          # the planes in between are untouched


def test_fp32_layers_loop(dy):
    nodes, prefix, Hq, Hkv, d = (32,), (128,), 8, 8, 64
    batch = dy.Batch.from_sizes(nodes, prefix)
    stack, mask = stacked_case(3, nodes, prefix, Hq, Hkv, d, "f32", 11)
    dev = [t.cuda() for t in stack]
    mask_dev = torch.from_numpy(mask.view(np.int64)).cuda()
    scale = 1.0 / math.sqrt(d)
    out = dy.tree_attn_layers(*dev, mask_dev, batch, scale)
    torch.cuda.synchronize()
    check_layers(dy, out, stack, mask, batch, nodes, Hq, "f32", scale, 11)
    for l in range(3):
        assert torch.equal(out[l], dy.tree_attn(*[t[l] for t in dev], mask_dev, batch, scale))


def test_layers_bad_arguments(dy):
    nodes, prefix = (8,), (16,)
    batch = dy.Batch.from_sizes(nodes, prefix)
    lib = dy.load_library()
    cb = batch._c()
    t = torch.zeros((2, 8, 4, 128), dtype=torch.bfloat16, device="cuda")
    kp = torch.zeros((2, 16, 4, 128), dtype=torch.bfloat16, device="cuda")
    m = torch.zeros((8, 1), dtype=torch.int64, device="cuda")
    call = lambda L, qs: lib.dyspec_tree_attn_layers(
        t.data_ptr(), kp.data_ptr(), kp.data_ptr(), t.data_ptr(), t.data_ptr(), m.data_ptr(), ctypes.byref(cb),
        L, qs, kp.stride(0), t.stride(0), 4, 4, 128, 1, ctypes.c_float(0.1), t.data_ptr(), None, 0, None)
    assert call(0, t.stride(0)) == -2           # no layers
    assert call(2, -1) == -1                    # negative stride
    assert call(2, 4) == -1                     # layers would lose their 16-byte alignment
    assert lib.dyspec_tree_attn_layers_workspace_bytes(ctypes.byref(cb), 0, 4, 4, 128) == 0


@pytest.mark.parametrize("name,L", [("llama2_70b", 3), ("llama2_70b_n32", 3), ("llama2_7b", 4), ("llama2_70b_ragged8", 2)])
def test_full_size_configs_through_the_stacked_call(dy, name, L):
    """Benchmark shapes, the tree the builder makes for them, a few stacked layers: sampled rows of
    every layer against the fp64 oracle (the N = 32 shape splits its prefix inside the stacked call)."""
    from paper_2410_11744_amd import synth
    cfg = synth.CONFIGS[name]
    print(f"stacked full size {name} L={L}", flush=True)
    batch = dy.Batch.from_sizes(cfg.n_nodes, cfg.prefix_len)
    draft, _ = synth.make_logits(cfg)
    built = dy.build_tree(torch.from_numpy(draft).cuda(), batch, cfg.temps, cfg.seed)
    per_layer = [synth.make_attention_inputs(cfg, l, device="cuda") for l in range(L)]
    dev = [torch.stack([per_layer[l][k] for l in range(L)]) for k in range(5)]
    del per_layer
    scale = 1.0 / math.sqrt(cfg.head_dim)
    out = dy.tree_attn_layers(*dev, built.anc_mask, batch, scale)
    torch.cuda.synchronize()
    mask = built.anc_mask.cpu().numpy().view(np.uint64)
    stack = [t.cpu() for t in dev]
    nodes = [int(batch.node_offset[s + 1] - batch.node_offset[s]) for s in range(batch.n_seq)]
    check_layers(dy, out, stack, mask, batch, nodes, cfg.n_q_heads, "bf16", scale, 5, max_rows=96)
    one = dy.tree_attn(*[t[L - 1] for t in dev], built.anc_mask, batch, scale)
    assert float((one.float() - out[L - 1].float()).abs().max()) <= 2.0 ** -6
