"""The step's calls under HIP graph capture: a serving loop may record its layers' dyspec_tree_attn
calls (split and unsplit walks, the static-scratch entry point) and dyspec_verify once and replay
them.  The library allocates nothing, clears nothing and waits for nothing inside those calls (the
arrival counters of a split are reset by the kernel itself), so a capture holds kernel launches
only.  Every replay is compared bit for bit with the eager result, several times, with eager calls
of the same entry points and other work of the process between the replays."""
import math

import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dy():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as m
    m.load_library()
    m.init()                      # code loading and kernel attributes before anything is captured
    return m


def test_replays_of_a_captured_step_equal_the_eager_step(dy):
    dev = torch.device("cuda:0")
    # shapes: a split walk (8 groups x parts), an unsplit one (no prefix worth splitting) and verification
    nodes, prefix, Hq, Hkv, d, V = (96, 40), (1024, 640), 8, 8, 128, 4000
    batch = dy.Batch.from_sizes(nodes, prefix)
    g = torch.Generator().manual_seed(7)
    N, P = sum(nodes), sum(prefix)
    draft = (2.0 * torch.randn((N, V), generator=g)).to(dev)
    target = (draft.cpu() + 1.0 * torch.randn((N, V), generator=g)).to(dev)
    temps = (0.8, 1.1)
    built = dy.build_tree(draft, batch, temps, 5)
    mk = lambda *sh: torch.randn(sh, generator=g, dtype=torch.float32).to(torch.bfloat16).to(dev)
    layers = [(mk(N, Hq, d), mk(P, Hkv, d), mk(P, Hkv, d), mk(N, Hkv, d), mk(N, Hkv, d)) for _ in range(3)]
    scale = 1.0 / math.sqrt(d)
    import ctypes
    assert dy.load_library().dyspec_workspace_bytes(1, ctypes.byref(batch._c()), 0, Hq, Hkv, d) > 0, "meant to be split"
    unsplit_batch = dy.Batch.from_sizes(nodes, (0, 0))
    empty = torch.empty((0, Hkv, d), dtype=torch.bfloat16, device=dev)

    # ---- eager results
    eager_outs = [dy.tree_attn(*layers[l], built.anc_mask, batch, scale) for l in range(3)]
    eager_unsplit = dy.tree_attn(layers[0][0], empty, empty, layers[0][3], layers[0][4], built.anc_mask, unsplit_batch, scale)
    eager_static = torch.empty_like(layers[1][0])
    dy.tree_attn(*layers[1], built.anc_mask, batch, scale, out=eager_static, static_scratch=True)
    eager_v = dy.VerifyOutput.empty(batch, dev)
    eager_v.row_stats.zero_(); eager_v.accept_ratio.zero_()
    eager_v.accepted_nodes.fill_(-7); eager_v.n_accepted.fill_(-7); eager_v.final_token.fill_(-7)
    dy.verify(draft, target, batch, built.tree, temps, temps, 11, out=eager_v)
    torch.cuda.synchronize()
    assert torch.equal(eager_static.view(torch.int16), eager_outs[1].view(torch.int16))

    # ---- capture on a side stream: prepared calls on that stream, outputs of their own
    s = torch.cuda.Stream()
    outs = [torch.empty_like(layers[l][0]) for l in range(3)]
    out_unsplit, out_static = torch.empty_like(layers[0][0]), torch.empty_like(layers[1][0])
    vout = dy.VerifyOutput.empty(batch, dev)
    with torch.cuda.stream(s):
        calls = [dy.tree_attn_call(*layers[l], built.anc_mask, batch, scale, out=outs[l], stream=s) for l in range(3)]
        calls.append(dy.tree_attn_call(layers[0][0], empty, empty, layers[0][3], layers[0][4], built.anc_mask, unsplit_batch, scale,
                                       out=out_unsplit, stream=s))
        calls.append(dy.tree_attn_call(*layers[1], built.anc_mask, batch, scale, out=out_static, stream=s, static_scratch=True))
        calls.append(dy.verify_call(draft, target, batch, built.tree, temps, temps, 11, out=vout, stream=s))
        for c in calls:                                         # once eagerly on this stream (workspace exists, code is loaded)
            c()
        s.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        for c in calls:
            c()

    def check(tag):
        for l in range(3):
            assert torch.equal(outs[l].view(torch.int16), eager_outs[l].view(torch.int16)), f"{tag}: layer {l}"
        assert torch.equal(out_unsplit.view(torch.int16), eager_unsplit.view(torch.int16)), f"{tag}: unsplit walk"
        assert torch.equal(out_static.view(torch.int16), eager_outs[1].view(torch.int16)), f"{tag}: static scratch"
        for name in ("accepted_nodes", "n_accepted", "final_token"):
            assert torch.equal(getattr(vout, name), getattr(eager_v, name)), f"{tag}: {name}"
        assert torch.equal(vout.row_stats.view(torch.int32), eager_v.row_stats.view(torch.int32)), f"{tag}: row_stats"
        assert torch.equal(vout.accept_ratio.view(torch.int32), eager_v.accept_ratio.view(torch.int32)), f"{tag}: accept_ratio"

    for rep in range(4):
        for t in outs + [out_unsplit, out_static, vout.row_stats, vout.accept_ratio]:
            t.zero_()
        vout.accepted_nodes.fill_(-7); vout.n_accepted.fill_(-7); vout.final_token.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check(f"replay {rep}")
        # the process's own eager work between replays: the same entry points with other arguments, a reduction
        other = dy.tree_attn(*layers[(rep + 1) % 3], built.anc_mask, batch, scale)
        dy.verify(draft, target, batch, built.tree, temps, temps, 100 + rep)
        assert torch.isfinite(other.float().sum()).item()
        torch.cuda.synchronize()
