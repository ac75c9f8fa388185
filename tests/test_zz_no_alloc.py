"""dyspec_tree_attn_static_scratch (the entry point for callers that cannot allocate: partial
results of a split prefix go to the library's static device array) against dyspec_tree_attn with
a caller workspace, through the C ABI: same kernels, same split, so the outputs are equal bit
for bit; and both within the attention tolerance of the fp64 oracle.  Two calls in a row, the
second on a smaller input, so that whatever the first call left in the array is there when the
second runs."""
import math

import numpy as np
import pytest

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


def chain_and_branches_mask(n, rng):
    """Ancestor mask of a random tree (parent of node i uniform among the earlier nodes)."""
    words = (n + 63) // 64
    m = np.zeros((n, words), np.uint64)
    par = [-1] + [int(rng.integers(0, i)) for i in range(1, n)]
    for j in range(n):
        a = j
        while a >= 0:
            m[j, a // 64] |= np.uint64(1) << np.uint64(a % 64)
            a = par[a]
    return m


def one_case(dy, nodes, prefix, Hq, Hkv, d, seed):
    import ctypes
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed)
    batch = dy.Batch.from_sizes(nodes, prefix)
    g = torch.Generator().manual_seed(seed)
    mk = lambda *sh: torch.randn(sh, generator=g, dtype=torch.float32).to(torch.bfloat16)
    N, P = sum(nodes), sum(prefix)
    host = [mk(N, Hq, d), mk(P, Hkv, d), mk(P, Hkv, d), mk(N, Hkv, d), mk(N, Hkv, d)]
    words = batch.mask_words
    mask = np.zeros((N, words), np.uint64)
    off = 0
    for n in nodes:
        m = chain_and_branches_mask(n, rng)
        mask[off:off + n, :m.shape[1]] = m
        off += n
    q, kp, vp, kt, vt = [t.to(dev) for t in host]
    mask_d = torch.from_numpy(mask.view(np.int64)).to(dev)
    scale = 1.0 / math.sqrt(d)
    lib = dy.load_library()
    need = lib.dyspec_workspace_bytes(1, ctypes.byref(batch._c()), 0, Hq, Hkv, d)
    assert need > 0, "the case must split its prefix, or no scratch memory is involved"
    want = dy.tree_attn(q, kp, vp, kt, vt, mask_d, batch, scale)
    got = torch.full_like(q, float("nan"))
    dy.tree_attn(q, kp, vp, kt, vt, mask_d, batch, scale, out=got, static_scratch=True)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    hf = [t.float().numpy() for t in host]
    g32 = got.float().cpu().numpy()
    for s, n in enumerate(nodes):
        pick = rng.choice(n * Hq, min(n * Hq, 400), replace=False)
        rj, rh = np.divmod(pick, Hq)
        ref = oracle_attention_rows(*hf, mask, batch, s, scale, rj, rh)
        a = int(batch.node_offset[s])
        assert float(np.abs(g32[a + rj, rh] - ref).max()) <= ATTN_TOL["bf16"]


def test_static_scratch_matches_workspace_call_twice_in_a_row(dy):
    print("static scratch: 70B-shaped narrow tree, then a smaller ragged batch", flush=True)
    one_case(dy, (32,), (4096,), 64, 8, 128, 1)            # 8-way split
    one_case(dy, (20, 7), (2100, 1500), 64, 8, 128, 2)     # smaller, ragged, fewer splits
    one_case(dy, (32,), (4096,), 64, 8, 128, 3)            # and the larger one again


def test_static_scratch_refuses_what_does_not_fit(dy):
    import ctypes
    batch = dy.Batch.from_sizes((128,), (4096,))           # 256 workgroups x 34 KB of parts > 8 MiB
    lib = dy.load_library()
    assert lib.dyspec_workspace_bytes(1, ctypes.byref(batch._c()), 0, 32, 32, 128) > (8 << 20)
    z = torch.zeros((128, 32, 128), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((4096, 32, 128), dtype=torch.bfloat16, device="cuda")
    m = torch.zeros((128, 2), dtype=torch.int64, device="cuda")
    with pytest.raises(dy.DyspecError) as e:
        dy.tree_attn(z, kv, kv, z, z, m, batch, 0.1, out=torch.empty_like(z), static_scratch=True)
    assert e.value.status == -4
