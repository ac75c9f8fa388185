"""Host side of a call: after dyspec_init() and with the interpreter's cyclic collector parked, no
call of a 1000-dispatch loop stalls the host (a process used to show one launch of 35-40 ms around
its 350th dispatch: a full CPython garbage collection walking everything torch holds, triggered
by the ctypes objects the binding creates per call)."""
import gc
import math
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_no_host_stall_over_a_thousand_dispatches():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_11744_amd as dy
    dy.load_library()
    dy.init()
    nodes, prefix, Hq, Hkv, d = (64,), (512,), 8, 2, 128
    batch = dy.Batch.from_sizes(nodes, prefix)
    g = torch.Generator().manual_seed(0)
    mk = lambda *sh: torch.randn(sh, generator=g, dtype=torch.float32).to(torch.bfloat16).cuda()
    q, kp, vp, kt, vt = mk(64, Hq, d), mk(512, Hkv, d), mk(512, Hkv, d), mk(64, Hkv, d), mk(64, Hkv, d)
    mask = torch.zeros((64, 1), dtype=torch.int64, device="cuda")
    mask[:, 0] = torch.tensor([(1 << (j + 1)) - 1 for j in range(63)] + [-1], dtype=torch.int64)   # a chain
    out = torch.empty_like(q)
    scale = 1.0 / math.sqrt(d)
    dy.tree_attn(q, kp, vp, kt, vt, mask, batch, scale, out=out)
    torch.cuda.synchronize()
    gc.collect()
    gc.freeze()
    try:
        host = np.empty(1000)
        for i in range(1000):
            t0 = time.perf_counter()
            dy.tree_attn(q, kp, vp, kt, vt, mask, batch, scale, out=out)
            host[i] = time.perf_counter() - t0
            if i % 200 == 199:
                torch.cuda.synchronize()
    finally:
        gc.unfreeze()
    print(f"host time per call: median {np.median(host) * 1e6:.1f} us, max {host.max() * 1e3:.2f} ms", flush=True)
    assert host.max() < 1e-3           # measured: 0.14 ms at most (the first call after a synchronisation); the old stall was 35 ms
    assert np.median(host) < 2e-4
