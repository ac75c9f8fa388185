"""Pins for the oracle's random stream: Philox4x32-10 known answers and an independent
integer re-implementation; uniform conversion."""
import os

import numpy as np

import oracle

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox_py(ctr, key):
    """Philox4x32-10 in Python integers, written from the SC'11 description: per round
    two 32x32->64 products, a word permutation with key injection, Weyl key schedule."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK, p1 & MASK, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK, p0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def test_known_answers(golden_dir):
    rows = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            got = oracle.philox4x32_10(w[0:4], w[4:6])
            assert [int(x) for x in got] == w[6:10]
            assert philox_py(w[0:4], w[4:6]) == w[6:10]
            rows += 1
    assert rows == 3


def test_matches_integer_reimplementation():
    rng = np.random.default_rng(1)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == philox_py(ctr, key)


def test_u01_is_top_24_bits_of_word0():
    seed = 0x0123456789ABCDEF
    for pk_lo, pk_hi, rank, kind in [(0, 0, 0, 1), (7, 0, 3, 2), (0xDEADBEEF, 0x1234, 17, 3)]:
        w = philox_py([pk_lo, pk_hi, rank, kind], [seed & MASK, seed >> 32])
        assert oracle.u01(seed, pk_lo, pk_hi, rank, kind) == (w[0] >> 8) / 2.0**24


def test_u01_uniform():
    u = np.array([oracle.u01(5, i, 0, 0, oracle.KIND_ACCEPT) for i in range(20000)])
    assert 0.0 <= u.min() and u.max() < 1.0
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    chi2 = ((hist - 1250.0) ** 2 / 1250.0).sum()
    assert chi2 < 44.3          # 15 dof, p ~ 1e-4
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03
