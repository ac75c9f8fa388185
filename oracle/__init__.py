"""CPU oracle for the DySpec hot path -- TEST INFRASTRUCTURE ONLY.

numpy-facing wrappers over ``dyspec_oracle.c`` (plain C, fp64).  Only ``tests/``, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package; the GPU
library never does, and the two share no code.

Each wrapper names the passage of the paper (arXiv 2410.11744) it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dyspec_oracle.c")
_LIB = os.path.join(_HERE, "libdyspec_oracle.so")

KIND_PATH, KIND_BUILD, KIND_ACCEPT, KIND_RESID = 0, 1, 2, 3


def compile_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP only spreads independent attention rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(compile_oracle())
        _lib.oracle_u01.restype = ctypes.c_double
        _lib.oracle_u01.argtypes = [ctypes.c_uint64] + [ctypes.c_uint32] * 4
    return _lib


def num_threads() -> int:
    """Threads the attention routines use (OpenMP over independent rows)."""
    return int(_L().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for the attention routines from now on (timing only; results do not depend on it)."""
    _L().oracle_set_num_threads(ctypes.c_int(int(n)))


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def philox4x32_10(ctr, key) -> np.ndarray:
    """Philox4x32-10 block function (Salmon et al., SC'11): 4 counter words, 2 key words."""
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    _L().oracle_philox4x32_10(_p(c, ctypes.c_uint32), _p(k, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def u01(seed: int, pk_lo: int, pk_hi: int, rank: int, kind: int) -> float:
    return float(_L().oracle_u01(seed, pk_lo, pk_hi, rank, kind))


def softmax(logits, temp: float) -> np.ndarray:
    """softmax(logits / temp) of one row in fp64."""
    x = _f32(logits)
    out = np.zeros(x.shape[0], dtype=np.float64)
    _L().oracle_softmax(_p(x, ctypes.c_float), ctypes.c_int(x.shape[0]), ctypes.c_double(temp),
                        _p(out, ctypes.c_double))
    return out


def softmax_stats(draft_logits, target_logits, temp_d: float, temp_t: float) -> np.ndarray:
    """[n_rows,4] = (max_d, sumexp_d, max_t, sumexp_t) of logits/temp per row."""
    d, t = _f32(draft_logits), _f32(target_logits)
    n, V = d.shape
    out = np.zeros((n, 4), dtype=np.float64)
    _L().oracle_softmax_stats(_p(d, ctypes.c_float), _p(t, ctypes.c_float), ctypes.c_int(n),
                              ctypes.c_int(V), ctypes.c_double(temp_d), ctypes.c_double(temp_t),
                              _p(out, ctypes.c_double))
    return out


@dataclass
class Tree:
    """Token tree in creation order; row 0 is the root (the prefix's last token)."""
    parent: np.ndarray
    token: np.ndarray
    sib_rank: np.ndarray
    first_child: np.ndarray
    next_sibling: np.ndarray
    depth: np.ndarray
    est_value: np.ndarray      # fp64
    mask: np.ndarray           # [N, words] uint64
    n_built: int
    margin_pop: np.ndarray     # per created node, relative margin of the arg-max
    margin_cdf: np.ndarray     # per created node, relative margin of the token draw


def _tree_buffers(N):
    words = (N + 63) // 64
    i = lambda: np.zeros(N, dtype=np.int32)
    return (i(), i(), i(), i(), i(), i(), np.zeros(N, dtype=np.float64),
            np.zeros((N, words), dtype=np.uint64), ctypes.c_int32(0),
            np.zeros(N, dtype=np.float64), np.zeros(N, dtype=np.float64), words)


def build_tree(draft_logits, n_budget: int, temp: float, seed: int, seq: int = 0) -> Tree:
    """Greedy fixed-budget construction (Algorithm 1); n_budget counts the root."""
    d = _f32(draft_logits)
    assert d.shape[0] >= n_budget
    V = d.shape[1]
    par, tok, rk, fc, ns, dep, ev, mask, nb, mp, mc, words = _tree_buffers(n_budget)
    I, D = ctypes.c_int32, ctypes.c_double
    _L().oracle_build_tree(_p(d, ctypes.c_float), ctypes.c_int(V), ctypes.c_int(n_budget),
                           D(temp), ctypes.c_uint64(seed), ctypes.c_uint32(seq),
                           _p(par, I), _p(tok, I), _p(rk, I), _p(fc, I), _p(ns, I), _p(dep, I),
                           _p(ev, D), _p(mask, ctypes.c_uint64), ctypes.c_int(words),
                           ctypes.byref(nb), _p(mp, D), _p(mc, D))
    return Tree(par, tok, rk, fc, ns, dep, ev, mask, nb.value, mp, mc)


def build_tree_explicit(draft_logits, n_budget: int, temp: float, u_build) -> Tree:
    """Algorithm 1 with the uniform of the expansion that creates node i given as u_build[i]."""
    d = _f32(draft_logits)
    V = d.shape[1]
    u = np.ascontiguousarray(u_build, dtype=np.float64)
    assert u.shape[0] >= n_budget
    par, tok, rk, fc, ns, dep, ev, mask, nb, mp, mc, words = _tree_buffers(n_budget)
    I, D = ctypes.c_int32, ctypes.c_double
    _L().oracle_build_tree_explicit(_p(d, ctypes.c_float), ctypes.c_int(V), ctypes.c_int(n_budget),
                                    D(temp), _p(u, D),
                                    _p(par, I), _p(tok, I), _p(rk, I), _p(fc, I), _p(ns, I),
                                    _p(dep, I), _p(ev, D), _p(mask, ctypes.c_uint64),
                                    ctypes.c_int(words), ctypes.byref(nb), _p(mp, D), _p(mc, D))
    return Tree(par, tok, rk, fc, ns, dep, ev, mask, nb.value, mp, mc)


def ancestor_mask(parent) -> np.ndarray:
    """Bit i of row j set iff i is an ancestor of j or i == j (Section 2, tree attention)."""
    par = _i32(parent)
    N = par.shape[0]
    words = (N + 63) // 64
    mask = np.zeros((N, words), dtype=np.uint64)
    _L().oracle_ancestor_mask(_p(par, ctypes.c_int32), ctypes.c_int(N), _p(mask, ctypes.c_uint64),
                              ctypes.c_int(words))
    return mask


def links_from_parent(parent):
    """first_child / next_sibling (children in index order) and depth from a parent array."""
    par = np.asarray(parent, dtype=np.int32)
    N = par.shape[0]
    fc = np.full(N, -1, np.int32)
    ns = np.full(N, -1, np.int32)
    last = np.full(N, -1, np.int32)
    dep = np.zeros(N, np.int32)
    for i in range(1, N):
        p = par[i]
        if p < 0:
            continue
        dep[i] = dep[p] + 1
        if last[p] < 0:
            fc[p] = i
        else:
            ns[last[p]] = i
        last[p] = i
    return fc, ns, dep


def dfs_order(parent, first_child, next_sibling) -> np.ndarray:
    """Depth-first (pre-order) visiting order of a token tree, children in sampling order
    (Appendix "Block-Sparsity Friendly Token Order"): order[new] = old node index.  Rows that
    were never attached to the tree (parent -1, not the root) follow the tree, in index order."""
    par, fc, ns = (np.asarray(a, dtype=np.int64) for a in (parent, first_child, next_sibling))
    N = par.shape[0]
    order = []
    stack = [0]
    while stack:
        node = stack.pop()
        order.append(node)
        kids = []
        c = fc[node]
        while c >= 0:
            kids.append(int(c))
            c = ns[c]
        stack.extend(reversed(kids))                 # first-sampled child is visited first
    seen = set(order)
    order.extend(i for i in range(N) if i not in seen)
    return np.asarray(order, dtype=np.int32)


def relabel_tree(order, parent, token, sib_rank, first_child, next_sibling, depth):
    """The same tree with node order[new] renamed to new.  Returns the six arrays and the
    ancestor mask of the renamed tree (rows outside the tree keep only their own bit)."""
    order = np.asarray(order, dtype=np.int64)
    N = order.shape[0]
    rank = np.empty(N, dtype=np.int64)
    rank[order] = np.arange(N)
    ren = lambda a: np.where(np.asarray(a)[order] >= 0, rank[np.maximum(np.asarray(a)[order], 0)], -1).astype(np.int32)
    keep = lambda a: np.asarray(a)[order].astype(np.int32)
    par_n = ren(parent)
    words = (N + 63) // 64
    mask = np.zeros((N, words), dtype=np.uint64)
    for j in range(N):
        a = j
        while a >= 0:
            mask[j, a // 64] |= np.uint64(1) << np.uint64(a % 64)
            a = int(par_n[a])
    return par_n, keep(token), keep(sib_rank), ren(first_child), ren(next_sibling), keep(depth), mask


def mask_block_count(mask, n: int, block: int = 32) -> int:
    """Number of block x block tiles of the n x n ancestor mask that hold at least one set bit."""
    m = np.asarray(mask, dtype=np.uint64)
    bits = ((m[:n, :, None] >> np.arange(64, dtype=np.uint64)[None, None, :]) & np.uint64(1)).astype(bool)
    dense = bits.reshape(n, -1)[:, :n]
    nb = (n + block - 1) // block
    pad = np.zeros((nb * block, nb * block), dtype=bool)
    pad[:n, :n] = dense
    return int(pad.reshape(nb, block, nb, block).any(axis=(1, 3)).sum())


def tree_attn(q, k_prefix, v_prefix, k_tree, v_tree, mask, scale: float) -> np.ndarray:
    """Tree-masked attention, plain definition in fp64.  q [N,Hq,d]; k/v_prefix [P,Hkv,d];
    k/v_tree [N,Hkv,d]; mask [N,words] uint64.  Returns [N,Hq,d] fp64."""
    q, kp, vp, kt, vt = map(_f32, (q, k_prefix, v_prefix, k_tree, v_tree))
    N, Hq, d = q.shape
    P, Hkv = kp.shape[0], kp.shape[1]
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    out = np.zeros((N, Hq, d), dtype=np.float64)
    F = ctypes.c_float
    _L().oracle_tree_attn(_p(q, F), _p(kp, F), _p(vp, F), _p(kt, F), _p(vt, F),
                          _p(mask, ctypes.c_uint64), ctypes.c_int(mask.shape[1]),
                          ctypes.c_int(N), ctypes.c_int(P), ctypes.c_int(Hq), ctypes.c_int(Hkv),
                          ctypes.c_int(d), ctypes.c_double(scale), _p(out, ctypes.c_double))
    return out


def tree_attn_rows(q, k_prefix, v_prefix, k_tree, v_tree, mask, scale: float, rows_j, rows_h):
    """As tree_attn but only for the sampled (node, head) rows; returns [n_rows, d] fp64."""
    q, kp, vp, kt, vt = map(_f32, (q, k_prefix, v_prefix, k_tree, v_tree))
    N, Hq, d = q.shape
    P, Hkv = kp.shape[0], kp.shape[1]
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    rj, rh = _i32(rows_j), _i32(rows_h)
    out = np.zeros((rj.shape[0], d), dtype=np.float64)
    F = ctypes.c_float
    _L().oracle_tree_attn_rows(_p(q, F), _p(kp, F), _p(vp, F), _p(kt, F), _p(vt, F),
                               _p(mask, ctypes.c_uint64), ctypes.c_int(mask.shape[1]),
                               ctypes.c_int(N), ctypes.c_int(P), ctypes.c_int(Hq),
                               ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_double(scale),
                               ctypes.c_int(rj.shape[0]), _p(rj, ctypes.c_int32),
                               _p(rh, ctypes.c_int32), _p(out, ctypes.c_double))
    return out


@dataclass
class VerifyResult:
    accepted_nodes: np.ndarray   # accepted node indices in order, root excluded
    final_token: int             # token sampled when the walk stops (-1 if none)
    stop_node: int
    tested_margin: np.ndarray    # |c - R[y]/D[y]| per tested node, +inf elsewhere
    resid_margin: float          # inverse-CDF margin of the final sample

    @property
    def n_accepted(self):
        return int(self.accepted_nodes.shape[0])

    @property
    def min_accept_margin(self):
        return float(np.min(self.tested_margin)) if self.tested_margin.size else float("inf")


def _verify_common(fn, draft_logits, target_logits, token, first_child, next_sibling,
                   temp_d, temp_t, emit_bonus, extra):
    d, t = _f32(draft_logits), _f32(target_logits)
    tok, fc, ns = _i32(token), _i32(first_child), _i32(next_sibling)
    N, V = tok.shape[0], d.shape[1]
    assert d.shape[0] >= N and t.shape[0] >= N and t.shape[1] == V
    acc = np.zeros(N, dtype=np.int32)
    na, fin, stop = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    tm = np.zeros(N, dtype=np.float64)
    rm = ctypes.c_double(0)
    I, D, F = ctypes.c_int32, ctypes.c_double, ctypes.c_float
    fn(_p(d, F), _p(t, F), ctypes.c_int(V), ctypes.c_int(N), _p(tok, I), _p(fc, I), _p(ns, I),
       D(temp_d), D(temp_t), ctypes.c_int(int(emit_bonus)), *extra,
       _p(acc, I), ctypes.byref(na), ctypes.byref(fin), ctypes.byref(stop), _p(tm, D),
       ctypes.byref(rm))
    return VerifyResult(acc[:na.value].copy(), fin.value, stop.value, tm, rm.value)


def verify(draft_logits, target_logits, token, first_child, next_sibling, temp_d, temp_t,
           seed: int, seq: int = 0, emit_bonus: bool = True) -> VerifyResult:
    """Tree verification (Algorithm 3) with Philox draws named by the sibling-rank path."""
    return _verify_common(_L().oracle_verify, draft_logits, target_logits, token, first_child,
                          next_sibling, temp_d, temp_t, emit_bonus,
                          (ctypes.c_uint64(seed), ctypes.c_uint32(seq)))


def verify_explicit(draft_logits, target_logits, token, first_child, next_sibling, temp_d,
                    temp_t, u_accept, u_resid, emit_bonus: bool = True) -> VerifyResult:
    """Algorithm 3 with the accept draw of node i = u_accept[i] and the final-sample draw
    taken at node i = u_resid[i]."""
    ua = np.ascontiguousarray(u_accept, dtype=np.float64)
    ur = np.ascontiguousarray(u_resid, dtype=np.float64)
    return _verify_common(_L().oracle_verify_explicit, draft_logits, target_logits, token,
                          first_child, next_sibling, temp_d, temp_t, emit_bonus,
                          (_p(ua, ctypes.c_double), _p(ur, ctypes.c_double)))


def accept_ratio_all(draft_logits, target_logits, token, first_child, next_sibling,
                     temp_d, temp_t) -> np.ndarray:
    """R_k[y]/D_k[y] seen by every node when it is tested (inner loop of Algorithm 3)."""
    d, t = _f32(draft_logits), _f32(target_logits)
    tok, fc, ns = _i32(token), _i32(first_child), _i32(next_sibling)
    N, V = tok.shape[0], d.shape[1]
    out = np.zeros(N, dtype=np.float64)
    I, D, F = ctypes.c_int32, ctypes.c_double, ctypes.c_float
    _L().oracle_accept_ratio_all(_p(d, F), _p(t, F), ctypes.c_int(V), ctypes.c_int(N), _p(tok, I),
                                 _p(fc, I), _p(ns, I), D(temp_d), D(temp_t), _p(out, D))
    return out


def monte_carlo(draft_logits, target_logits, n_budget, temp_d, temp_t, seed0, n_trials):
    """n_trials seeded build+verify steps on fixed logit tables; returns counts of the first
    emitted token [V], of the first two emitted tokens [V,V], and the mean accepted count."""
    d, t = _f32(draft_logits), _f32(target_logits)
    V = d.shape[1]
    c1 = np.zeros(V, dtype=np.int64)
    c2 = np.zeros((V, V), dtype=np.int64)
    tot = ctypes.c_int64(0)
    _L().oracle_monte_carlo(_p(d, ctypes.c_float), _p(t, ctypes.c_float), ctypes.c_int(V),
                            ctypes.c_int(n_budget), ctypes.c_double(temp_d),
                            ctypes.c_double(temp_t), ctypes.c_uint64(seed0),
                            ctypes.c_int64(n_trials), _p(c1, ctypes.c_int64),
                            _p(c2, ctypes.c_int64), ctypes.byref(tot))
    return c1, c2, tot.value / float(n_trials)


from .threshold import ThresholdTree, threshold_tree  # noqa: E402  (Algorithm 2; needs the definitions above)
