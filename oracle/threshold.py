"""DySpec CPU oracle, token tree construction with a threshold -- TEST INFRASTRUCTURE ONLY.

Algorithm 2 (Section 4.4, Appendix A.2) in plain numpy fp64: the tree grows level by level;
every node of the current level keeps drawing children from its own draft distribution,
without replacement, while the estimated value of its next draw stays at or above the
threshold t.

Readings (the listing is garbled in places):
  * the inner loop's condition is printed with the opposite sign; the text says nodes are extended while
    their estimated value is ABOVE the threshold, so the loop runs while the value is >= t;
  * the paper relaxes the node budget but still states a maximum tree size in its
    experiments (Appendix B): nodes are numbered in creation order (level by level, the level's
    nodes in order, children in sampling order) and construction stops when `max_nodes` rows,
    the root included, exist;
  * a draw that finds nothing left in the node's distribution ends that node's loop;
  * est_value of a node is the value its draw was made at, as for Algorithm 1.

Draws are the path-named Philox uniforms of the rest of the oracle (kind BUILD, rank = number
of children the parent already has), so a node reached by the same path of sibling ranks gets
the same uniform under Algorithm 1 and Algorithm 2.

Pins (tests/test_oracle_threshold.py): with t = the smallest estimated value Algorithm 1
opened, the same set of paths, tokens and values as Algorithm 1 (Appendix A.1's last
paragraph); the closed form of every value (Appendix D); every created node has value >= t
and every unopened slot < t; one level and V = 2 by hand.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional, Sequence, Tuple

import numpy as np

from . import KIND_BUILD, KIND_PATH, philox4x32_10, softmax, u01


def _child_key(seed: int, pk: Tuple[int, int], rank: int) -> Tuple[int, int]:
    w = philox4x32_10([pk[0], pk[1], rank, KIND_PATH], [seed & 0xFFFFFFFF, seed >> 32])
    return int(w[0]), int(w[1])


def _sample(d: np.ndarray, u: float):
    """Smallest y with sum_{x<=y} d[x] > u * sum(d), zero entries never chosen; also the
    distance of u * W to the nearest edge of y's interval over W."""
    W = float(d.sum())
    if not W > 0.0:
        return -1, 0.0, 0.0
    target = u * W
    cum = np.cumsum(d)
    above = np.nonzero((cum > target) & (d > 0.0))[0]
    if above.size == 0:                                  # rounding at the very top edge
        y = int(np.nonzero(d > 0.0)[0][-1])
        return y, W, 0.0
    y = int(above[0])
    lo = float(cum[y] - d[y])
    return y, W, min(target - lo, float(cum[y]) - target) / W


@dataclass
class ThresholdTree:
    parent: np.ndarray
    token: np.ndarray
    sib_rank: np.ndarray
    first_child: np.ndarray
    next_sibling: np.ndarray
    depth: np.ndarray
    est_value: np.ndarray      # fp64: value the node's draw was made at
    child_value: np.ndarray    # fp64: value of the node's own first draw (v * d[y])
    mask: np.ndarray           # [max_nodes, words] uint64
    n_built: int
    paths: list                # sibling-rank path of every node, root = ()
    margin_cdf: float          # smallest inverse-CDF margin of any draw
    margin_threshold: float    # smallest |v - t| / t over all loop tests
    n_levels: int


def threshold_tree(draft_logits, max_nodes: int, temp: float, t: float, seed: int, seq: int = 0,
                   row_of: Optional[Callable[[Tuple[int, ...], int], int]] = None) -> ThresholdTree:
    """Algorithm 2.  Row of draft_logits read by a node: row_of(path, index), default the
    node's own index (creation order)."""
    logits = np.asarray(draft_logits, dtype=np.float32)
    N = int(max_nodes)
    words = (N + 63) // 64
    parent = np.full(N, -1, np.int32)
    token = np.full(N, -1, np.int32)
    sib_rank = np.zeros(N, np.int32)
    first_child = np.full(N, -1, np.int32)
    next_sibling = np.full(N, -1, np.int32)
    depth = np.zeros(N, np.int32)
    est_value = np.zeros(N, np.float64)
    child_value = np.zeros(N, np.float64)
    mask = np.zeros((N, words), np.uint64)
    for i in range(N):
        mask[i, i // 64] = np.uint64(1) << np.uint64(i % 64)
    est_value[0] = 1.0
    child_value[0] = 1.0
    paths = [()]
    keys = [(int(seq), 0)]
    m_cdf, m_thr = float("inf"), float("inf")

    # The tree is held as flat arrays in creation order; a level is the run of rows the
    # previous level created, so "the nodes to expand next" is just a list of row indices.
    n = 1
    level = [0]
    levels = 0

    def append_child(node: int, y: int, rank: int, prev: int, drawn_at: float, own: float) -> int:
        """Row n becomes the child of `node` with token y; returns its index."""
        nonlocal n
        i = n
        n += 1
        parent[i], token[i], sib_rank[i], depth[i] = node, y, rank, depth[node] + 1
        if prev < 0:
            first_child[node] = i
        else:
            next_sibling[prev] = i
        mask[i] |= mask[node]
        est_value[i] = drawn_at                 # the value at which this draw was made
        child_value[i] = own                    # what the child's own first draw will be worth
        paths.append(paths[node] + (rank,))
        keys.append(_child_key(seed, keys[node], rank))
        return i

    while level and n < N:
        created = []
        levels += 1
        for node in level:
            if n >= N:                          # capacity cut: later nodes of the level get nothing
                break
            v = float(child_value[node])
            m_thr = min(m_thr, abs(v - t) / t)
            if not v >= t:                      # below the threshold: this node is never expanded
                continue
            row = node if row_of is None else row_of(paths[node], node)
            d = softmax(logits[row], temp)      # the node's draft distribution over next tokens
            rank, prev = 0, -1
            while v >= t and n < N:
                u = u01(seed, keys[node][0], keys[node][1], rank, KIND_BUILD)
                y, W, margin = _sample(d, u)    # a token from what is left of the distribution
                if y < 0:                       # nothing left to draw
                    break
                m_cdf = min(m_cdf, margin)
                dy = float(d[y]) / W
                prev = append_child(node, y, rank, prev, v, v * dy)
                created.append(prev)
                # the next draw at this node is worth the mass that did not go to y; y leaves
                # the distribution (sampling without replacement) and the rest is renormalised
                v = v * (1.0 - dy)
                d[y] = 0.0
                left = float(d.sum())
                if left > 0.0:
                    d = d / left
                rank += 1
                m_thr = min(m_thr, abs(v - t) / t)
        level = created
    return ThresholdTree(parent, token, sib_rank, first_child, next_sibling, depth, est_value, child_value,
                         mask, n, paths, m_cdf, m_thr, levels)
