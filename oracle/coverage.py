"""Coverage-corrected aggregation (oracle; test infrastructure).

Follows the paper's section "Coverage-Corrected Aggregation" for neighbours of equal
weight (p_v(u) = 1/d_global, q_v(u) = 1/d_local):

  node-level weight        w_v = d_local(v) / d_global(v)           (the uniform special
                                                                     case of the
                                                                     asymptotically
                                                                     unbiased estimator)
  minimum-distance factor  c_uniform = (1/|S|) sum_{v in S} d_local(v)/d_global(v)
                                                                     (the uniform form of
                                                                     the batch-level factor)
  shrinkage factor         c_resampling = 1 / sum_{v in S} (d_global/d_local - 1) |S_v|
                                                                     (the shrinkage
                                                                     equation)
  aggregation              G = (1/K) sum_p c_p g_p : each partition's gradient is scaled by
                           its own factor and only then reduced, as the phase-parallel
                           algorithm orders it.

General (non-uniform) neighbour weights: with edge weights w(u->v) the target distribution
is p_v(u) = w(u->v)/W_global(v) and the local one q_v(u) = p_v(u)/sum_{i local} p_v(i) (the
choice the paper names for the general case), so p_v(u)/q_v(u) = W_local(v)/W_global(v) for every
local neighbour: the weight masses W take the place of the degrees in the node-level weight and in
the minimum-distance factor.  The shrinkage factor is only given for degrees; its term becomes
(W_global - W_local) d_local / W_local (the missing mass counted in units of the node's mean local
edge weight), and d_global for a node without local in-edges, which is d_global - d_local again
when every weight is 1.

Readings where the paper is silent (boundary conventions):
  * S = the nodes that carry loss (seeds in mini-batch mode), degrees are the partition's
    in-degrees with multiplicity;
  * d_global = 0  -> ratio 1 (nothing is missing); d_local = 0 < d_global -> ratio 0;
  * the shrinkage sum uses the algebraic form (d_global - d_local) |S_v| / d_local, with
    the term 0 when d_local = 0; in full-graph mode |S_v| = d_local so the term is exactly
    d_global - d_local (also when d_local = 0), an integer count of dropped in-edges;
  * sum R = 0 (full coverage) -> c_resampling := 1; otherwise exactly 1/R, unclamped;
  * the K partitions play the role of the estimator's T terms: plain mean over K, and a
    partition with an empty S contributes a zero gradient but still counts in K.
"""
from __future__ import annotations

import numpy as np

NONE, NODE_LEVEL, BATCH_MIN_DIST, SHRINKAGE = 0, 1, 2, 3


def node_weights(d_local, d_global) -> np.ndarray:
    dl = np.asarray(d_local, dtype=np.float64)
    dg = np.asarray(d_global, dtype=np.float64)
    w = np.ones_like(dl)
    pos = dg > 0
    w[pos] = dl[pos] / dg[pos]
    return w


def coverage_stats(d_local, d_global, loss_nodes, sampled_count=None) -> dict:
    """|S|, sum of degree ratios and the shrinkage sum R over the loss nodes.

    ``sampled_count[v]`` = |S_v| for mini-batch mode; ``None`` means full-graph mode.
    """
    s = np.asarray(loss_nodes, dtype=np.int64)
    dl = np.asarray(d_local, dtype=np.int64)[s]
    dg = np.asarray(d_global, dtype=np.int64)[s]
    sum_ratio = float(node_weights(dl, dg).sum())
    if sampled_count is None:
        r = float((dg - dl).sum())
    else:
        sc = np.asarray(sampled_count, dtype=np.float64)[s]
        ok = dl > 0
        r = float(((dg[ok] - dl[ok]).astype(np.float64) * sc[ok] / dl[ok]).sum())
    return dict(S=int(s.size), sum_ratio=sum_ratio, R=r)


def coverage_stats_weighted(w_local, w_global, d_local, d_global, loss_nodes) -> dict:
    """Full-graph coverage statistics for weighted neighbour distributions (see the module header)."""
    s = np.asarray(loss_nodes, dtype=np.int64)
    wl = np.asarray(w_local, dtype=np.float64)[s]
    wg = np.asarray(w_global, dtype=np.float64)[s]
    dl = np.asarray(d_local, dtype=np.int64)[s]
    dg = np.asarray(d_global, dtype=np.int64)[s]
    sum_ratio = float(node_weights(wl, wg).sum())
    ok = dl > 0
    r = float(((wg[ok] - wl[ok]) * dl[ok] / wl[ok]).sum() + dg[~ok].sum())
    return dict(S=int(s.size), sum_ratio=sum_ratio, R=r)


def factor(stats: dict, variant: int) -> float:
    if variant in (NONE, NODE_LEVEL):
        return 1.0
    if variant == BATCH_MIN_DIST:
        return stats["sum_ratio"] / stats["S"] if stats["S"] > 0 else 1.0
    if variant == SHRINKAGE:
        return 1.0 / stats["R"] if stats["R"] > 0 else 1.0
    raise ValueError("unknown variant")


def aggregate(grads, stats_list, variant: int):
    """(G, c) with G = (1/K) sum_p c_p g_p in fp64."""
    k = len(grads)
    if k < 1 or k != len(stats_list):
        raise ValueError("need one stats record per gradient")
    c = np.array([factor(st, variant) for st in stats_list], dtype=np.float64)
    g = np.zeros_like(np.asarray(grads[0], dtype=np.float64))
    for p in range(k):
        g += c[p] * np.asarray(grads[p], dtype=np.float64)
    return g / k, c
