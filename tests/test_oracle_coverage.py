"""Pins for oracle.coverage: the estimator's invariants (full coverage -> plain average,
the minimum-distance factor is the mean of the node-level weights), the literal
per-neighbour formulas written as loops, the closed form of the shrinkage sum as a count
of dropped in-edges, and linearity / permutation of the aggregation."""
import numpy as np
import pytest

import synth
from oracle import coverage as cov
from oracle import gnn, graph, step

VARIANTS = [cov.NONE, cov.NODE_LEVEL, cov.BATCH_MIN_DIST, cov.SHRINKAGE]


def _parts(N=400, E=4000, K=4, seed=1, gseed=31):
    s, d = synth.uniform_graph(N, E, seed=gseed)
    s, d = s.numpy(), d.numpy()
    return s, d, [graph.partition(s, d, N, K, seed, p) for p in range(K)]


def test_full_coverage_reduces_to_plain_average():
    # K = 1 split of the graph replicated: d_local == d_global for every node
    s, d = synth.uniform_graph(50, 300, seed=3)
    part = graph.partition(s.numpy(), d.numpy(), 50, 1, 0, 0)
    dims = [4, 5, 3]
    x = synth.normal_matrix(50, 4, 1).double().numpy()
    y = synth.labels(50, 3, 1).numpy()
    grads, stats = [], []
    for t in range(3):
        theta = synth.model_weights("sage", dims, 10 + t).double().numpy()
        for est in VARIANTS:
            g, st = step.train_step(part, "sage", dims, theta, x, y, estimator=est)
            if est == cov.NONE:
                g0 = g
            np.testing.assert_array_equal(g, g0)          # node weights are all exactly 1
        grads.append(g0)
        stats.append(st)
    plain = sum(grads) / 3
    for v in VARIANTS:
        G, c = cov.aggregate(grads, stats, v)
        assert (c == 1.0).all()
        np.testing.assert_allclose(G, plain, rtol=1e-15, atol=0)


def test_min_distance_factor_is_mean_of_node_weights_and_literal_formula():
    s, d, parts = _parts()
    for part in parts:
        n = part["n"]
        nodes = np.arange(n)
        st = cov.coverage_stats(part["d_local_in"], part["d_global_in"], nodes)
        w = cov.node_weights(part["d_local_in"], part["d_global_in"])
        assert abs(cov.factor(st, cov.BATCH_MIN_DIST) - w.mean()) < 1e-15
        # literal batch-level factor: mean_v mean_{u in local N_v} p_v(u)/q_v(u), with
        # p = 1/d_global and q = 1/d_local, for nodes that have a local neighbour
        tot = 0.0
        for v in range(n):
            dl, dg = int(part["d_local_in"][v]), int(part["d_global_in"][v])
            if dl > 0:
                tot += sum((1.0 / dg) / (1.0 / dl) for _ in range(dl)) / dl
            elif dg == 0:
                tot += 1.0
        assert abs(tot / n - cov.factor(st, cov.BATCH_MIN_DIST)) < 1e-12


def test_hash_partition_gives_factor_near_one_over_k():
    N, E, K = 10000, 100000, 4
    s, d = synth.uniform_graph(N, E, seed=2602018721)
    part = graph.partition(s.numpy(), d.numpy(), N, K, 1, 0)
    st = cov.coverage_stats(part["d_local_in"], part["d_global_in"], np.arange(part["n"]))
    c = cov.factor(st, cov.BATCH_MIN_DIST)
    assert abs(c - 1.0 / K) < 0.02


def test_shrinkage_sum_counts_dropped_in_edges():
    N, K, seed = 400, 4, 1
    s, d, parts = _parts(N=N, K=K, seed=seed)
    own = graph.owner(N, K, seed)
    for p, part in enumerate(parts):
        mask = synth.train_mask(part["n"], 0.5, 9).numpy()
        nodes = np.flatnonzero(mask)
        st = cov.coverage_stats(part["d_local_in"], part["d_global_in"], nodes)
        in_s = np.zeros(N, dtype=bool)
        in_s[part["l2g"][nodes]] = True
        dropped = sum(1 for u, v in zip(s.tolist(), d.tolist()) if in_s[v] and own[u] != p)
        assert st["R"] == float(dropped) and dropped > 1
        c = cov.factor(st, cov.SHRINKAGE)
        assert c == 1.0 / dropped
        assert c <= 1.0
        assert c < cov.factor(st, cov.BATCH_MIN_DIST)          # "lower correction factors"


def test_shrinkage_literal_formula_in_minibatch_mode():
    dl = np.array([4, 0, 3, 10, 2])
    dg = np.array([8, 5, 3, 40, 0 + 2])
    sc = np.array([2, 0, 3, 5, 2])                             # |S_v| <= d_local
    st = cov.coverage_stats(dl, dg, np.arange(5), sc)
    lit = sum((dg[v] / dl[v] - 1.0) * sc[v] for v in range(5) if dl[v] > 0)
    assert abs(st["R"] - lit) < 1e-12
    assert abs(cov.factor(st, cov.SHRINKAGE) - 1.0 / lit) < 1e-15
    # full-graph mode: |S_v| = d_local, also where d_local = 0
    st2 = cov.coverage_stats(dl, dg, np.arange(5), None)
    assert st2["R"] == float((dg - dl).sum())


def test_boundary_conventions():
    w = cov.node_weights([0, 0, 3], [0, 4, 3])
    assert w.tolist() == [1.0, 0.0, 1.0]
    assert cov.factor(dict(S=5, sum_ratio=5.0, R=0.0), cov.SHRINKAGE) == 1.0
    assert cov.factor(dict(S=5, sum_ratio=5.0, R=0.5), cov.SHRINKAGE) == 2.0    # literal, unclamped
    assert cov.factor(dict(S=0, sum_ratio=0.0, R=0.0), cov.BATCH_MIN_DIST) == 1.0
    with pytest.raises(ValueError):
        cov.factor(dict(S=1, sum_ratio=1.0, R=0.0), 9)


def test_aggregate_is_scale_then_reduce_linear_and_permutation_invariant():
    rng = np.random.default_rng(0)
    K, P = 5, 37
    grads = [rng.standard_normal(P) for _ in range(K)]
    stats = [dict(S=10 + p, sum_ratio=3.0 + p, R=float(2 + 3 * p)) for p in range(K)]
    for v in VARIANTS:
        G, c = cov.aggregate(grads, stats, v)
        pre = [c[p] * grads[p] for p in range(K)]
        np.testing.assert_allclose(G, sum(pre) / K, rtol=1e-15)
        perm = [3, 0, 4, 1, 2]
        G2, c2 = cov.aggregate([grads[i] for i in perm], [stats[i] for i in perm], v)
        np.testing.assert_allclose(G2, G, rtol=1e-12, atol=1e-15)
        G3, _ = cov.aggregate([2.0 * g for g in grads], stats, v)
        np.testing.assert_allclose(G3, 2.0 * G, rtol=1e-15)
    same = [grads[0]] * K
    G, _ = cov.aggregate(same, stats, cov.NONE)
    np.testing.assert_allclose(G, grads[0], rtol=1e-15)
    Gm, cm = cov.aggregate(grads, stats, cov.BATCH_MIN_DIST)
    assert cm.tolist() == [(3.0 + p) / (10 + p) for p in range(K)]
    Gs, cs = cov.aggregate(grads, stats, cov.SHRINKAGE)
    assert cs.tolist() == [1.0 / (2 + 3 * p) for p in range(K)]


def test_empty_partition_counts_in_k():
    e = np.zeros(0, dtype=np.int64)
    dims = [3, 2]
    theta = synth.model_weights("gcn", dims, 1).double().numpy()
    sizes = [graph.partition(e, e, 2, 8, 0, p)["n"] for p in range(8)]
    p_empty = sizes.index(0)
    part = graph.partition(e, e, 2, 8, 0, p_empty)
    g, st = step.train_step(part, "gcn", dims, theta, np.zeros((0, 3)), np.zeros(0, dtype=np.int32))
    assert st["S"] == 0 and st["loss"] == 0.0 and (g == 0).all()
    G, c = cov.aggregate([g, np.ones_like(g)], [st, dict(S=1, sum_ratio=1.0, R=0.0)], cov.BATCH_MIN_DIST)
    np.testing.assert_allclose(G, 0.5 * np.ones_like(g))
