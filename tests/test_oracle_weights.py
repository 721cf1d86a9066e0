"""Pins for the general (non-uniform) neighbour weights in the oracle: brute-force partition
arrays, constant weights = the uniform case, integer weights = a multigraph, a dense weighted-mean
forward pass, finite differences, and the importance-sampling identity behind the node-level
weight W_local / W_global."""
import numpy as np
import pytest

import synth
from oracle import coverage as cov
from oracle import gnn, graph, step


def _graph(N=60, E=400, seed=3):
    s, d = synth.uniform_graph(N, E, seed=seed)
    s, d = s.numpy().copy(), d.numpy().copy()
    # duplicates with different weights, a self-loop
    s = np.concatenate([s, [5, 5, 5, 7]])
    d = np.concatenate([d, [9, 9, 9, 7]])
    rng = np.random.default_rng(seed)
    w = rng.uniform(0.1, 3.0, s.size).astype(np.float32)
    return s, d, w, N


def test_partition_weight_arrays_by_brute_force():
    s, d, w, N = _graph()
    K = 3
    own = graph.owner(N, K, 4)
    for p in range(K):
        part = graph.partition(s, d, N, K, 4, p, weights=w)
        plain = graph.partition(s, d, N, K, 4, p)
        for key in ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_global_in"):
            assert np.array_equal(part[key], plain[key])
        loc = {int(v): i for i, v in enumerate(part["l2g"])}
        kept = [(loc[int(b)], loc[int(a)], float(x), e) for e, (a, b, x) in enumerate(zip(s, d, w))
                if own[a] == p and own[b] == p]
        csr = sorted(kept, key=lambda t: (t[0], t[1], t[3]))            # equal pairs stay in edge order
        csc = sorted(kept, key=lambda t: (t[1], t[0], t[3]))
        assert [t[2] for t in csr] == [float(x) for x in part["csr_w"]]
        assert [t[2] for t in csc] == [float(x) for x in part["csc_w"]]
        wl = np.zeros(part["n"]); wg = np.zeros(part["n"])
        for t in csr:
            wl[t[0]] += t[2]
        for a, b, x in zip(s, d, w):
            if own[b] == p:
                wg[loc[int(b)]] += float(x)
        assert np.array_equal(wl, part["w_local_in"]) and np.array_equal(wg, part["w_global_in"])
    with pytest.raises(ValueError):
        graph.partition(s, d, N, K, 4, 0, weights=np.zeros_like(w))


def _inputs(n, dims, seed=2):
    x = synth.normal_matrix(n, dims[0], seed).double().numpy()
    y = synth.labels(n, dims[-1], seed).numpy()
    theta = synth.model_weights("sage", dims, seed).double().numpy()
    return x, y, theta


@pytest.mark.parametrize("c", [1.0, 2.5])
@pytest.mark.parametrize("est", [cov.NONE, cov.NODE_LEVEL])
def test_constant_weights_are_the_uniform_case(c, est):
    s, d, _, N = _graph()
    dims = [5, 7, 6, 3]
    for p in range(2):
        a = graph.partition(s, d, N, 2, 1, p, weights=np.full(s.size, c, dtype=np.float32))
        b = graph.partition(s, d, N, 2, 1, p)
        x, y, theta = _inputs(a["n"], dims)
        ga, sa = step.train_step(a, "sage", dims, theta, x, y, estimator=est)
        gb, sb = step.train_step(b, "sage", dims, theta, x, y, estimator=est)
        np.testing.assert_allclose(ga, gb, rtol=1e-9, atol=1e-13)
        for k in ("S", "sum_ratio", "R", "loss"):
            assert abs(sa[k] - sb[k]) <= 1e-9 * max(1.0, abs(sb[k])), k
        for v in (cov.BATCH_MIN_DIST, cov.SHRINKAGE):
            assert abs(cov.factor(sa, v) - cov.factor(sb, v)) < 1e-9


def test_integer_weights_are_a_multigraph():
    rng = np.random.default_rng(8)
    N, E = 40, 150
    s, d = rng.integers(0, N, E), rng.integers(0, N, E)
    mult = rng.integers(1, 4, E)
    dims = [4, 6, 3]
    for p in range(2):
        a = graph.partition(s, d, N, 2, 6, p, weights=mult.astype(np.float32))
        b = graph.partition(np.repeat(s, mult), np.repeat(d, mult), N, 2, 6, p)
        x, y, theta = _inputs(a["n"], dims, seed=5)
        for est in (cov.NONE, cov.NODE_LEVEL):
            ga, sa = step.train_step(a, "sage", dims, theta, x, y, estimator=est)
            gb, sb = step.train_step(b, "sage", dims, theta, x, y, estimator=est)
            np.testing.assert_allclose(ga, gb, rtol=1e-10, atol=1e-13)
            assert abs(sa["sum_ratio"] - sb["sum_ratio"]) < 1e-10 and abs(sa["loss"] - sb["loss"]) < 1e-12


def test_forward_is_the_dense_weighted_mean_and_gradient_matches_finite_differences():
    s, d, w, N = _graph(N=18, E=70, seed=9)
    part = graph.partition(s, d, N, 1, 0, 0, weights=w)
    dims = [3, 5, 4, 2]
    x, y, theta = _inputs(N, dims, seed=7)
    blk = gnn.block_from_csr(part["rowptr"], part["col"], ew=part["csr_w"])
    nodes = np.array([0, 3, 4, 9, 17])
    nw = np.linspace(0.5, 1.5, N)
    loss, g, logits = gnn.forward_backward("sage", dims, theta, x, [blk] * 3, y, nw, nodes, return_logits=True)
    a = np.zeros((N, N))
    for u, v, ww in zip(s, d, w):
        a[v, u] += float(ww)
    mass = a.sum(axis=1)
    h = x
    for l, (ws, wn, b) in enumerate(gnn.unpack_params(theta, "sage", dims)):
        m = np.where(mass[:, None] > 0, (a @ h) / np.where(mass > 0, mass, 1)[:, None], 0.0)
        z = h @ ws + m @ wn + b
        h = z if l == 2 else np.maximum(z, 0)
    np.testing.assert_allclose(logits, h, rtol=1e-12, atol=1e-12)

    def f(t):
        return gnn.forward_backward("sage", dims, t, x, [blk] * 3, y, nw, nodes)[0]
    fd = np.zeros_like(theta)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += 1e-6
        tm[i] -= 1e-6
        fd[i] = (f(tp) - f(tm)) / 2e-6
    np.testing.assert_allclose(g, fd, rtol=5e-6, atol=5e-8)
    # and the weights matter
    g0 = gnn.forward_backward("sage", dims, theta, x, [gnn.block_from_csr(part["rowptr"], part["col"])] * 3, y, nw, nodes)[1]
    assert np.abs(g - g0).max() > 1e-3


def test_node_level_weight_is_the_importance_ratio():
    # Splitting a node's in-neighbours over disjoint partitions: the local weighted means, each
    # multiplied by W_local / W_global, add up to the global weighted mean (p/q of the general case).
    rng = np.random.default_rng(1)
    for _ in range(20):
        deg = int(rng.integers(1, 30))
        w = rng.uniform(0.05, 4.0, deg)
        g = rng.normal(size=(deg, 3))
        group = rng.integers(0, 4, deg)
        want = (w[:, None] * g).sum(axis=0) / w.sum()
        got = np.zeros(3)
        for p in range(4):
            sel = group == p
            if not sel.any():
                continue
            local_mean = (w[sel, None] * g[sel]).sum(axis=0) / w[sel].sum()
            got += cov.node_weights(np.array([w[sel].sum()]), np.array([w.sum()]))[0] * local_mean
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_weighted_stats_and_refusals():
    s, d, w, N = _graph()
    part = graph.partition(s, d, N, 3, 2, 1, weights=w)
    nodes = np.arange(part["n"])
    st = cov.coverage_stats_weighted(part["w_local_in"], part["w_global_in"], part["d_local_in"], part["d_global_in"], nodes)
    r = 0.0
    ratio = 0.0
    for v in range(part["n"]):
        wl, wg, dl, dg = part["w_local_in"][v], part["w_global_in"][v], int(part["d_local_in"][v]), int(part["d_global_in"][v])
        ratio += wl / wg if wg > 0 else 1.0
        r += (wg - wl) * dl / wl if dl > 0 else dg
    assert abs(st["sum_ratio"] - ratio) < 1e-12 and abs(st["R"] - r) < 1e-9 and st["S"] == part["n"]
    x, y, theta = _inputs(part["n"], [4, 3])
    with pytest.raises(ValueError):
        step.train_step(part, "gcn", [4, 3], synth.model_weights("gcn", [4, 3], 1).double().numpy(), x, y)
    with pytest.raises(ValueError):
        step.train_step(part, "sage", [4, 3], theta, x, y,
                        minibatch=dict(seeds=np.arange(3), fanouts=(2,), sampler_seed=1, batch_id=0))
