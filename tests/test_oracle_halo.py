"""Pins for oracle.graph.partition_halo: brute force on tiny graphs, hops = 0 is the plain
partition, owned nodes of a 1-hop halo partition see their whole in-neighbourhood, and a
k-hop halo makes a k-layer model exact on the owned nodes (same logits, loss and gradient as
the whole graph restricted to them)."""
import numpy as np
import pytest

import synth
from oracle import coverage as cov
from oracle import gnn, graph, step

KEYS = ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in")


def _graph(N=200, E=1500, seed=6):
    s, d = synth.uniform_graph(N, E, seed=seed)
    return s.numpy(), d.numpy()


def test_zero_hops_is_the_plain_partition():
    s, d = _graph()
    for p in range(3):
        a = graph.partition_halo(s, d, 200, 3, 5, p, hops=0)
        b = graph.partition(s, d, 200, 3, 5, p)
        for k in KEYS:
            assert np.array_equal(a[k], b[k]), k
        assert a["owned_mask"].all()


@pytest.mark.parametrize("hops", [1, 2, 3])
def test_brute_force_tiny(hops):
    rng = np.random.default_rng(hops)
    N, E, K = 30, 70, 3
    s, d = rng.integers(0, N, E), rng.integers(0, N, E)
    own = graph.owner(N, K, 9)
    for p in range(K):
        part = graph.partition_halo(s, d, N, K, 9, p, hops)
        layers = [set(np.flatnonzero(own == p).tolist())]
        for _ in range(hops):
            cur = set().union(*layers)
            layers.append({int(u) for u, v in zip(s, d) if int(v) in cur} - cur)
        members = sorted(set().union(*layers))
        inner = set().union(*layers[:hops])
        assert list(part["l2g"]) == members
        loc = {v: i for i, v in enumerate(members)}
        rows = [[] for _ in members]
        for u, v in zip(s, d):
            if int(v) in inner:
                rows[loc[int(v)]].append(loc[int(u)])
        assert list(part["col"]) == [x for r in rows for x in sorted(r)]
        assert list(part["owned_mask"]) == [1 if own[v] == p else 0 for v in members]


def test_one_hop_gives_owned_nodes_their_whole_neighbourhood():
    s, d = _graph()
    part = graph.partition_halo(s, d, 200, 4, 1, 2, hops=1)
    m = part["owned_mask"].astype(bool)
    assert np.array_equal(part["d_local_in"][m], part["d_global_in"][m])
    assert (part["d_local_in"][~m] == 0).all()
    st = cov.coverage_stats(part["d_local_in"], part["d_global_in"], np.flatnonzero(m), None)
    assert cov.factor(st, cov.BATCH_MIN_DIST) == 1.0 and st["R"] == 0.0


@pytest.mark.parametrize("arch,dims", [("sage", [5, 6, 3]), ("sage", [5, 4, 4, 3]), ("gat", [5, 6, 3])])
def test_k_hop_halo_is_exact_for_a_k_layer_model(arch, dims):
    N = 160
    s, d = _graph(N=N, E=900, seed=12)
    k = len(dims) - 1
    x = synth.normal_matrix(N, dims[0], 1).double().numpy()
    y = synth.labels(N, dims[-1], 2).numpy()
    theta = synth.model_weights(arch, dims, 3).double().numpy()
    whole = graph.partition(s, d, N, 1, 0, 0)
    own = graph.owner(N, 3, 4) == 1
    # (GCN is left out: its symmetric normalisation also uses out-degrees, which in-edge halos do not complete)
    g_ref, st_ref = step.train_step(whole, arch, dims, theta, x, y, own.astype(np.uint8))
    part = graph.partition_halo(s, d, N, 3, 4, 1, hops=k)
    g, st = step.train_step(part, arch, dims, theta, x[part["l2g"]], y[part["l2g"]], part["owned_mask"])
    assert st["S"] == st_ref["S"]
    np.testing.assert_allclose(st["loss"], st_ref["loss"], rtol=1e-12)
    np.testing.assert_allclose(g, g_ref, rtol=1e-10, atol=1e-13)
    # one hop fewer is not exact
    part1 = graph.partition_halo(s, d, N, 3, 4, 1, hops=k - 1)
    g1, _ = step.train_step(part1, arch, dims, theta, x[part1["l2g"]], y[part1["l2g"]], part1["owned_mask"])
    assert np.abs(g1 - g_ref).max() > 1e-6
