"""Pins for oracle.graph: the node hash against published SplitMix64 vectors, the local
subgraph against brute-force Python loops, and the structural invariants of a hash
partition (disjoint cover, edge accounting, CSC = transpose of CSR, K = 1 identity)."""
import os

import numpy as np
import pytest

import synth
from oracle import graph

GOLD = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_vectors.txt")


def test_hash_matches_published_splitmix64_vectors():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 2
    for r in rows:
        seed, want = int(r[0]), [int(x) for x in r[1:]]
        got = graph.splitmix64_output(seed, np.arange(len(want)))
        assert [int(x) for x in got] == want


def test_owner_is_hash_mod_k_unsigned():
    own = graph.owner(1000, 7, 99)
    h = graph.splitmix64_output(99, np.arange(1000))
    assert [int(x) % 7 for x in h] == own.tolist()


def _brute_partition(src, dst, n_nodes, K, seed, p):
    own = [int(graph.splitmix64_output(seed, v)) % K for v in range(n_nodes)]
    l2g = [v for v in range(n_nodes) if own[v] == p]
    g2l = {g: i for i, g in enumerate(l2g)}
    rows = [[] for _ in l2g]
    cols = [[] for _ in l2g]
    dg = [0] * n_nodes
    for u, v in zip(src, dst):
        dg[v] += 1
        if own[u] == p and own[v] == p:
            rows[g2l[v]].append(g2l[u])
            cols[g2l[u]].append(g2l[v])
    rowptr, col, colptr, row = [0], [], [0], []
    for r in rows:
        col += sorted(r)
        rowptr.append(len(col))
    for c in cols:
        row += sorted(c)
        colptr.append(len(row))
    return l2g, rowptr, col, colptr, row, [dg[g] for g in l2g]


@pytest.mark.parametrize("K,seed", [(1, 0), (3, 5), (4, 1), (50, 2)])
def test_partition_matches_brute_force(K, seed):
    n_nodes, n_edges = 40, 300
    s, d = synth.uniform_graph(n_nodes, n_edges, seed=11)
    s, d = s.numpy(), d.numpy()
    total_nnz = 0
    seen = np.zeros(n_nodes, dtype=int)
    for p in range(K):
        part = graph.partition(s, d, n_nodes, K, seed, p)
        l2g, rowptr, col, colptr, row, dg = _brute_partition(s.tolist(), d.tolist(), n_nodes, K, seed, p)
        assert part["l2g"].tolist() == l2g
        assert part["rowptr"].tolist() == rowptr
        assert part["col"].tolist() == col
        assert part["colptr"].tolist() == colptr
        assert part["row"].tolist() == row
        assert part["d_global_in"].tolist() == dg
        assert part["d_local_in"].tolist() == np.diff(rowptr).tolist()
        assert part["d_local_out"].tolist() == np.diff(colptr).tolist()
        assert (part["d_local_in"] <= part["d_global_in"]).all()
        assert part["col"].dtype == np.int32 and part["rowptr"].dtype == np.int64
        seen[part["l2g"]] += 1
        total_nnz += part["nnz"]
    assert (seen == 1).all()                      # parts are disjoint and cover [0, N)
    own = graph.owner(n_nodes, K, seed)
    cut = int((own[s] != own[d]).sum())
    assert total_nnz + cut == n_edges


def test_k1_is_identity_relabel_and_counting_sort():
    s, d = synth.uniform_graph(30, 200, seed=3)
    s, d = s.numpy(), d.numpy()
    part = graph.partition(s, d, 30, 1, 123, 0)
    assert part["l2g"].tolist() == list(range(30))
    assert part["nnz"] == 200
    pairs = sorted(zip(d.tolist(), s.tolist()))
    assert part["col"].tolist() == [u for _, u in pairs]
    assert (part["d_local_in"] == part["d_global_in"]).all()


def test_csc_is_transpose_multiset():
    s, d = synth.rmat_graph(8, 4000, seed=4)
    part = graph.partition(s.numpy(), d.numpy(), 256, 2, 1, 0)
    n = part["n"]
    e1 = sorted(zip(np.repeat(np.arange(n), np.diff(part["rowptr"])).tolist(), part["col"].tolist()))
    e2 = sorted(zip(part["row"].tolist(), np.repeat(np.arange(n), np.diff(part["colptr"])).tolist()))
    assert e1 == e2
    for r in range(n):                              # ascending inside every row / column
        seg = part["col"][part["rowptr"][r]:part["rowptr"][r + 1]]
        assert (np.diff(seg) >= 0).all()
        seg = part["row"][part["colptr"][r]:part["colptr"][r + 1]]
        assert (np.diff(seg) >= 0).all()


def test_hash_partition_statistics():
    N, E, K = 20000, 200000, 4
    s, d = synth.uniform_graph(N, E, seed=2602018721)
    s, d = s.numpy(), d.numpy()
    sizes, kept = [], 0
    for p in range(K):
        part = graph.partition(s, d, N, K, 1, p)
        sizes.append(part["n"])
        kept += part["nnz"]
    sigma = (N * (1 / K) * (1 - 1 / K)) ** 0.5
    assert all(abs(x - N / K) < 4 * sigma for x in sizes)
    assert abs(kept / E - 1 / K) < 0.01            # an edge survives iff both ends collide


def test_edge_cases():
    e = np.zeros(0, dtype=np.int64)
    part = graph.partition(e, e, 10, 3, 0, 1)
    assert part["nnz"] == 0 and part["rowptr"].tolist() == [0] * (part["n"] + 1)
    # more partitions than nodes: some parts are empty
    sizes = [graph.partition(e, e, 3, 64, 0, p)["n"] for p in range(64)]
    assert sum(sizes) == 3
    with pytest.raises(ValueError):
        graph.partition(np.array([0]), np.array([10]), 10, 2, 0, 0)
    with pytest.raises(ValueError):
        graph.partition(e, e, 10, 2, 0, 2)
    with pytest.raises(ValueError):
        graph.owner(10, 0, 0)


def test_local_graph_from_edges_agrees_with_k1_partition():
    s, d = synth.uniform_graph(25, 120, seed=8)
    a = graph.partition(s.numpy(), d.numpy(), 25, 1, 0, 0)
    b = graph.local_graph_from_edges(s.numpy(), d.numpy(), 25)
    for k in ("rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in"):
        assert a[k].tolist() == b[k].tolist()
