"""The seeded input generators: the directly generated sorted share must be the same edge multiset as the
edge-list generator's, in the canonical order the oracle defines."""
import numpy as np
import torch

import synth
from oracle import graph as ograph


def test_rmat_local_csr_is_the_canonical_csr_of_the_edge_list():
    for n, E, chunk, slice_edges in ((1000, 50000, 7000, 6000), (4096, 30000, 1 << 20, 1 << 20), (17, 900, 100, 50)):
        s, d = synth.rmat_graph(12, E, seed=5, n_nodes=n)
        want = ograph.local_graph_from_edges(s.numpy(), d.numpy(), n)
        rowptr, col = synth.rmat_local_csr(12, E, seed=5, n_nodes=n, chunk=chunk, slice_edges=slice_edges)
        assert rowptr.dtype == torch.int64 and col.dtype == torch.int32
        assert np.array_equal(rowptr.numpy(), want["rowptr"]) and np.array_equal(col.numpy(), want["col"])


def test_rmat_graph_does_not_depend_on_the_chunk_size():
    a = synth.rmat_graph(10, 5000, seed=3, chunk=777)
    b = synth.rmat_graph(10, 5000, seed=3)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
