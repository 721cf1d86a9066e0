"""Random node assignment and the isolated local subgraph (oracle; test infrastructure).

Follows the paper's "Graph Partitioning" paragraph (nodes are assigned to partitions at
random, with no regard to structure) and its "Isolated Training" paragraph (a partition
trains on exclusively local nodes and edges).  Halo nodes are not modelled: an edge
whose two endpoints are not owned by the same partition is dropped.

Readings taken where the paper is silent:
  * "random" = the SplitMix64 sequence: ``owner(v)`` is output number ``v`` (counting
    from 0) of the SplitMix64 generator seeded with ``seed``, reduced ``mod K``
    (unsigned).  Output ``v`` is ``mix(seed + (v + 1) * GAMMA)`` in wrapping 64-bit
    arithmetic, with ``mix`` the generator's finaliser.
  * degrees are in-degrees counted with multiplicity (node ``v`` aggregates over the
    edges ``u -> v``); duplicate edges and self-loops are kept as given.
  * local ids number a partition's nodes in ascending global id.
  * canonical CSR: rows are destinations, columns (sources) ascending inside a row;
    canonical CSC: rows are sources, destinations ascending.  Equal entries are
    indistinguishable, so the arrays are unique.
"""
from __future__ import annotations

import numpy as np

GAMMA = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def splitmix64_output(seed: int, index) -> np.ndarray:
    """Output number ``index`` (0-based) of the SplitMix64 sequence seeded with ``seed``."""
    idx = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + (idx + np.uint64(1)) * GAMMA
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
        z = z ^ (z >> np.uint64(31))
    return z


def owner(n_nodes: int, n_parts: int, seed: int) -> np.ndarray:
    """Partition id of every global node id in ``[0, n_nodes)`` (int32)."""
    if n_parts < 1:
        raise ValueError("n_parts must be >= 1")
    h = splitmix64_output(seed, np.arange(n_nodes, dtype=np.uint64))
    return (h % np.uint64(n_parts)).astype(np.int32)


def partition(src, dst, n_nodes: int, n_parts: int, seed: int, part_id: int, weights=None) -> dict:
    """Local subgraph of partition ``part_id`` with cut edges removed.

    ``src[e] -> dst[e]`` are global ids; node ``dst`` aggregates from ``src``.
    Returns a dict of numpy arrays:
      n, nnz, l2g[int64 n], rowptr[int64 n+1], col[int32 nnz] (CSR by destination),
      colptr[int64 n+1], row[int32 nnz] (CSC by source),
      d_local_in[int32 n], d_local_out[int32 n], d_global_in[int64 n].
    ``weights[e] > 0`` (optional, fp32 values): the neighbour distribution of node v is
    p_v(u) = w(u->v) / sum of the weights of all in-edges of v (the general, non-uniform case of
    the coverage-corrected estimators).  The dict then also holds csr_w[float32 nnz] and
    csc_w[float32 nnz] (the kept edges' weights in CSR / CSC order; equal (dst, src) pairs keep
    their order in the edge list), w_local_in[float64 n] (sum of the local in-edge weights, added
    in CSR order) and w_global_in[float64 n] (sum over all in-edges, added in edge-list order).
    """
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if src.shape != dst.shape:
        raise ValueError("src/dst length mismatch")
    if not (0 <= part_id < n_parts):
        raise ValueError("part_id out of range")
    if src.size and (src.min() < 0 or dst.min() < 0 or src.max() >= n_nodes or dst.max() >= n_nodes):
        raise ValueError("node id out of range")

    own = owner(n_nodes, n_parts, seed)
    mine = own == part_id
    l2g = np.flatnonzero(mine).astype(np.int64)          # ascending global id
    n = int(l2g.size)
    g2l = np.full(n_nodes, -1, dtype=np.int64)
    g2l[l2g] = np.arange(n, dtype=np.int64)

    d_global_all = np.bincount(dst, minlength=n_nodes).astype(np.int64)

    keep = mine[src] & mine[dst]
    ls = g2l[src[keep]]
    ld = g2l[dst[keep]]
    nnz = int(ls.size)

    order = np.lexsort((ls, ld))                          # primary: destination, then source
    col = ls[order].astype(np.int32)
    d_in = np.bincount(ld, minlength=n).astype(np.int64)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(d_in, out=rowptr[1:])

    order_t = np.lexsort((ld, ls))                        # primary: source, then destination
    row = ld[order_t].astype(np.int32)
    d_out = np.bincount(ls, minlength=n).astype(np.int64)
    colptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(d_out, out=colptr[1:])

    out = dict(n=n, nnz=nnz, l2g=l2g, rowptr=rowptr, col=col, colptr=colptr, row=row,
               d_local_in=d_in.astype(np.int32), d_local_out=d_out.astype(np.int32),
               d_global_in=d_global_all[l2g])
    if weights is not None:
        w = np.asarray(weights, dtype=np.float32)
        if w.shape != src.shape or not np.all(w > 0) or not np.all(np.isfinite(w)):
            raise ValueError("edge weights must be positive, finite and one per edge")
        wk = w[keep]
        out["csr_w"] = wk[order]
        out["csc_w"] = wk[order_t]
        w_local = np.zeros(n, dtype=np.float64)
        np.add.at(w_local, ld[order], wk[order].astype(np.float64))           # CSR order
        w_global_all = np.zeros(n_nodes, dtype=np.float64)
        np.add.at(w_global_all, dst, w.astype(np.float64))                    # edge-list order
        out["w_local_in"] = w_local
        out["w_global_in"] = w_global_all[l2g]
    return out


def local_graph_from_edges(src_local, dst_local, n: int, d_global_in=None) -> dict:
    """Canonical CSR/CSC of an already-local edge list (ids in ``[0, n)``).

    Used when a partition's share is generated directly.  ``d_global_in`` defaults to the
    local in-degree (full coverage).
    """
    ls = np.asarray(src_local, dtype=np.int64)
    ld = np.asarray(dst_local, dtype=np.int64)
    order = np.lexsort((ls, ld))
    col = ls[order].astype(np.int32)
    d_in = np.bincount(ld, minlength=n).astype(np.int64)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(d_in, out=rowptr[1:])
    order_t = np.lexsort((ld, ls))
    row = ld[order_t].astype(np.int32)
    d_out = np.bincount(ls, minlength=n).astype(np.int64)
    colptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(d_out, out=colptr[1:])
    dg = d_in.copy() if d_global_in is None else np.asarray(d_global_in, dtype=np.int64)
    return dict(n=int(n), nnz=int(ls.size), l2g=np.arange(n, dtype=np.int64), rowptr=rowptr,
                col=col, colptr=colptr, row=row, d_local_in=d_in.astype(np.int32),
                d_local_out=d_out.astype(np.int32), d_global_in=dg)


def partition_halo(src, dst, n_nodes: int, n_parts: int, seed: int, part_id: int, hops: int = 1) -> dict:
    """Partition ``part_id`` extended by ``hops`` hops of read-only halo nodes.

    The paper's "Graph Partitioning" paragraph: the edges linked to a partition's nodes are
    included, and an endpoint that is not part of the partition is incorporated as a halo node.
    Reading: hop 0 is the owned node set; hop h adds the sources of every edge whose
    destination is in hops 0..h-1; the local edges are the edges whose destination is in hops
    0..hops-1 (so the outermost halo nodes have features but no in-edges).  Local ids number
    the whole set in ascending global id; ``owned_mask`` (uint8) marks the owned nodes, which
    are the only loss nodes.  With hops = 0 this is ``partition``.  Same arrays otherwise.
    """
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if hops < 0:
        raise ValueError("hops must be >= 0")
    if not (0 <= part_id < n_parts):
        raise ValueError("part_id out of range")
    if src.size and (src.min() < 0 or dst.min() < 0 or src.max() >= n_nodes or dst.max() >= n_nodes):
        raise ValueError("node id out of range")
    owned = owner(n_nodes, n_parts, seed) == part_id
    inner = owned.copy()                                  # hops 0..h-1: nodes that keep their in-edges
    member = owned.copy()
    for _ in range(hops):
        inner = member.copy()
        member = member.copy()
        member[src[inner[dst]]] = True
    if hops == 0:
        keep = member[src] & member[dst]
    else:
        keep = inner[dst]
    l2g = np.flatnonzero(member).astype(np.int64)
    n = int(l2g.size)
    g2l = np.full(n_nodes, -1, dtype=np.int64)
    g2l[l2g] = np.arange(n, dtype=np.int64)
    d_global_all = np.bincount(dst, minlength=n_nodes).astype(np.int64)
    part = local_graph_from_edges(g2l[src[keep]], g2l[dst[keep]], n, d_global_all[l2g])
    part["l2g"] = l2g
    part["owned_mask"] = owned[l2g].astype(np.uint8)
    return part
