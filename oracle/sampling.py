"""Isolated k-hop neighbour sampling inside one partition (oracle; test infrastructure).

The paper samples k-hop subgraphs from the local partition only (its "Isolated
Training" paragraph and the first step of each worker in the phase-parallel algorithm)
but fixes neither the sampler nor its random numbers.  Reading taken here:

  * uniform sampling without replacement per destination node: a node with at most ``f``
    local in-edges keeps them all; otherwise it keeps the ``f`` in-edges with the smallest
    64-bit key, ties broken by position;
  * key(e) = M(M(M(M(M(sampler_seed) ^ batch_id) ^ layer) ^ global_id(v)) ^ j) where ``j``
    is the edge's position inside v's canonical CSR row and M(x) is the SplitMix64
    finaliser applied to ``x + GAMMA`` (wrapping 64-bit);
  * layers are built from the seed side inwards; ``fanouts[l]`` belongs to layer ``l``
    (layer 0 = input side), so the seeds draw ``fanouts[k-1]`` neighbours;
  * a block's source list is its destination list (same order) followed by the newly
    reached nodes in ascending local id; a block's edges are ordered by destination and,
    inside a destination, by ascending ``j``.

Because keys depend only on (seed, batch, layer, node, position) the result is
independent of evaluation order.
"""
from __future__ import annotations

import numpy as np

from .graph import GAMMA, _C1, _C2


def _M(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + GAMMA
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
        z = z ^ (z >> np.uint64(31))
    return z


def edge_keys(sampler_seed: int, batch_id: int, layer: int, gid, j) -> np.ndarray:
    h = _M(np.uint64(sampler_seed & 0xFFFFFFFFFFFFFFFF))
    h = _M(h ^ np.uint64(batch_id))
    h = _M(h ^ np.uint64(layer))
    h = _M(h ^ np.asarray(gid, dtype=np.uint64))
    return _M(h ^ np.asarray(j, dtype=np.uint64))


def sample_layer(part: dict, dst_nodes, fanout: int, sampler_seed: int, batch_id: int, layer: int):
    """Sampled in-edges of ``dst_nodes`` (local ids).  Returns (edst_pos, esrc_local):
    ``edst_pos[e]`` indexes ``dst_nodes``; edges ordered by destination then position."""
    rowptr, col, l2g = part["rowptr"], part["col"], part["l2g"]
    dst_nodes = np.asarray(dst_nodes, dtype=np.int64)
    beg = rowptr[dst_nodes]
    deg = rowptr[dst_nodes + 1] - beg
    tot = int(deg.sum())
    owner_pos = np.repeat(np.arange(dst_nodes.size, dtype=np.int64), deg)
    first = np.repeat(np.cumsum(deg) - deg, deg)
    j = np.arange(tot, dtype=np.int64) - first                 # position inside the row
    epos = np.repeat(beg, deg) + j
    big = np.repeat(deg > fanout, deg)
    keep = ~big
    if big.any():
        bi = np.flatnonzero(big)
        keys = edge_keys(sampler_seed, batch_id, layer, l2g[dst_nodes[owner_pos[bi]]], j[bi])
        order = np.lexsort((j[bi], keys, owner_pos[bi]))       # by row, then key, then position
        sorted_rows = owner_pos[bi][order]
        start = np.r_[0, np.flatnonzero(np.diff(sorted_rows)) + 1]
        run_start = np.repeat(start, np.diff(np.r_[start, sorted_rows.size]))
        rank = np.arange(sorted_rows.size) - run_start
        keep[bi[order[rank < fanout]]] = True
    sel = np.flatnonzero(keep)                                  # already (row, position) ordered
    return owner_pos[sel], col[epos[sel]].astype(np.int64)


def sample_blocks(part: dict, seeds, fanouts, sampler_seed: int, batch_id: int):
    """k bipartite blocks (input side first) and the input node list (local ids)."""
    k = len(fanouts)
    dst_nodes = np.asarray(seeds, dtype=np.int64)
    blocks = [None] * k
    for layer in range(k - 1, -1, -1):
        edst, esrc_local = sample_layer(part, dst_nodes, fanouts[layer], sampler_seed, batch_id, layer)
        new = np.setdiff1d(esrc_local, dst_nodes)               # ascending, unique
        src_nodes = np.concatenate([dst_nodes, new])
        lookup = np.full(part["n"], -1, dtype=np.int64)
        lookup[src_nodes] = np.arange(src_nodes.size)
        blocks[layer] = dict(n_dst=int(dst_nodes.size), n_src=int(src_nodes.size),
                             esrc=lookup[esrc_local], edst=edst, src_nodes=src_nodes)
        dst_nodes = src_nodes
    return blocks, dst_nodes
