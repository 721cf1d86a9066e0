"""Isolated k-hop neighbour sampling inside one partition (oracle; test infrastructure).

The paper samples k-hop subgraphs from the local partition only (its "Isolated
Training" paragraph and the first step of each worker in the phase-parallel algorithm)
but fixes neither the sampler nor its random numbers.  Reading taken here:

  * uniform sampling without replacement per destination node: a node with at most ``f``
    local in-edges keeps them all; otherwise it keeps a uniformly random ``f``-subset of the
    ``d`` positions of its canonical CSR row, drawn by the classical subset-growing scheme
    (Floyd): for t = 0..f-1 let top = d - f + t and draw r uniformly from [0, top]; the
    subset gains r if it does not hold r yet and top otherwise.  Every f-subset comes out
    with the same probability, and the work per node is O(f) whatever its degree;
  * the t-th draw of node v is r = floor(u * (top + 1) / 2^64) with the 64-bit integer
    u = M(M(M(M(M(sampler_seed) ^ batch_id) ^ layer) ^ global_id(v)) ^ t), where M(x) is the
    SplitMix64 finaliser applied to ``x + GAMMA`` (wrapping 64-bit);
  * layers are built from the seed side inwards; ``fanouts[l]`` belongs to layer ``l``
    (layer 0 = input side), so the seeds draw ``fanouts[k-1]`` neighbours;
  * a block's source list is its destination list (same order) followed by the newly
    reached nodes in ascending local id; a block's edges are ordered by destination and,
    inside a destination, by ascending position.

  * the seeds of an epoch (the paper lets every worker iterate over all of its training nodes once
    per epoch, in no stated order): the partition's training nodes sorted by the 64-bit key
    M(M(M(sampler_seed) ^ epoch) ^ global_id(v)), ties by local id; batch b of the epoch is the slice
    [b * B, (b + 1) * B) of that order, the last one possibly shorter.

Because the draws depend only on (seed, batch, layer, node, t) the result is independent of
evaluation order.
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


def draw_bits(sampler_seed: int, batch_id: int, layer: int, gid, t) -> np.ndarray:
    """The 64 random bits behind draw ``t`` of the node with global id ``gid``."""
    h = _M(np.uint64(sampler_seed & 0xFFFFFFFFFFFFFFFF))
    h = _M(h ^ np.uint64(batch_id))
    h = _M(h ^ np.uint64(layer))
    h = _M(h ^ np.asarray(gid, dtype=np.uint64))
    return _M(h ^ np.asarray(t, dtype=np.uint64))


def scale_draw(u, span) -> np.ndarray:
    """floor(u * span / 2^64) for 64-bit u and span: the uniform draw from [0, span)."""
    u = np.asarray(u, dtype=np.uint64)
    span = np.asarray(span, dtype=np.uint64)
    lo32 = np.uint64(0xFFFFFFFF)
    s32 = np.uint64(32)
    with np.errstate(over="ignore"):
        u0, u1 = u & lo32, u >> s32
        v0, v1 = span & lo32, span >> s32
        mid = (u0 * v0 >> s32) + (u1 * v0 & lo32) + (u0 * v1 & lo32)
        return u1 * v1 + (u1 * v0 >> s32) + (u0 * v1 >> s32) + (mid >> s32)


def grow_subset(d: int, draws) -> list:
    """The subset-growing scheme for one row: ``draws[t]`` is the value drawn from
    [0, d - f + t]; returns the f = len(draws) chosen positions in ascending order."""
    f = len(draws)
    chosen = []
    for t in range(f):
        top = d - f + t
        r = int(draws[t])
        if not 0 <= r <= top:
            raise ValueError("draw outside its range")
        chosen.append(top if r in chosen else r)
    return sorted(chosen)


def sample_layer(part: dict, dst_nodes, fanout: int, sampler_seed: int, batch_id: int, layer: int):
    """Sampled in-edges of ``dst_nodes`` (local ids).  Returns (edst_pos, esrc_local):
    ``edst_pos[e]`` indexes ``dst_nodes``; edges ordered by destination then position."""
    rowptr, col, l2g = part["rowptr"], part["col"], part["l2g"]
    dst_nodes = np.asarray(dst_nodes, dtype=np.int64)
    edst, epos = [], []
    steps = np.arange(fanout, dtype=np.int64)
    for i, v in enumerate(dst_nodes.tolist()):
        b = int(rowptr[v])
        d = int(rowptr[v + 1]) - b
        if d <= fanout:
            pos = range(d)
        else:
            bits = draw_bits(sampler_seed, batch_id, layer, l2g[v], steps)
            pos = grow_subset(d, scale_draw(bits, d - fanout + steps + 1))
        edst.extend([i] * len(pos))
        epos.extend(b + j for j in pos)
    edst = np.asarray(edst, dtype=np.int64)
    epos = np.asarray(epos, dtype=np.int64)
    return edst, col[epos].astype(np.int64)


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


def epoch_seed_order(part: dict, train_mask, sampler_seed: int, epoch: int) -> np.ndarray:
    """Local ids of the partition's training nodes (``train_mask`` non-zero; None = all) in the order an
    epoch visits them: ascending key M(M(M(sampler_seed) ^ epoch) ^ global_id), ties by local id."""
    n = part["n"]
    ids = np.arange(n, dtype=np.int64) if train_mask is None else np.flatnonzero(np.asarray(train_mask) != 0).astype(np.int64)
    h = _M(_M(np.uint64(sampler_seed & 0xFFFFFFFFFFFFFFFF)) ^ np.uint64(epoch))
    keys = _M(h ^ np.asarray(part["l2g"], dtype=np.uint64)[ids])
    return ids[np.lexsort((ids, keys))]
