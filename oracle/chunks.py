"""Chunks, sweeping partitions and the switching controller (oracle; test infrastructure).

Follows the paper's "Chunks and Efficient Partition Construction" paragraph, its coverage
guarantee and the "Training Controller and Partitions Switching" subsection: the graph is
split once into chunks; a worker pins a base chunk and its partition for a super-epoch is
the base chunk combined with one other ("swept") chunk; across super-epochs the swept chunk
advances round-robin, so that every pair of chunks co-resides in some partition.

Readings taken where the paper is silent:
  * chunks are a random (hash) split: ``chunk(v) = owner(v)`` of ``oracle.graph`` with
    ``n_parts = n_chunks``;
  * a partition's nodes are the union of the two chunks, numbered in ascending global id;
    its edges are the edges with both endpoints in that union (no halos), in the same
    canonical CSR/CSC as a plain partition;
  * worker i (base chunk i) sweeps chunk ``(i + 1 + t) mod c`` in super-epoch ``t``; with
    ``c`` chunks the cycle has ``c - 1`` super-epochs, and every chunk is swept by exactly one
    worker in each of them;
  * a partition's loss nodes are the training nodes of its *base* chunk (each training node
    then belongs to exactly one partition per epoch, "a full pass over training nodes");
    the swept chunk only supplies neighbours;
  * controller: a super-epoch lasts ``ceil(e / (c - 1))`` epochs for ``e`` epochs in total;
    the coverage deficit of a step is ``1 - c_hat`` with ``c_hat`` the mean over the active
    partitions of the minimum-distance factor (mean of d_local / d_global over the loss
    nodes); an earlier switch is triggered once the deficit has exceeded ``threshold`` for
    ``patience`` consecutive steps.
"""
from __future__ import annotations

import numpy as np

from . import graph


def chunk_of(n_nodes: int, n_chunks: int, seed: int) -> np.ndarray:
    """Chunk id of every node (the random split, done once)."""
    return graph.owner(n_nodes, n_chunks, seed)


def sweep_schedule(n_chunks: int):
    """List over the super-epochs of a cycle of [(base, swept) for every worker]."""
    if n_chunks < 2:
        return [[(0, 0)]] if n_chunks == 1 else []
    return [[(i, (i + 1 + t) % n_chunks) for i in range(n_chunks)] for t in range(n_chunks - 1)]


def partition_from_chunks(src, dst, n_nodes: int, n_chunks: int, seed: int, base: int, swept: int,
                          assignment=None) -> dict:
    """Local subgraph of the partition base-chunk + swept-chunk (``swept == base``: the base
    chunk alone).  Same dict as ``graph.partition`` plus ``base_mask`` (uint8 per local node:
    1 for the base chunk's nodes).  ``assignment`` (optional int array [n_nodes], values in
    [0, n_chunks)) replaces the random split by any partitioner's output (the paper's chunks come
    from strategies "such as random or METIS"); ``seed`` is then unused."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if not (0 <= base < n_chunks and 0 <= swept < n_chunks):
        raise ValueError("chunk id out of range")
    if src.size and (src.min() < 0 or dst.min() < 0 or src.max() >= n_nodes or dst.max() >= n_nodes):
        raise ValueError("node id out of range")
    if assignment is None:
        ch = chunk_of(n_nodes, n_chunks, seed)
    else:
        ch = np.asarray(assignment, dtype=np.int32)
        if ch.shape != (n_nodes,) or (ch.size and (ch.min() < 0 or ch.max() >= n_chunks)):
            raise ValueError("assignment must give every node a chunk in [0, n_chunks)")
    member = (ch == base) | (ch == swept)
    l2g = np.flatnonzero(member).astype(np.int64)
    n = int(l2g.size)
    g2l = np.full(n_nodes, -1, dtype=np.int64)
    g2l[l2g] = np.arange(n, dtype=np.int64)
    keep = member[src] & member[dst]
    d_global_all = np.bincount(dst, minlength=n_nodes).astype(np.int64)
    part = graph.local_graph_from_edges(g2l[src[keep]], g2l[dst[keep]], n, d_global_all[l2g])
    part["l2g"] = l2g
    part["base_mask"] = (ch[l2g] == base).astype(np.uint8)
    return part


class Controller:
    """Decides when the next super-epoch starts."""

    def __init__(self, total_epochs: int, n_chunks: int, threshold: float = 1.0, patience: int = 1 << 30):
        self.n_chunks = n_chunks
        self.epochs_per_super_epoch = max(1, -(-total_epochs // max(1, n_chunks - 1)))
        self.threshold, self.patience = threshold, patience
        self.super_epoch = 0
        self.epochs_in_super_epoch = 0
        self.over = 0

    def observe_step(self, c_hats) -> None:
        """``c_hats``: the active partitions' minimum-distance factors of this step."""
        deficit = 1.0 - float(np.mean(c_hats))
        self.over = self.over + 1 if deficit > self.threshold else 0

    def end_epoch(self) -> bool:
        """True if the partitions must be switched before the next epoch."""
        self.epochs_in_super_epoch += 1
        if self.epochs_in_super_epoch >= self.epochs_per_super_epoch or self.over >= self.patience:
            self.super_epoch += 1
            self.epochs_in_super_epoch = 0
            self.over = 0
            return True
        return False

    def pairs(self):
        """(base, swept) of every worker for the current super-epoch (the cycle repeats)."""
        sched = sweep_schedule(self.n_chunks)
        return sched[self.super_epoch % len(sched)]
