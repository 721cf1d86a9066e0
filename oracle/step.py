"""One partition's isolated train step (oracle glue; test infrastructure).

Puts the pieces in the order of the paper's phase-parallel algorithm: (isolated
sampling) -> forward -> backward -> coverage statistics.  The scaling by the coverage
factor and the reduction over partitions are in ``coverage.aggregate``.
"""
from __future__ import annotations

import numpy as np

from . import coverage, dropout as dropout_mod, gat, gnn, sampling


def train_step(part: dict, arch: str, dims, theta, x, labels, train_mask=None,
               estimator: int = coverage.NONE, gcn_self_loops: bool = True,
               minibatch: dict | None = None, relu_flip=None, near_kink=None,
               dropout: dict | None = None, relu_set=None, keep_z=None):
    """Returns (grad[P] float64, stats dict) for one partition.

    full-graph mode (``minibatch is None``): every local node is an input, the loss runs
    over the local nodes selected by ``train_mask`` (all if None).
    mini-batch mode: ``minibatch = dict(seeds=int array of local ids, fanouts=(f_0..f_{k-1}),
    sampler_seed=int, batch_id=int)``; fanouts[l] belongs to layer l, layer 0 being the input
    side, so the seeds draw fanouts[k-1] neighbours.
    ``relu_flip`` / ``near_kink`` / ``relu_set`` / ``keep_z`` are passed to ``gnn.forward_backward``; with
    ``near_kink`` the stats dict gains the key "near_kink".
    A partition built with edge weights (``graph.partition(..., weights=)``) trains the weighted-mean
    GraphSAGE aggregator and reports the coverage statistics of the weight masses (full-graph mode).
    ``dropout = dict(rate=, seed=, batch_id=)`` drops hidden activations as ``dropout.py`` describes,
    keyed on the nodes' global ids ``part["l2g"]`` (in mini-batch mode a block row is the node it stands
    for, and batch_id defaults to the sampler's).
    """
    n = part["n"]
    k = len(dims) - 1
    dl, dg = part["d_local_in"], part["d_global_in"]
    weighted = part.get("csr_w") is not None
    if weighted and (arch != "sage" or minibatch is not None):
        raise ValueError("edge weights are defined for full-graph GraphSAGE steps only")
    if weighted:
        ratio = coverage.node_weights(part["w_local_in"], part["w_global_in"])
    else:
        ratio = coverage.node_weights(dl, dg)
    w_all = ratio if estimator == coverage.NODE_LEVEL else np.ones(n)

    drop = None
    if dropout is not None and float(dropout["rate"]) != 0.0 and minibatch is None:
        drop = dropout_mod.layer_factors(dropout["seed"], dropout.get("batch_id", 0), part["l2g"], dims,
                                         dropout["rate"])
    if minibatch is None:
        blk = gnn.block_from_csr(part["rowptr"], part["col"], ew=part["csr_w"] if weighted else None)
        if train_mask is None:
            loss_nodes = np.arange(n, dtype=np.int64)
        else:
            loss_nodes = np.flatnonzero(np.asarray(train_mask) != 0).astype(np.int64)
        if arch == "gat":
            res = gat.forward_backward(dims, theta, x, blk, labels, w_all, loss_nodes,
                                       relu_flip=relu_flip, near_kink=near_kink, drop=drop, relu_set=relu_set, keep_z=keep_z)
        else:
            res = gnn.forward_backward(arch, dims, theta, x, [blk] * k, labels, w_all, loss_nodes,
                                       gcn_self_loops, relu_flip=relu_flip, near_kink=near_kink, drop=drop, relu_set=relu_set,
                                       keep_z=keep_z)
        loss, grad = res[0], res[1]
        if weighted:
            st = coverage.coverage_stats_weighted(part["w_local_in"], part["w_global_in"], dl, dg, loss_nodes)
        else:
            st = coverage.coverage_stats(dl, dg, loss_nodes, None)
        if near_kink is not None:
            st["near_kink"] = res[2]
        st["loss"] = loss
        st["nnz_used"] = int(part["nnz"])
        return grad, st

    if arch != "sage":
        raise ValueError("mini-batch mode is defined for GraphSAGE only")
    seeds = np.asarray(minibatch["seeds"], dtype=np.int64)
    blocks, input_nodes = sampling.sample_blocks(part, seeds, minibatch["fanouts"],
                                                 minibatch["sampler_seed"], minibatch["batch_id"])
    xin = np.asarray(x)[input_nodes].astype(np.float64)      # gather, then widen (same values)
    nseed = seeds.size
    if dropout is not None and float(dropout["rate"]) != 0.0:
        # a block row is dropped as the node it stands for: layer l's rows are the first n_dst entries of
        # its source list (partition-local ids), keyed by their global ids
        sc = dropout_mod.scale(dropout["rate"])
        drop = []
        for l in range(k - 1):
            nodes_l = blocks[l]["src_nodes"][:blocks[l]["n_dst"]]
            keep = dropout_mod.keep_mask(dropout["seed"], dropout.get("batch_id", minibatch["batch_id"]), l,
                                         np.asarray(part["l2g"])[nodes_l], dims[l + 1], dropout["rate"])
            drop.append(keep.astype(np.float64) * sc)
    res = gnn.forward_backward(arch, dims, theta, xin, blocks, np.asarray(labels)[seeds],
                               w_all[seeds], np.arange(nseed, dtype=np.int64),
                               gcn_self_loops, relu_flip=relu_flip, near_kink=near_kink, relu_set=relu_set, drop=drop,
                               keep_z=keep_z)
    loss, grad = res[0], res[1]
    last = blocks[-1]
    sampled = np.bincount(last["edst"], minlength=nseed)
    st = coverage.coverage_stats(np.asarray(dl)[seeds], np.asarray(dg)[seeds],
                                 np.arange(nseed, dtype=np.int64), sampled)
    st["loss"] = loss
    if near_kink is not None:
        st["near_kink"] = res[2]
    st["nnz_used"] = int(sum(b["esrc"].size for b in blocks))
    return grad, st
