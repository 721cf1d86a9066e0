"""Optimizer step and the phase-parallel epoch loop (oracle; test infrastructure).

The paper's phase-parallel algorithm ends every iteration with
``theta <- optimizer_step(theta, grad)`` and carries theta and the optimizer state from one
phase to the next; it names no optimizer (the experimental setup fixes only the learning
rate, 0.003).  Reading taken here: Adam as published by Kingma & Ba (2015, their
Algorithm 1: bias-corrected first and second moments, beta1 = 0.9, beta2 = 0.999,
eps = 1e-8, no weight decay), with plain SGD (theta <- theta - lr * grad) as the other
choice.  Everything is float64 numpy.
"""
from __future__ import annotations

import numpy as np

from . import chunks, coverage, sampling, step

SGD, ADAM = 0, 1


def sgd_step(theta, grad, lr):
    """theta - lr * grad."""
    return np.asarray(theta, dtype=np.float64) - lr * np.asarray(grad, dtype=np.float64)


def adam_step(theta, grad, m, v, t, lr=0.003, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update; ``t`` is the 1-based count of this step.  Returns (theta, m, v).

    m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
    theta <- theta - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
    """
    g = np.asarray(grad, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return np.asarray(theta, dtype=np.float64) - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def phase_schedule(n_parts: int, max_active: int):
    """Partitions of phase i = the i-th run of ``max_active`` consecutive partition ids
    (ceil(n_parts / max_active) phases; the last one may be shorter)."""
    return [list(range(lo, min(n_parts, lo + max_active))) for lo in range(0, n_parts, max_active)]


def train_epochs(parts, arch, dims, theta0, xs, ys, masks, n_epochs, max_active, estimator,
                 optimizer=ADAM, lr=0.003, gcn_self_loops=True, dropout=None):
    """The phase-parallel algorithm in full-graph mode (one iteration per phase and epoch).

    ``dropout = dict(rate=, seed=)``: hidden-layer dropout; every partition of a phase draws its
    masks with batch_id = the number of optimizer steps taken so far.

    ``parts`` are the partitions of one graph; ``xs[p]``, ``ys[p]``, ``masks[p]`` their
    features, labels and train masks (mask None = every node).  In every phase the active
    partitions each take one isolated train step at the current theta, their gradients are
    scaled by the coverage factor of ``estimator`` and averaged over the active partitions,
    and one optimizer step follows; theta and the optimizer state carry over to the next
    phase.  Returns (theta, history) where history lists per optimizer step the mean of the
    active partitions' losses.
    """
    theta = np.asarray(theta0, dtype=np.float64).copy()
    m = np.zeros_like(theta)
    v = np.zeros_like(theta)
    t = 0
    history = []
    for _ in range(n_epochs):
        for active in phase_schedule(len(parts), max_active):
            grads, stats = [], []
            for p in active:
                g, st = step.train_step(parts[p], arch, dims, theta, xs[p], ys[p], masks[p],
                                        estimator=estimator, gcn_self_loops=gcn_self_loops,
                                        dropout=None if dropout is None else dict(dropout, batch_id=t))
                grads.append(g)
                stats.append(st)
            G, _ = coverage.aggregate(grads, stats, estimator)
            t += 1
            if optimizer == ADAM:
                theta, m, v = adam_step(theta, G, m, v, t, lr)
            else:
                theta = sgd_step(theta, G, lr)
            history.append(float(np.mean([s["loss"] for s in stats])))
    return theta, history


def _apply(optimizer, theta, G, m, v, t, lr):
    if optimizer == ADAM:
        return adam_step(theta, G, m, v, t, lr)
    return sgd_step(theta, G, lr), m, v


def minibatch_epoch(parts, arch, dims, state, xs, ys, masks, epoch, max_active, estimator, batch_size, fanouts,
                    sampler_seed, optimizer, lr, on_step=None, dropout=None):
    """One epoch of the mini-batch loop.  ``state`` = dict(theta, m, v, t, iteration) is updated in place:
    ``t`` counts optimizer steps, ``iteration`` counts iterations (it is the sampler's batch_id, the same in
    every partition of an iteration, and also the batch_id of the dropout masks when
    ``dropout = dict(rate=, seed=)`` is given).  Returns the mean active loss of every optimizer step;
    ``on_step(stats)`` is called after each one."""
    n_train = [parts[p]["n"] if masks[p] is None else int(np.count_nonzero(masks[p])) for p in range(len(parts))]
    iters = max(1, max(-(-c // batch_size) for c in n_train))
    order = [sampling.epoch_seed_order(parts[p], masks[p], sampler_seed, epoch) for p in range(len(parts))]
    history = []
    for it in range(iters):
        for active in phase_schedule(len(parts), max_active):
            grads, stats = [], []
            for p in active:
                seeds = order[p][it * batch_size:(it + 1) * batch_size]
                if seeds.size == 0:
                    grads.append(np.zeros_like(state["theta"]))
                    stats.append(dict(S=0, sum_ratio=0.0, R=0.0, loss=0.0, nnz_used=0))
                    continue
                mb = dict(seeds=seeds, fanouts=fanouts, sampler_seed=sampler_seed, batch_id=state["iteration"])
                g, st = step.train_step(parts[p], arch, dims, state["theta"], xs[p], ys[p], estimator=estimator, minibatch=mb,
                                        dropout=dropout)
                grads.append(g)
                stats.append(st)
            G, _ = coverage.aggregate(grads, stats, estimator)
            state["t"] += 1
            state["theta"], state["m"], state["v"] = _apply(optimizer, state["theta"], G, state["m"], state["v"],
                                                            state["t"], lr)
            history.append(float(np.mean([s["loss"] for s in stats])))
            if on_step is not None:
                on_step(stats)
        state["iteration"] += 1
    return history


def train_epochs_minibatch(parts, arch, dims, theta0, xs, ys, masks, n_epochs, max_active, estimator, batch_size,
                           fanouts, sampler_seed, optimizer=ADAM, lr=0.003, dropout=None):
    """The phase-parallel algorithm in mini-batch mode.

    Every epoch each partition visits its training nodes once, in the order ``sampling.epoch_seed_order``
    gives, ``batch_size`` seeds per iteration; an epoch has as many iterations as the partition with the
    most training nodes needs, and a partition whose nodes are used up takes part with an empty batch (a
    zero gradient that still counts in the average, as for a partition without loss nodes).  The sampler's
    batch_id is the number of iterations done so far, the same in every partition.  Within an
    iteration the phases run as in ``train_epochs``: the active partitions step at the current theta,
    their gradients are scaled and averaged, one optimizer step follows.  Returns (theta, history).
    """
    theta = np.asarray(theta0, dtype=np.float64).copy()
    state = dict(theta=theta, m=np.zeros_like(theta), v=np.zeros_like(theta), t=0, iteration=0)
    history = []
    for epoch in range(n_epochs):
        history += minibatch_epoch(parts, arch, dims, state, xs, ys, masks, epoch, max_active, estimator, batch_size,
                                   fanouts, sampler_seed, optimizer, lr, dropout=dropout)
    return state["theta"], history


def train_sweeping(src, dst, n_nodes, n_chunks, chunk_seed, arch, dims, theta0, x, y, train_mask, total_epochs,
                   max_active, estimator, optimizer=ADAM, lr=0.003, controller=None, gcn_self_loops=True, dropout=None,
                   minibatch=None):
    """The phase-parallel algorithm over sweeping partitions (chunks + controller).

    The graph (global edge list ``src -> dst``, features ``x[n_nodes, F]``, labels ``y``, optional
    uint8 ``train_mask``) is split once into ``n_chunks`` chunks; worker i trains the partition
    base chunk i + the chunk swept in the current super-epoch, with the training nodes of its
    base chunk as loss nodes.  After every epoch the controller decides whether the next
    super-epoch starts (partitions are then rebuilt from the chunks).  Returns
    (theta, history, switches) with history the mean active loss per optimizer step and
    switches the list of epochs (0-based) after which the partitions were switched.
    ``dropout`` as in ``train_epochs`` (batch_id = optimizer steps taken so far, across super-epochs).
    ``minibatch = dict(batch_size=, fanouts=, sampler_seed=)``: every epoch is a mini-batch epoch
    (``minibatch_epoch``) over the current partitions, the seed order keyed by the global epoch number and
    the iteration count running on across super-epochs.
    """
    ctl = controller if controller is not None else chunks.Controller(total_epochs, n_chunks)
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y)
    tm = np.ones(n_nodes, dtype=np.uint8) if train_mask is None else np.asarray(train_mask, dtype=np.uint8)
    theta = np.asarray(theta0, dtype=np.float64).copy()
    m = np.zeros_like(theta)
    v = np.zeros_like(theta)
    t = 0
    iteration = 0
    history, switches = [], []
    parts = None
    for epoch in range(total_epochs):
        if parts is None:
            parts = [chunks.partition_from_chunks(src, dst, n_nodes, n_chunks, chunk_seed, b, w) for b, w in ctl.pairs()]
            xs = [x[p["l2g"]] for p in parts]
            ys = [y[p["l2g"]] for p in parts]
            masks = [p["base_mask"] & tm[p["l2g"]] for p in parts]
        if minibatch is not None:
            state = dict(theta=theta, m=m, v=v, t=t, iteration=iteration)
            history += minibatch_epoch(parts, arch, dims, state, xs, ys, masks, epoch, max_active, estimator,
                                       minibatch["batch_size"], minibatch["fanouts"], minibatch["sampler_seed"],
                                       optimizer, lr,
                                       on_step=lambda stats: ctl.observe_step([coverage.factor(s, coverage.BATCH_MIN_DIST)
                                                                               for s in stats]),
                                       dropout=dropout)
            theta, m, v, t, iteration = state["theta"], state["m"], state["v"], state["t"], state["iteration"]
        for active in (phase_schedule(len(parts), max_active) if minibatch is None else []):
            grads, stats = [], []
            for p in active:
                g, st = step.train_step(parts[p], arch, dims, theta, xs[p], ys[p], masks[p], estimator=estimator,
                                        gcn_self_loops=gcn_self_loops,
                                        dropout=None if dropout is None else dict(dropout, batch_id=t))
                grads.append(g)
                stats.append(st)
            G, _ = coverage.aggregate(grads, stats, estimator)
            t += 1
            if optimizer == ADAM:
                theta, m, v = adam_step(theta, G, m, v, t, lr)
            else:
                theta = sgd_step(theta, G, lr)
            history.append(float(np.mean([s["loss"] for s in stats])))
            ctl.observe_step([coverage.factor(s, coverage.BATCH_MIN_DIST) for s in stats])
        if ctl.end_epoch():
            switches.append(epoch)
            parts = None
    return theta, history, switches
