"""Phase-parallel epoch loop over the C ABI (the paper's phase-parallel algorithm, one GPU).

Sequencing only: every partition step, the scale-and-reduce and the optimizer step are
library calls; the partitions of a phase are independent of each other, so they are processed
in turn on the one GPU or, with ``streams`` > 1, side by side on that many HIP streams (small
partitions leave most of the chip idle); their gradients are kept resident for the reduction.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import torch

from . import binding as g
from .controller import Controller


class PhaseParallelTrainer:
    """Holds theta, the optimizer state and the per-partition buffers across phases.

    ``parts``: list of ``Partition``; ``xs`` / ``ys`` / ``masks``: per-partition device
    tensors (features, int32 labels, uint8 train mask or None).  ``max_active`` = M, the
    number of partitions per phase.  Full-graph mode (one iteration per phase and epoch).
    ``dropout_rate`` / ``dropout_seed``: hidden-layer dropout; the masks of a phase are drawn with
    batch_id = the number of optimizer steps taken so far.
    ``streams``: number of streams (default priority) the steps of a phase are spread over, each with a
    workspace of its own; 1 = everything on the current stream.  The result does not depend on it.
    """

    def __init__(self, parts, model, xs, ys, masks, theta0, estimator, max_active, optimizer=None,
                 dropout_rate=0.0, dropout_seed=0, streams=1):
        self.parts, self.model, self.xs, self.ys, self.masks = parts, model, xs, ys, masks
        self.estimator, self.max_active = estimator, max_active
        self.opt = optimizer if optimizer is not None else g.optimizer_desc()
        dev = theta0.device
        self.P = g.grp_param_count(model)
        self.ld = (self.P + 3) // 4 * 4
        self.theta = theta0.detach().clone().to(torch.float32).contiguous()
        self.m = torch.zeros(self.P, device=dev)
        self.v = torch.zeros(self.P, device=dev)
        self.update = torch.zeros(self.P, device=dev)
        self.opts = g.step_opts(estimator=estimator, full_graph=True, dropout_rate=dropout_rate,
                                dropout_seed=dropout_seed)
        self.grads = torch.zeros(max_active, self.ld, device=dev)
        self.stats = g.new_stats(max_active, device=dev)
        ws_bytes = max(g.grp_step_workspace_bytes(p, model, self.opts) for p in parts)
        n_lanes = max(1, min(int(streams), max_active))
        self.ws = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(n_lanes)]
        self.side = [torch.cuda.Stream(device=dev) for _ in range(n_lanes)] if n_lanes > 1 else []
        self.step_count = 0
        self.history = []          # per optimizer step: device tensor views are copied lazily

    def phases(self):
        K, M = len(self.parts), self.max_active
        return [list(range(lo, min(K, lo + M))) for lo in range(0, K, M)]

    def run_phase(self, active):
        self.opts.batch_id = self.step_count
        main = torch.cuda.current_stream()
        if self.side:                 # the side streams start once theta (and everything before) is ready
            ready = main.record_event()
            for st in self.side:
                st.wait_event(ready)
        for slot, p in enumerate(active):
            lane = slot % len(self.ws)
            g.grp_train_step(self.parts[p], self.model, self.opts, self.xs[p], self.ys[p], self.masks[p],
                             self.theta, self.ws[lane], self.grads[slot],
                             self.stats[slot * g.STATS_BYTES:(slot + 1) * g.STATS_BYTES],
                             stream=self.side[lane] if self.side else None)
        for st in self.side:          # the reduction waits for every step
            main.wait_stream(st)
        g.grp_aggregate(self.grads, self.ld, self.stats, len(active), self.P, self.estimator, self.update)
        self.step_count += 1
        g.grp_optimizer_step(self.opt, self.P, self.step_count, self.theta, self.update, self.m, self.v)
        self.history.append(self.stats[:len(active) * g.STATS_BYTES].clone())

    def run_epoch(self):
        for active in self.phases():
            self.run_phase(active)

    def losses(self):
        """Mean loss of the active partitions for every optimizer step so far (host floats)."""
        return [float(g.read_stats(h)["loss"].mean()) for h in self.history]


class MiniBatchTrainer:
    """The phase-parallel loop in mini-batch mode (GraphSAGE): every epoch each partition visits its
    training nodes once in the order ``grp_epoch_seeds`` gives, ``batch_size`` seeds per iteration; an epoch
    has as many iterations as the partition with the most training nodes needs, and a partition whose
    nodes are used up takes part with a zero gradient that still counts in the average.  The sampler's
    batch_id is the number of iterations done so far (``iteration``).  Within an iteration the phases run as
    in ``PhaseParallelTrainer``.  Sequencing only: the seed order, sampling, steps, reduction and update
    are library calls.
    ``lanes``: the steps of a phase are independent, and a mini-batch step is a chain of ~60 small launches
    that leaves most of the chip idle; with ``lanes`` > 1 that many host threads each queue their share of
    the phase's steps on a stream (default priority) with a workspace of their own, so the steps overlap
    on the GPU.  The result does not depend on it.
    ``graphs``: the step of every partition is captured once in a HIP graph (a full batch; the seeds and the
    batch id are read from device buffers that are rewritten before each replay), so an iteration costs the
    host three launches per partition instead of ~60: one thread then keeps ``lanes`` streams busy.  Batches
    shorter than ``batch_size`` (the last of an epoch) run uncaptured.  Same bits as without.
    """

    def __init__(self, parts, model, xs, ys, masks, theta0, estimator, max_active, batch_size, fanouts,
                 sampler_seed, optimizer=None, dropout_rate=0.0, dropout_seed=0, lanes=1, graphs=False):
        self.dropout_rate, self.dropout_seed = dropout_rate, dropout_seed
        self.parts, self.model, self.xs, self.ys, self.masks = parts, model, xs, ys, masks
        self.estimator, self.max_active = estimator, max_active
        self.batch_size, self.fanouts, self.sampler_seed = int(batch_size), tuple(fanouts), sampler_seed
        self.opt = optimizer if optimizer is not None else g.optimizer_desc()
        dev = theta0.device
        self.P = g.grp_param_count(model)
        self.ld = (self.P + 3) // 4 * 4
        self.theta = theta0.detach().clone().to(torch.float32).contiguous()
        self.m = torch.zeros(self.P, device=dev)
        self.v = torch.zeros(self.P, device=dev)
        self.update = torch.zeros(self.P, device=dev)
        self.grads = torch.zeros(max_active, self.ld, device=dev)
        self.stats = g.new_stats(max_active, device=dev)
        self.seeds = [torch.zeros(max(p.n, 1), dtype=torch.int32, device=dev) for p in parts]
        self.n_train = [g.grp_epoch_seeds(p, mk, sampler_seed, 0, sd) for p, mk, sd in zip(parts, masks, self.seeds)]
        self.iters = max(1, max(-(-c // self.batch_size) for c in self.n_train))
        probe = g.step_opts(estimator=estimator, full_graph=False, seeds=self.seeds[0][:1], fanouts=self.fanouts)
        ws_bytes = 0
        for p, sd, c in zip(parts, self.seeds, self.n_train):       # the workspace is sized from the seed count alone
            probe.n_seeds = max(1, min(self.batch_size, c))
            ws_bytes = max(ws_bytes, g.grp_step_workspace_bytes(p, model, probe))
        n_lanes = max(1, min(int(lanes), max_active))
        self.ws = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(n_lanes)]
        self.graphs = bool(graphs)
        self.side = [torch.cuda.Stream(device=dev) for _ in range(n_lanes)] if (n_lanes > 1 or self.graphs) else []
        self.pool = ThreadPoolExecutor(max_workers=n_lanes) if (n_lanes > 1 and not self.graphs) else None
        self.bid_dev = torch.zeros(1, dtype=torch.int64, device=dev)          # the batch id of the captured steps
        self.batch_seeds = [torch.zeros(self.batch_size, dtype=torch.int32, device=dev) for _ in parts] if self.graphs else []
        self.captured = {}                                                     # partition -> its step's graph
        self.step_count = 0
        self.epoch = 0
        self.iteration = 0
        self.history = []

    def phases(self):
        K, M = len(self.parts), self.max_active
        return [list(range(lo, min(K, lo + M))) for lo in range(0, K, M)]

    def run_epoch(self):
        B = self.batch_size
        counts = [g.grp_epoch_seeds(p, mk, self.sampler_seed, self.epoch, sd)
                  for p, mk, sd in zip(self.parts, self.masks, self.seeds)]
        assert counts == self.n_train
        def one_step(slot, p, it, lane, stream):
            lo, hi = it * B, min((it + 1) * B, counts[p])
            st = self.stats[slot * g.STATS_BYTES:(slot + 1) * g.STATS_BYTES]
            if hi <= lo:                               # no seeds left: a zero gradient and an empty record
                self.grads[slot].zero_()
                st.zero_()
                return
            opts = g.step_opts(estimator=self.estimator, full_graph=False, seeds=self.seeds[p][lo:hi],
                               fanouts=self.fanouts, sampler_seed=self.sampler_seed, batch_id=self.iteration,
                               dropout_rate=self.dropout_rate, dropout_seed=self.dropout_seed)
            g.grp_train_step(self.parts[p], self.model, opts, self.xs[p], self.ys[p], None, self.theta,
                             self.ws[lane], self.grads[slot], st, stream=stream)

        def lane_job(lane, active, it):                # one host thread: its share of the phase, in order
            with torch.cuda.stream(self.side[lane]):
                for slot, p in enumerate(active):
                    if slot % len(self.side) == lane:
                        one_step(slot, p, it, lane, self.side[lane])

        def graph_step(slot, p, it):                    # replay (capturing at first use) the partition's full-batch step
            lane = slot % len(self.side)
            lo = it * B
            with torch.cuda.stream(self.side[lane]):
                self.batch_seeds[p].copy_(self.seeds[p][lo:lo + B])
                if p not in self.captured:
                    st = self.stats[slot * g.STATS_BYTES:(slot + 1) * g.STATS_BYTES]
                    opts = g.step_opts(estimator=self.estimator, full_graph=False, seeds=self.batch_seeds[p],
                                       fanouts=self.fanouts, sampler_seed=self.sampler_seed, batch_id_dev=self.bid_dev,
                                       dropout_rate=self.dropout_rate, dropout_seed=self.dropout_seed,
                                       flags=g.STEP_ONE_STREAM if len(self.side) > 1 else 0)   # the lanes fill the GPU
                    # once uncaptured on this stream first: nothing lazy (a kernel's first load) is left for the capture
                    g.grp_train_step(self.parts[p], self.model, opts, self.xs[p], self.ys[p], None, self.theta,
                                     self.ws[lane], self.grads[slot], st)
                    graph = torch.cuda.CUDAGraph()
                    torch.cuda.synchronize()
                    with torch.cuda.graph(graph, stream=self.side[lane]):
                        g.grp_train_step(self.parts[p], self.model, opts, self.xs[p], self.ys[p], None, self.theta,
                                         self.ws[lane], self.grads[slot], st)
                    self.captured[p] = (graph, opts)
                self.captured[p][0].replay()

        for it in range(self.iters):
            if self.graphs:
                self.bid_dev.fill_(self.iteration)
            for active in self.phases():
                if self.graphs:
                    main = torch.cuda.current_stream()
                    ready = main.record_event()
                    for sd in self.side:
                        sd.wait_event(ready)
                    for slot, p in enumerate(active):
                        if min((it + 1) * B, counts[p]) - it * B == B:
                            graph_step(slot, p, it)
                        else:
                            lane = slot % len(self.side)
                            with torch.cuda.stream(self.side[lane]):
                                one_step(slot, p, it, lane, self.side[lane])
                    for sd in self.side:
                        main.wait_stream(sd)
                elif self.pool is None:
                    for slot, p in enumerate(active):
                        one_step(slot, p, it, 0, None)
                else:
                    main = torch.cuda.current_stream()
                    ready = main.record_event()        # theta and everything before
                    for sd in self.side:
                        sd.wait_event(ready)
                    for job in [self.pool.submit(lane_job, lane, active, it) for lane in range(len(self.side))]:
                        job.result()
                    for sd in self.side:               # the reduction waits for every step
                        main.wait_stream(sd)
                g.grp_aggregate(self.grads, self.ld, self.stats, len(active), self.P, self.estimator, self.update)
                self.step_count += 1
                g.grp_optimizer_step(self.opt, self.P, self.step_count, self.theta, self.update, self.m, self.v)
                self.history.append(self.stats[:len(active) * g.STATS_BYTES].clone())
            self.iteration += 1
        self.epoch += 1

    def losses(self):
        return [float(g.read_stats(h)["loss"].mean()) for h in self.history]


class SweepingTrainer:
    """Phase-parallel training over sweeping partitions: the graph is split once into chunks
    (``grp_chunks_build``); every super-epoch each worker's partition base + swept chunk is
    rebuilt on the GPU (``grp_partition_from_chunks``) and its rows of the global feature /
    label / mask tensors are gathered by ``l2g``; the controller decides after each epoch
    whether to switch.  theta and the optimizer state persist across super-epochs.
    ``minibatch = dict(batch_size=, fanouts=, sampler_seed=[, lanes=, graphs=])``: every epoch is a mini-batch epoch
    (``MiniBatchTrainer``) over the current partitions; the epoch number and the iteration count run on
    across super-epochs.
    """

    def __init__(self, src, dst, n_nodes, n_chunks, chunk_seed, model, x, y, train_mask, theta0, estimator,
                 max_active, total_epochs, optimizer=None, controller=None, dropout_rate=0.0, dropout_seed=0,
                 minibatch=None):
        self.minibatch = minibatch
        self.iteration = 0
        self.chunks = g.grp_chunks_build(src, dst, n_nodes, n_chunks, chunk_seed)
        self.dropout_rate, self.dropout_seed = dropout_rate, dropout_seed
        self.model, self.x, self.y, self.train_mask = model, x, y, train_mask
        self.estimator, self.max_active = estimator, max_active
        self.opt = optimizer if optimizer is not None else g.optimizer_desc()
        self.ctl = controller if controller is not None else Controller(total_epochs, n_chunks)
        self.theta = theta0.detach().clone().to(torch.float32).contiguous()
        P = g.grp_param_count(model)
        self.m = torch.zeros(P, device=self.theta.device)
        self.v = torch.zeros(P, device=self.theta.device)
        self.step_count = 0
        self.inner = None
        self.switches = []
        self.epoch = 0
        self._losses = []

    def _build(self):
        parts, xs, ys, masks = [], [], [], []
        for base, swept in self.ctl.pairs():
            part = g.grp_partition_from_chunks(self.chunks, base, swept)
            l2g = torch.from_numpy(part.array("l2g")).to(self.x.device)
            mask = torch.from_numpy(part.base_mask()).to(self.x.device)
            if self.train_mask is not None:            # the training nodes among the base chunk's nodes
                mask = g.grp_gather_rows(self.train_mask, l2g, keep=mask)
            parts.append(part)
            xs.append(g.grp_gather_rows(self.x, l2g))  # this worker's rows of the global tensors
            ys.append(g.grp_gather_rows(self.y, l2g))
            masks.append(mask)
        if self.minibatch is not None:
            mb = self.minibatch
            tr = MiniBatchTrainer(parts, self.model, xs, ys, masks, self.theta, self.estimator, self.max_active,
                                  mb["batch_size"], mb["fanouts"], mb["sampler_seed"], self.opt,
                                  dropout_rate=self.dropout_rate, dropout_seed=self.dropout_seed, lanes=mb.get("lanes", 1),
                                  graphs=mb.get("graphs", False))
            tr.epoch, tr.iteration = self.epoch, self.iteration
        else:
            tr = PhaseParallelTrainer(parts, self.model, xs, ys, masks, self.theta, self.estimator, self.max_active, self.opt,
                                      dropout_rate=self.dropout_rate, dropout_seed=self.dropout_seed)
        tr.theta, tr.m, tr.v, tr.step_count = self.theta, self.m, self.v, self.step_count   # carried state
        return tr

    def run_epoch(self):
        if self.inner is None:
            self.inner = self._build()
        first = len(self.inner.history)
        self.inner.run_epoch()
        self.step_count = self.inner.step_count
        if self.minibatch is not None:
            self.iteration = self.inner.iteration
        for h in self.inner.history[first:]:
            rec = g.read_stats(h)
            self._losses.append(float(rec["loss"].mean()))
            self.ctl.observe_stats(rec)                   # the deficit is derived from the records inside the library
        if self.ctl.end_epoch():
            self.switches.append(self.epoch)
            for p in self.inner.parts:
                p.destroy()
            self.inner = None
        self.epoch += 1

    def losses(self):
        return list(self._losses)
