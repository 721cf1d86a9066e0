"""A train step (full-graph or mini-batch), the aggregation and the optimizer step allocate nothing, synchronise
nothing and clear memory with kernels only, so they can be captured in a HIP graph: the replays
(interleaved with eager work and synchronisations) must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

import synth
from tests._cases import make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("arch,dims", [("sage", [64, 64, 8]), ("gcn_res", [32, 48, 48, 6]), ("gat", [24, 40, 5])])
def test_captured_step_replays_match_eager(arch, dims):
    import paper_2602_01872_amd as g
    g.load()
    print(f"[case] graph capture {arch} {dims}", flush=True)
    code = {"sage": g.ARCH_SAGE_MEAN, "gcn_res": g.ARCH_GCN_RESIDUAL, "gat": g.ARCH_GAT}[arch]
    N, E = 2500, 10000                       # small: launch-bound, where a graph pays
    s, d = synth.rmat_graph(12, E, seed=5, n_nodes=N)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, 1, 1, 0)
    x, y, theta0 = make_inputs(N, dims, arch, 3)
    x, y = x.to(DEV), y.to(DEV)
    model = g.model_desc(code, dims)
    opts = g.step_opts(estimator=g.EST_NODE_LEVEL, full_graph=True, dropout_rate=0.25, dropout_seed=7)
    P = g.grp_param_count(model)
    ld = (P + 3) // 4 * 4
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    opt = g.optimizer_desc(g.OPT_SGD, lr=0.05)

    def make_state():
        return dict(theta=theta0.to(DEV).clone(), grads=torch.zeros(1, ld, device=DEV), stats=g.new_stats(1),
                    upd=torch.zeros(P, device=DEV))

    def one_iteration(st):
        g.grp_train_step(part, model, opts, x, y, None, st["theta"], ws, st["grads"][0], st["stats"])
        g.grp_aggregate(st["grads"], ld, st["stats"], 1, P, g.EST_BATCH_MIN_DIST, st["upd"])
        g.grp_optimizer_step(opt, P, 1, st["theta"], st["upd"])

    eager = make_state()
    trail = []
    for _ in range(4):
        one_iteration(eager)
        torch.cuda.synchronize()
        trail.append(eager["theta"].clone())

    cap = make_state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_iteration(cap)                   # warm-up on the capture stream (nothing lazy is left to initialise)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    cap = make_state()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_iteration(cap)
    for i in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(cap["theta"], trail[i]), f"replay {i}"
        junk = torch.randn(1 << 16, device=DEV).sum()     # eager work between the replays
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
    part.destroy()


@pytest.mark.parametrize("capture_on_warm_stream", [False, True])
def test_captured_minibatch_step_replays_match_eager(capture_on_warm_stream):
    """A mini-batch step (isolated sampling, the sampled blocks' layers, reduction, update) waits for the device
    nowhere: the block sizes stay in device memory.  Captured once, it is replayed with new seeds written
    and a new batch id written into the same device buffers; every replay must equal the eager step with those
    seeds and that batch id (given as a host argument) bit for bit, and the sampled blocks must differ from
    replay to replay (the graph holds no sizes of the captured batch)."""
    import paper_2602_01872_amd as g
    g.load()
    print(f"[case] graph capture of a mini-batch step, on the warm stream: {capture_on_warm_stream}", flush=True)
    N, E, dims, fanouts, B = 6000, 90000, [48, 64, 32, 7], (6, 4, 3), 96
    s, d = synth.rmat_graph(13, E, seed=11, n_nodes=N)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, 1, 1, 0)
    x, y, theta0 = make_inputs(N, dims, "sage", 4)
    x, y = x.to(DEV), y.to(DEV)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    P = g.grp_param_count(model)
    ld = (P + 3) // 4 * 4
    opt = g.optimizer_desc(g.OPT_SGD, lr=0.05)
    gen = torch.Generator().manual_seed(5)
    batches = [torch.randperm(N, generator=gen)[:B].to(torch.int32).to(DEV) for _ in range(4)]

    def make_state(batch_id=0, on_device=False):
        st = dict(theta=theta0.to(DEV).clone(), grads=torch.zeros(1, ld, device=DEV), stats=g.new_stats(1),
                  upd=torch.zeros(P, device=DEV), seeds=torch.zeros(B, dtype=torch.int32, device=DEV),
                  bid=torch.full((1,), batch_id, dtype=torch.int64, device=DEV))
        st["opts"] = g.step_opts(estimator=g.EST_SHRINKAGE, full_graph=False, seeds=st["seeds"], fanouts=fanouts,
                                 sampler_seed=3, batch_id=batch_id, dropout_rate=0.25, dropout_seed=7,
                                 batch_id_dev=st["bid"] if on_device else None)
        st["ws"] = torch.empty(g.grp_step_workspace_bytes(part, model, st["opts"]), dtype=torch.uint8, device=DEV)
        return st

    def one_iteration(st):
        g.grp_train_step(part, model, st["opts"], x, y, None, st["theta"], st["ws"], st["grads"][0], st["stats"])
        g.grp_aggregate(st["grads"], ld, st["stats"], 1, P, g.EST_SHRINKAGE, st["upd"])
        g.grp_optimizer_step(opt, P, 1, st["theta"], st["upd"])

    trail, edges = [], []
    theta = theta0.to(DEV).clone()
    for i, b in enumerate(batches):
        eager = make_state(batch_id=9 + i)           # the batch id as a host argument
        eager["theta"] = theta
        eager["seeds"].copy_(b)
        one_iteration(eager)
        torch.cuda.synchronize()
        trail.append(eager["theta"].clone())
        edges.append(int(g.read_stats(eager["stats"])[0]["nnz_used"]))
    assert len(set(edges)) > 1 and min(edges) > 0        # the batches really sample blocks of different sizes

    cap = make_state(batch_id=12345, on_device=True)     # the host value must be ignored
    cap["seeds"].copy_(batches[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_iteration(cap)                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    cap["theta"].copy_(theta0.to(DEV))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side if capture_on_warm_stream else None):
        one_iteration(cap)
    for i, b in enumerate(batches):
        cap["seeds"].copy_(b)
        cap["bid"].fill_(9 + i)
        graph.replay()
        torch.cuda.synchronize()
        assert int(g.read_stats(cap["stats"])[0]["nnz_used"]) == edges[i], f"replay {i}"
        assert torch.equal(cap["theta"], trail[i]), f"replay {i}"
        junk = torch.randn(1 << 16, device=DEV).sum()     # eager work between the replays
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
    part.destroy()
