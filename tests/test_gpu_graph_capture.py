"""A full-graph train step, the aggregation and the optimizer step allocate nothing, synchronise
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
