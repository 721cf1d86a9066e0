"""Workload 2 at full size, in the launch configuration bench.py times: partition 0 of 8 of the
2.4 M-node / 62 M-edge R-MAT graph, 3-layer GraphSAGE-mean 100-256-256-47.

The partition arrays must be bit-exact.  The loss, the statistics, the last layer's gradients
and the aggregated update of those tensors do not pass through any ReLU derivative and must
hold 1e-4.  The lower layers contain ~1.5e8 hidden pre-activations, of which a few dozen lie
within fp32 rounding of 0; their derivative decisions cannot be enumerated at this size (see
tests/_cases.py for the exact treatment at small sizes), so those tensors are bounded at 5e-3
and the oracle must report that such elements exist whenever 1e-4 is exceeded."""
import numpy as np
import pytest
import torch

import synth
from oracle import graph as ograph
from oracle import step as ostep
from tests._cases import KINK_GUARD, TOL_FP32, grad_errors

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_workload2_partition0_full_size():
    import paper_2602_01872_amd as g
    g.load()
    print("[case] workload 2 full size", flush=True)
    N, E, K, dims = 2_400_000, 62_000_000, 8, [100, 256, 256, 47]
    seed = 2602018722
    s, d = synth.rmat_graph(22, E, seed=seed, n_nodes=N, device=DEV)
    part = g.grp_partition(s, d, N, K, 1, 0)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)
    del s, d
    assert part.n == op["n"] and part.nnz == op["nnz"]
    for key in ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in"):
        assert np.array_equal(part.array(key), op[key]), key
    l2g = torch.from_numpy(op["l2g"]).to(DEV)
    x = synth.normal_matrix(N, dims[0], seed, device=DEV)[l2g].contiguous()
    y = synth.labels(N, dims[-1], seed, device=DEV)[l2g].contiguous()
    theta = synth.model_weights("sage", dims, seed, device=DEV)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    opts = g.step_opts(estimator=g.EST_SHRINKAGE)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x, y, None, theta, ws, grad, stats)
    torch.cuda.synchronize()
    og, ost = ostep.train_step(op, "sage", dims, theta.cpu().double().numpy(), x.cpu().double().numpy(),
                               y.cpu().numpy(), near_kink=KINK_GUARD)
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == ost["S"] and int(st["nnz_used"]) == ost["nnz_used"] and float(st["R"]) == ost["R"]
    assert abs(float(st["sum_ratio"]) - ost["sum_ratio"]) <= 1e-9 * ost["sum_ratio"]
    assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    errs = grad_errors(grad.cpu().numpy(), og, "sage", dims)
    print("[case] per-tensor errors", {k: f"{v:.2e}" for k, v in errs.items()}, "near-kink", len(ost["near_kink"]), flush=True)
    for k in ("W2", "Wn2", "b2"):
        assert errs[k] <= TOL_FP32, (k, errs[k])
    for k, v in errs.items():
        assert v <= 5e-3, (k, v)
        if v > TOL_FP32:
            assert len(ost["near_kink"]) > 0
