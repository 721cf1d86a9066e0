"""GPU parity of the sweeping (chunk-based) phase-parallel loop against the oracle loop."""
import numpy as np
import pytest
import torch

import synth
from oracle import coverage as ocov
from oracle import optim as ooptim
from tests._cases import TOL_FP32, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("c,M,masked,drop", [(3, 2, False, 0.0), (4, 4, True, 0.0), (2, 1, False, 0.0), (3, 3, True, 0.5)])
def test_sweeping_loop_matches_oracle(c, M, masked, drop):
    import paper_2602_01872_amd as g
    g.load()
    print(f"[case] sweeping loop c={c} M={M} masked={masked} dropout={drop}", flush=True)
    N, E = 2400, 26000
    s, d = synth.uniform_graph(N, E, seed=91)
    dims = [12, 24, 4]
    x = synth.normal_matrix(N, dims[0], 92)
    y = synth.planted_labels(x, dims[-1], 93)
    tm = synth.train_mask(N, 0.6, 94) if masked else None
    theta0 = synth.model_weights("sage", dims, 95)
    total_epochs = 2 * max(1, c - 1)                # two epochs per super-epoch: the whole cycle is swept
    lr = 0.05
    tr = g.SweepingTrainer(s.to(DEV), d.to(DEV), N, c, 17, g.model_desc(g.ARCH_SAGE_MEAN, dims), x.to(DEV), y.to(DEV),
                           None if tm is None else tm.to(DEV), theta0.to(DEV), g.EST_BATCH_MIN_DIST, M, total_epochs,
                           g.optimizer_desc(g.OPT_SGD, lr=lr), dropout_rate=drop, dropout_seed=41)
    for _ in range(total_epochs):
        tr.run_epoch()
    want, hist, switches = ooptim.train_sweeping(s.numpy(), d.numpy(), N, c, 17, "sage", dims, theta0.double().numpy(),
                                                 x.double().numpy(), y.numpy(), None if tm is None else tm.numpy(),
                                                 total_epochs, M, ocov.BATCH_MIN_DIST, optimizer=ooptim.SGD, lr=lr,
                                                 dropout=dict(rate=drop, seed=41) if drop > 0 else None)
    assert tr.switches == switches
    assert tr.step_count == len(hist)
    np.testing.assert_allclose(tr.losses(), hist, rtol=2e-4)
    assert rel_err(tr.theta.cpu().double().numpy(), want) < TOL_FP32


@pytest.mark.parametrize("c,M,masked,drop", [(3, 2, True, 0.0), (2, 2, False, 0.0), (3, 3, False, 0.5)])
def test_sweeping_minibatch_loop_matches_oracle(c, M, masked, drop):
    """The loop as the paper runs it: sweeping partitions, mini-batches over every worker's training nodes,
    the shrinkage factor per batch; partitions are rebuilt at the switches and the epoch / iteration counts
    that key the seed order and the sampler run on across them."""
    import paper_2602_01872_amd as g
    g.load()
    print(f"[case] sweeping mini-batch loop c={c} M={M} masked={masked} dropout={drop}", flush=True)
    N, E = 1800, 20000
    s, d = synth.rmat_graph(11, E, seed=96, n_nodes=N)
    dims = [10, 20, 4]
    x = synth.normal_matrix(N, dims[0], 97)
    y = synth.planted_labels(x, dims[-1], 98)
    tm = synth.train_mask(N, 0.5, 99) if masked else None
    theta0 = synth.model_weights("sage", dims, 100)
    total_epochs = 2 * max(1, c - 1) if c > 2 else 3
    lr = 0.05
    mb = dict(batch_size=96, fanouts=(5, 4), sampler_seed=13, lanes=2 if drop > 0 else 1)   # lanes: host threads, same bits
    tr = g.SweepingTrainer(s.to(DEV), d.to(DEV), N, c, 17, g.model_desc(g.ARCH_SAGE_MEAN, dims), x.to(DEV), y.to(DEV),
                           None if tm is None else tm.to(DEV), theta0.to(DEV), g.EST_SHRINKAGE, M, total_epochs,
                           g.optimizer_desc(g.OPT_SGD, lr=lr), minibatch=mb, dropout_rate=drop, dropout_seed=43)
    for _ in range(total_epochs):
        tr.run_epoch()
    want, hist, switches = ooptim.train_sweeping(s.numpy(), d.numpy(), N, c, 17, "sage", dims, theta0.double().numpy(),
                                                 x.double().numpy(), y.numpy(), None if tm is None else tm.numpy(),
                                                 total_epochs, M, ocov.SHRINKAGE, optimizer=ooptim.SGD, lr=lr, minibatch=mb,
                                                 dropout=dict(rate=drop, seed=43) if drop > 0 else None)
    assert tr.switches == switches
    assert tr.step_count == len(hist) and tr.step_count > 3 * total_epochs
    np.testing.assert_allclose(tr.losses(), hist, rtol=2e-4)
    assert rel_err(tr.theta.cpu().double().numpy(), want) < TOL_FP32
