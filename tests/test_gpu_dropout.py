"""GPU parity of train steps with dropout against the oracle (same counter-based masks on both
sides), the mask statistics seen through the gradient, error paths, and the halo equivalence."""
import numpy as np
import pytest
import torch

import synth
from oracle import graph as ograph
from oracle import step as ostep
from tests._cases import TOL_FP32, assert_step_grads_close, make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"
ARCH = {"sage": 0, "gcn": 1, "gcn_res": 2, "gat": 3}


@pytest.fixture(scope="module")
def g():
    import paper_2602_01872_amd as lib
    lib.load()
    return lib


def _step(g, part, arch, dims, x, y, theta, mask, rate, seed, batch_id, bf16=False, est=0):
    model = g.model_desc(ARCH[arch], dims, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, True)
    opts = g.step_opts(estimator=est, full_graph=True, batch_id=batch_id, dropout_rate=rate, dropout_seed=seed)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None if mask is None else mask.to(DEV), theta.to(DEV), ws,
                     grad, stats)
    torch.cuda.synchronize()
    return grad.cpu().numpy(), g.read_stats(stats)[0]


@pytest.mark.parametrize("arch,dims,bf16,rate", [
    ("sage", [100, 256, 256, 47], False, 0.5),      # aggregate-first, aggregate-first, transform-first
    ("sage", [36, 20, 52, 7], False, 0.3),
    ("sage", [64, 128, 16], True, 0.5),
    ("gcn", [40, 72, 72, 10], False, 0.5),
    ("gcn_res", [24, 40, 40, 40, 6], False, 0.25),
    ("gat", [64, 128, 128, 16], False, 0.5),
    ("gat", [100, 64, 47], False, 0.1),
])
def test_dropout_step_matches_oracle(g, arch, dims, bf16, rate):
    print(f"[case] dropout {arch} dims={dims} bf16={bf16} rate={rate}", flush=True)
    scale, E, K = 13, 150000, 3
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018729)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, 2)
    op = ograph.partition(s.numpy(), d.numpy(), N, K, 1, 2)
    n = part.n
    assert n % 128 != 0
    x, y, theta = make_inputs(n, dims, arch, 21, bf16=bf16)
    mask = synth.train_mask(n, 0.4, 6)
    for batch_id in (0, 3):
        grad, st = _step(g, part, arch, dims, x, y, theta, mask, rate, 0xC0FFEE, batch_id, bf16)

        def oracle_fn(relu_flip=None, near_kink=None):
            return ostep.train_step(op, arch, dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                    train_mask=mask.numpy(), relu_flip=relu_flip, near_kink=near_kink,
                                    dropout=dict(rate=rate, seed=0xC0FFEE, batch_id=batch_id))
        og, ost = assert_step_grads_close(grad, oracle_fn, arch, dims, TOL_FP32)
        assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    # another batch id is another mask, rate 0 is the plain step
    g0, _ = _step(g, part, arch, dims, x, y, theta, mask, rate, 0xC0FFEE, 0, bf16)
    assert np.abs(g0 - grad).max() > 1e-3 * np.abs(g0).max()
    plain, _ = _step(g, part, arch, dims, x, y, theta, mask, 0.0, 0xC0FFEE, 0, bf16)
    want, _ = ostep.train_step(op, arch, dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                               train_mask=mask.numpy())
    assert np.abs(plain - want).max() <= 5 * TOL_FP32 * np.abs(want).max()


def test_dropout_is_reproducible_and_rejects_bad_options(g):
    print("[case] dropout determinism / errors", flush=True)
    dims = [32, 48, 8]
    s, d = synth.uniform_graph(3000, 30000, seed=3)
    part = g.grp_partition(s.to(DEV), d.to(DEV), 3000, 2, 1, 0)
    x, y, theta = make_inputs(part.n, dims, "sage", 5)
    a, _ = _step(g, part, "sage", dims, x, y, theta, None, 0.5, 9, 1)
    b, _ = _step(g, part, "sage", dims, x, y, theta, None, 0.5, 9, 1)
    assert np.array_equal(a, b)
    model = g.model_desc(0, dims, g.DTYPE_FP32, True)
    for bad in (1.0, -0.25, float("nan")):
        with pytest.raises(g.GrappaError):
            g.grp_step_workspace_bytes(part, model, g.step_opts(full_graph=True, dropout_rate=bad))


@pytest.mark.parametrize("arch", ["sage", "gat"])
def test_dropout_masks_follow_global_ids_across_halo_partitions(g, arch):
    print(f"[case] dropout halo equivalence {arch}", flush=True)
    N, E, K, dims = 6000, 50000, 3, [24, 40, 12]
    s, d = synth.uniform_graph(N, E, seed=12)
    x = synth.normal_matrix(N, dims[0], 13)
    y = synth.labels(N, dims[-1], 14)
    theta = synth.model_weights(arch, dims, 15)
    whole = g.grp_partition(s.to(DEV), d.to(DEV), N, 1, 0, 0)
    own = ograph.owner(N, K, 5)
    p = 1
    halo = g.grp_partition_halo(s.to(DEV), d.to(DEV), N, K, 5, p, 2)
    l2g = torch.from_numpy(halo.array("l2g"))
    gh, sh = _step(g, halo, arch, dims, x[l2g], y[l2g], theta, torch.from_numpy(halo.base_mask()), 0.5, 31, 2)
    gw, sw = _step(g, whole, arch, dims, x, y, theta, torch.from_numpy((own == p).astype(np.uint8)), 0.5, 31, 2)
    assert np.abs(gh - gw).max() <= TOL_FP32 * np.abs(gw).max()
    assert abs(float(sh["loss"]) - float(sw["loss"])) <= TOL_FP32 * abs(float(sw["loss"]))


def test_phase_parallel_loop_with_dropout_matches_oracle(g):
    """Two epochs of the phase-parallel loop (K = 4, M = 2, SGD) with dropout 0.5: the masks change
    with every optimizer step on both sides in the same way."""
    from oracle import coverage as ocov
    from oracle import optim as ooptim
    print("[case] phase-parallel loop with dropout", flush=True)
    N, E, K, M = 2000, 20000, 4, 2
    s, d = synth.uniform_graph(N, E, seed=77)
    dims = [16, 32, 5]
    x = synth.normal_matrix(N, dims[0], 78)
    y = synth.planted_labels(x, dims[-1], 79)
    theta0 = synth.model_weights("sage", dims, 80)
    oparts = [ograph.partition(s.numpy(), d.numpy(), N, K, 1, p) for p in range(K)]
    oxs = [x.double().numpy()[p["l2g"]] for p in oparts]
    oys = [y.numpy()[p["l2g"]] for p in oparts]
    parts = [g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, p) for p in range(K)]
    xs = [x.to(DEV)[torch.from_numpy(p["l2g"]).to(DEV)].contiguous() for p in oparts]
    ys = [y.to(DEV)[torch.from_numpy(p["l2g"]).to(DEV)].contiguous() for p in oparts]
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    lr = 0.05
    tr = g.PhaseParallelTrainer(parts, model, xs, ys, [None] * K, theta0.to(DEV), g.EST_BATCH_MIN_DIST, M,
                                g.optimizer_desc(g.OPT_SGD, lr=lr), dropout_rate=0.5, dropout_seed=123)
    for _ in range(2):
        tr.run_epoch()
    want, hist = ooptim.train_epochs(oparts, "sage", dims, theta0.double().numpy(), oxs, oys, [None] * K, 2, M,
                                     ocov.BATCH_MIN_DIST, optimizer=ooptim.SGD, lr=lr, dropout=dict(rate=0.5, seed=123))
    got = tr.theta.cpu().double().numpy()
    np.testing.assert_allclose(tr.losses(), hist, rtol=2e-4)
    assert np.abs(got - want).max() <= TOL_FP32 * np.abs(want).max()
    plain, _ = ooptim.train_epochs(oparts, "sage", dims, theta0.double().numpy(), oxs, oys, [None] * K, 2, M,
                                   ocov.BATCH_MIN_DIST, optimizer=ooptim.SGD, lr=lr)
    assert np.abs(plain - want).max() > 1e-3 * np.abs(want).max()
    for p in parts:
        p.destroy()


@pytest.mark.parametrize("dims,fanouts,bf16", [([32, 48, 40, 6], (5, 4, 3), False), ([64, 128, 16], (10, 64), True)])
def test_minibatch_dropout_matches_oracle(g, dims, fanouts, bf16):
    """Mini-batch steps with dropout: a block row is dropped as the node it stands for."""
    print(f"[case] mini-batch dropout dims={dims} fanouts={fanouts} bf16={bf16}", flush=True)
    scale, E, K = 13, 250000, 2
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018733)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, 0)
    op = ograph.partition(s.numpy(), d.numpy(), N, K, 1, 0)
    n = part.n
    x, y, theta = make_inputs(n, dims, "sage", 23, bf16=bf16)
    seeds = np.sort(np.random.default_rng(3).choice(n, 300, replace=False)).astype(np.int32)
    model = g.model_desc(0, dims, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, True)
    for batch in (0, 9):
        seeds_dev = torch.from_numpy(seeds).to(DEV)
        opts = g.step_opts(estimator=1, full_graph=False, seeds=seeds_dev, fanouts=fanouts, sampler_seed=5, batch_id=batch,
                           dropout_rate=0.5, dropout_seed=808)
        P = g.grp_param_count(model)
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
        grad = torch.full((P,), float("nan"), device=DEV)
        stats = g.new_stats(1)
        g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grad, stats)
        torch.cuda.synchronize()
        mb = dict(seeds=seeds, fanouts=fanouts, sampler_seed=5, batch_id=batch)

        def oracle_fn(relu_flip=None, near_kink=None, mb=mb, batch=batch):
            return ostep.train_step(op, "sage", dims, theta.double().numpy(), x.double().numpy(), y.numpy(), estimator=1,
                                    minibatch=mb, relu_flip=relu_flip, near_kink=near_kink,
                                    dropout=dict(rate=0.5, seed=808, batch_id=batch))
        og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, "sage", dims, TOL_FP32)
        st = g.read_stats(stats)[0]
        assert int(st["nnz_used"]) == ost["nnz_used"]
        assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    plain = ostep.train_step(op, "sage", dims, theta.double().numpy(), x.double().numpy(), y.numpy(), estimator=1, minibatch=mb)[0]
    assert np.abs(plain - og).max() > 1e-3 * np.abs(og).max()
