"""Pins for oracle.optim: Adam against torch.optim.Adam (a library routine) and against the
closed form of its first step, SGD against its definition on a quadratic with a known fixed
point, the phase schedule by brute force, and the epoch loop against its special cases (one
partition with full coverage = plain gradient descent on the whole graph; a planted-label
problem whose loss must fall)."""
import numpy as np
import pytest
import torch

import synth
from oracle import coverage as cov
from oracle import graph, optim, step


def test_adam_matches_library_adam():
    rng = np.random.default_rng(5)
    theta0 = rng.normal(size=37)
    grads = [rng.normal(size=37) * 10.0 ** rng.integers(-4, 2) for _ in range(6)]
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=0.003, betas=(0.9, 0.999), eps=1e-8)
    theta, m, v = theta0.copy(), np.zeros(37), np.zeros(37)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        theta, m, v = optim.adam_step(theta, g, m, v, t, lr=0.003)
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adam_first_step_closed_form():
    # t = 1: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps): lr * sign(g) for |g| >> eps, 0 for g = 0
    g = np.array([3.0, -0.25, 0.0, 1e-3])
    theta, m, v = optim.adam_step(np.zeros(4), g, np.zeros(4), np.zeros(4), 1, lr=0.01)
    np.testing.assert_allclose(theta, -0.01 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    assert theta[2] == 0.0
    np.testing.assert_allclose(m, 0.1 * g)
    np.testing.assert_allclose(v, 0.001 * g * g)


def test_sgd_converges_to_the_quadratic_minimum():
    a = np.array([1.0, 4.0, 0.5])
    target = np.array([2.0, -1.0, 3.0])
    th = np.zeros(3)
    for _ in range(400):
        th = optim.sgd_step(th, a * (th - target), 0.2)       # gradient of 0.5 * a * (th - target)^2
    np.testing.assert_allclose(th, target, atol=1e-12)
    np.testing.assert_array_equal(optim.sgd_step([1.0, 2.0], [0.5, -1.0], 0.1), [0.95, 2.1])


@pytest.mark.parametrize("P,M", [(1, 1), (4, 1), (4, 2), (5, 2), (8, 3), (3, 8)])
def test_phase_schedule_covers_every_partition_once(P, M):
    ph = optim.phase_schedule(P, M)
    assert len(ph) == -(-P // M)
    assert all(1 <= len(a) <= M for a in ph)
    assert sorted(p for a in ph for p in a) == list(range(P))


def _problem(N=120, E=900, K=1, seed=3):
    s, d = synth.uniform_graph(N, E, seed=seed)
    s, d = s.numpy(), d.numpy()
    parts = [graph.partition(s, d, N, K, 1, p) for p in range(K)]
    x = synth.normal_matrix(N, 6, 11)
    y = synth.planted_labels(x, 3, 12).numpy()
    x = x.double().numpy()
    xs = [x[p["l2g"]] for p in parts]
    ys = [y[p["l2g"]] for p in parts]
    return parts, xs, ys


def test_one_partition_full_coverage_is_plain_gradient_descent():
    parts, xs, ys = _problem(K=1)
    dims = [6, 8, 3]
    theta0 = synth.model_weights("sage", dims, 4).double().numpy()
    for est in (cov.NONE, cov.BATCH_MIN_DIST, cov.SHRINKAGE):
        th, hist = optim.train_epochs(parts, "sage", dims, theta0, xs, ys, [None], 3, 1, est,
                                      optimizer=optim.SGD, lr=0.05)
        ref = theta0.copy()
        for _ in range(3):
            g, _ = step.train_step(parts[0], "sage", dims, ref, xs[0], ys[0])
            ref = ref - 0.05 * g
        np.testing.assert_allclose(th, ref, rtol=1e-13, atol=1e-15)
        assert len(hist) == 3


@pytest.mark.parametrize("opt,lr", [(optim.ADAM, 0.01), (optim.SGD, 0.2)])
@pytest.mark.parametrize("M", [1, 2, 4])
def test_loss_falls_on_planted_labels(opt, lr, M):
    parts, xs, ys = _problem(N=400, E=4000, K=4)
    dims = [6, 16, 3]
    theta0 = synth.model_weights("sage", dims, 4).double().numpy()
    th, hist = optim.train_epochs(parts, "sage", dims, theta0, xs, ys, [None] * 4, 30, M, cov.BATCH_MIN_DIST,
                                  optimizer=opt, lr=lr)
    steps_per_epoch = -(-4 // M)
    assert len(hist) == 30 * steps_per_epoch
    first = np.mean(hist[:steps_per_epoch])
    last = np.mean(hist[-steps_per_epoch:])
    assert last < 0.8 * first, (first, last)
    assert np.isfinite(th).all()


def test_phase_order_state_is_carried():
    # M = K (one phase) and M = 1 (K phases) must differ after one epoch: with M = 1 every
    # partition sees the theta already updated by the partitions before it
    parts, xs, ys = _problem(N=300, E=3000, K=3)
    dims = [6, 5, 3]
    theta0 = synth.model_weights("sage", dims, 4).double().numpy()
    a, ha = optim.train_epochs(parts, "sage", dims, theta0, xs, ys, [None] * 3, 1, 3, cov.NONE, optimizer=optim.SGD, lr=0.1)
    b, hb = optim.train_epochs(parts, "sage", dims, theta0, xs, ys, [None] * 3, 1, 1, cov.NONE, optimizer=optim.SGD, lr=0.1)
    assert len(ha) == 1 and len(hb) == 3
    assert np.abs(a - b).max() > 1e-6
    # M = K: one step with the plain average of the three gradients
    gs = [step.train_step(parts[p], "sage", dims, theta0, xs[p], ys[p])[0] for p in range(3)]
    np.testing.assert_allclose(a, theta0 - 0.1 * sum(gs) / 3, rtol=1e-13, atol=1e-15)


def test_sweeping_with_two_chunks_is_the_whole_graph_with_split_loss_nodes():
    # c = 2: both partitions are chunk 0 + chunk 1 = the whole graph (full coverage); they differ
    # only in their loss nodes (their base chunk).  One phase, one epoch, SGD:
    # theta1 = theta0 - lr * (g(S_0) + g(S_1)) / 2 with g(S) the whole-graph gradient of the mean loss over S.
    from oracle import chunks
    N = 150
    s, d = synth.uniform_graph(N, 1200, seed=8)
    s, d = s.numpy(), d.numpy()
    dims = [5, 7, 3]
    x = synth.normal_matrix(N, 5, 21)
    y = synth.planted_labels(x, 3, 22).numpy()
    x = x.double().numpy()
    theta0 = synth.model_weights("sage", dims, 23).double().numpy()
    for est in (cov.NONE, cov.BATCH_MIN_DIST, cov.SHRINKAGE):
        th, hist, sw = optim.train_sweeping(s, d, N, 2, 4, "sage", dims, theta0, x, y, None, 1, 2, est,
                                            optimizer=optim.SGD, lr=0.1)
        whole = graph.partition(s, d, N, 1, 0, 0)
        ch = chunks.chunk_of(N, 2, 4)
        gs = [step.train_step(whole, "sage", dims, theta0, x, y, (ch == b).astype(np.uint8))[0] for b in (0, 1)]
        np.testing.assert_allclose(th, theta0 - 0.1 * (gs[0] + gs[1]) / 2, rtol=1e-12, atol=1e-14)
        assert sw == [0] and len(hist) == 1


def test_sweeping_switches_and_learns():
    N = 400
    s, d = synth.uniform_graph(N, 4000, seed=8)
    s, d = s.numpy(), d.numpy()
    dims = [6, 12, 3]
    x = synth.normal_matrix(N, 6, 21)
    y = synth.planted_labels(x, 3, 22).numpy()
    theta0 = synth.model_weights("sage", dims, 23).double().numpy()
    th, hist, sw = optim.train_sweeping(s, d, N, 4, 4, "sage", dims, theta0, x.double().numpy(), y, None, 30, 2,
                                        cov.BATCH_MIN_DIST, optimizer=optim.ADAM, lr=0.01)
    assert sw == [9, 19, 29]                       # ceil(30 / 3) = 10 epochs per super-epoch
    assert len(hist) == 30 * 2
    assert np.mean(hist[-4:]) < 0.8 * np.mean(hist[:4])


# ------------------------------------------------------------------ mini-batch epochs
@pytest.mark.parametrize("M", [1, 3])
def test_minibatch_epochs_with_one_full_batch_are_the_full_graph_epochs(M):
    # one batch holding every training node, fanouts covering every row: each iteration is the
    # full-graph step restricted to the training nodes, so the two loops must agree
    parts, xs, ys = _problem(N=200, E=1200, K=3)
    masks = [(np.arange(p["n"]) % 4 != 1).astype(np.uint8) for p in parts]
    dims = [6, 8, 8, 3]
    theta0 = synth.model_weights("sage", dims, 4).double().numpy()
    big = int(max(p["d_local_in"].max() for p in parts)) + 1
    for opt in (optim.SGD, optim.ADAM):
        want, hw = optim.train_epochs(parts, "sage", dims, theta0, xs, ys, masks, 3, M, cov.BATCH_MIN_DIST,
                                      optimizer=opt, lr=0.02)
        got, hg = optim.train_epochs_minibatch(parts, "sage", dims, theta0, xs, ys, masks, 3, M, cov.BATCH_MIN_DIST,
                                               batch_size=10 ** 6, fanouts=(big, big, big), sampler_seed=5,
                                               optimizer=opt, lr=0.02)
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(hg, hw, rtol=1e-10)


def test_minibatch_epochs_visit_every_training_node_once_and_learn():
    parts, xs, ys = _problem(N=500, E=5000, K=3)
    masks = [None, (np.arange(parts[1]["n"]) % 2 == 0).astype(np.uint8), None]
    dims = [6, 16, 3]
    theta0 = synth.model_weights("sage", dims, 4).double().numpy()
    B = 32
    n_train = [parts[0]["n"], int(masks[1].sum()), parts[2]["n"]]
    iters = max(-(-c // B) for c in n_train)
    th, hist = optim.train_epochs_minibatch(parts, "sage", dims, theta0, xs, ys, masks, 6, 2, cov.SHRINKAGE, B,
                                            (5, 5), 9, optimizer=optim.ADAM, lr=0.01)
    assert len(hist) == 6 * iters * 2                       # two phases (2 + 1 partitions) per iteration
    assert np.isfinite(th).all()
    assert np.mean(hist[-2 * iters:]) < 0.9 * np.mean(hist[:2 * iters])
    # the shorter partition runs out of seeds first and then contributes empty batches
    from oracle import sampling
    order = sampling.epoch_seed_order(parts[1], masks[1], 9, 0)
    assert order.size == n_train[1] < max(n_train)


def test_sweeping_minibatch_with_one_full_batch_is_sweeping_full_graph():
    # same reduction as above through the chunk / controller loop: identical theta, losses and switches
    N = 300
    s, d = synth.uniform_graph(N, 2400, seed=8)
    s, d = s.numpy(), d.numpy()
    dims = [6, 10, 3]
    x = synth.normal_matrix(N, 6, 21)
    y = synth.planted_labels(x, 3, 22).numpy()
    tm = (np.arange(N) % 5 != 0).astype(np.uint8)
    theta0 = synth.model_weights("sage", dims, 23).double().numpy()
    big = int(np.bincount(d, minlength=N).max()) + 1
    want = optim.train_sweeping(s, d, N, 3, 4, "sage", dims, theta0, x.double().numpy(), y, tm, 8, 2,
                                cov.BATCH_MIN_DIST, optimizer=optim.ADAM, lr=0.01)
    got = optim.train_sweeping(s, d, N, 3, 4, "sage", dims, theta0, x.double().numpy(), y, tm, 8, 2,
                               cov.BATCH_MIN_DIST, optimizer=optim.ADAM, lr=0.01,
                               minibatch=dict(batch_size=10 ** 6, fanouts=(big, big), sampler_seed=3))
    np.testing.assert_allclose(got[0], want[0], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(got[1], want[1], rtol=1e-10)
    assert got[2] == want[2] and len(want[2]) >= 2
