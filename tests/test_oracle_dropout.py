"""Pins for oracle.dropout and the dropout branch of the model oracles: the generator against
SplitMix64's published first outputs and a pure-Python restatement of the counter layout, the
keep frequency, a dense textbook forward pass with the mask applied by hand, central finite
differences with the masks held fixed, rate 0 = no dropout, and independence of the partition
(a k-hop halo step with dropout equals the whole-graph step on the owned nodes)."""
import numpy as np
import pytest

import synth
from oracle import dropout, gat, gnn, graph, step

M64 = (1 << 64) - 1


def _mix_py(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def test_mix_reproduces_the_published_splitmix64_stream():
    # first three outputs of SplitMix64 seeded with 0 (reference test vector of the generator)
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    got = [int(dropout._mix(np.uint64((i * 0x9E3779B97F4A7C15) & M64))) for i in (1, 2, 3)]
    assert got == want


def test_mask_matches_python_integer_arithmetic():
    seed, batch, layer, width, rate = 0xDEADBEEFCAFEF00D, 7, 2, 5, 0.3
    gids = np.array([0, 1, 17, 2**40 + 3, 2**62], dtype=np.int64)
    got = dropout.keep_mask(seed, batch, layer, gids, width, rate)
    g = 0x9E3779B97F4A7C15
    key = _mix_py((seed + (batch * 16 + layer + 1) * g) & M64)
    thr = int(np.floor(float(np.float32(rate)) * 2**24))
    for i, v in enumerate(gids.tolist()):
        for f in range(width):
            bits = _mix_py((key + ((v * width + f + 1) & M64) * g) & M64) >> 40
            assert bool(got[i, f]) == (bits >= thr)


@pytest.mark.parametrize("rate", [0.1, 0.5, 0.9])
def test_keep_frequency_and_scale(rate):
    m = dropout.keep_mask(3, 0, 0, np.arange(4000), 64, rate)
    assert abs(m.mean() - (1 - rate)) < 4 * np.sqrt(rate * (1 - rate) / m.size) + 1e-6
    assert abs(dropout.scale(rate) - 1 / (1 - float(np.float32(rate)))) < 1e-6
    # other layers, batches and seeds give other masks
    assert (m != dropout.keep_mask(3, 0, 1, np.arange(4000), 64, rate)).any()
    assert (m != dropout.keep_mask(3, 1, 0, np.arange(4000), 64, rate)).any()
    assert (m != dropout.keep_mask(4, 0, 0, np.arange(4000), 64, rate)).any()


def test_rate_limits():
    assert dropout.keep_mask(1, 0, 0, np.arange(50), 8, 0.0).all()
    assert dropout.layer_factors(1, 0, np.arange(5), [3, 4, 2], 0.0) == []
    with pytest.raises(ValueError):
        dropout.threshold(1.0)
    with pytest.raises(ValueError):
        dropout.threshold(-0.1)


def _setup(arch, dims, seed=2, n=16, e=70):
    s, d = synth.uniform_graph(n, e, seed=seed)
    s, d = s.numpy().copy(), d.numpy().copy()
    part = graph.partition(s, d, n, 1, 0, 0)
    x = synth.normal_matrix(n, dims[0], seed).double().numpy()
    y = synth.labels(n, dims[-1], seed).numpy()
    kind = "gat" if arch == "gat" else ("sage" if arch == "sage" else "gcn")
    theta = synth.model_weights(kind, dims, seed).double().numpy()
    return s, d, n, part, x, y, theta


def test_sage_forward_with_mask_applied_by_hand():
    dims = [4, 6, 5, 3]
    s, d, n, part, x, y, theta = _setup("sage", dims)
    drop = dropout.layer_factors(11, 3, part["l2g"], dims, 0.5)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    _, _, logits = gnn.forward_backward("sage", dims, theta, x, [blk] * 3, y, np.ones(n), np.arange(n),
                                        return_logits=True, drop=drop)
    a = np.zeros((n, n))
    for u, v in zip(s.tolist(), d.tolist()):
        a[v, u] += 1
    deg = np.maximum(a.sum(axis=1), 1)
    h = x
    for l, (ws, wn, b) in enumerate(gnn.unpack_params(theta, "sage", dims)):
        z = h @ ws + ((a @ h) / deg[:, None]) @ wn + b
        if l < 2:
            keep = dropout.keep_mask(11, 3, l, part["l2g"], dims[l + 1], 0.5)
            h = np.where(keep, np.maximum(z, 0) * 2.0, 0.0)
        else:
            h = z
    np.testing.assert_allclose(logits, h, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("arch,dims", [("sage", [3, 5, 4, 2]), ("gcn", [3, 5, 2]), ("gcn_res", [3, 4, 4, 4, 2]),
                                       ("gat", [3, 5, 4, 2])])
def test_gradient_with_fixed_masks_matches_finite_differences(arch, dims):
    s, d, n, part, x, y, theta = _setup(arch, dims, seed=4)
    k = len(dims) - 1
    drop = dropout.layer_factors(5, 1, part["l2g"], dims, 0.4)
    assert len(drop) == k - 1 and all(0 < (f > 0).mean() < 1 for f in drop)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    nodes = np.array([0, 2, 3, 7, 11, 15])
    w = np.linspace(0.3, 1.7, n)

    def run(t):
        if arch == "gat":
            return gat.forward_backward(dims, t, x, blk, y, w, nodes, drop=drop)
        return gnn.forward_backward(arch, dims, t, x, [blk] * k, y, w, nodes, True, drop=drop)

    _, g = run(theta)
    h = 1e-6
    fd = np.zeros_like(theta)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        fd[i] = (run(tp)[0] - run(tm)[0]) / (2 * h)
    assert np.abs(g).max() > 1e-3
    np.testing.assert_allclose(g, fd, rtol=5e-6, atol=5e-8)
    # and the masks matter: without them the gradient is another one
    g0 = (gat.forward_backward(dims, theta, x, blk, y, w, nodes) if arch == "gat"
          else gnn.forward_backward(arch, dims, theta, x, [blk] * k, y, w, nodes, True))[1]
    assert np.abs(g - g0).max() > 1e-3


def test_rate_zero_is_no_dropout():
    dims = [4, 6, 3]
    s, d, n, part, x, y, theta = _setup("sage", dims)
    g0, st0 = step.train_step(part, "sage", dims, theta, x, y)
    g1, st1 = step.train_step(part, "sage", dims, theta, x, y, dropout=dict(rate=0.0, seed=9))
    assert np.array_equal(g0, g1) and st0["loss"] == st1["loss"]


def test_minibatch_with_full_fanout_and_dropout_is_the_full_graph_step_on_the_seeds():
    # fanouts above every degree keep all local in-edges, so the sampled blocks span the seeds' whole
    # k-hop neighbourhood; the masks are keyed on global ids, so the mini-batch step with dropout is the
    # full-graph step with dropout whose loss nodes are the seeds
    dims = [5, 7, 6, 3]
    N, E = 120, 500
    s, d = synth.uniform_graph(N, E, seed=14)
    part = graph.partition(s.numpy(), d.numpy(), N, 2, 3, 1)
    n = part["n"]
    x = synth.normal_matrix(n, dims[0], 4).double().numpy()
    y = synth.labels(n, dims[-1], 4).numpy()
    theta = synth.model_weights("sage", dims, 4).double().numpy()
    seeds = np.array([1, 5, 8, 13, 21, 34], dtype=np.int64)
    assert int(part["d_local_in"].max()) < 64
    mask = np.zeros(n, dtype=np.uint8)
    mask[seeds] = 1
    dr = dict(rate=0.5, seed=21, batch_id=6)
    gm, sm = step.train_step(part, "sage", dims, theta, x, y, dropout=dr,
                             minibatch=dict(seeds=seeds, fanouts=(64, 64, 64), sampler_seed=1, batch_id=6))
    gf, sf = step.train_step(part, "sage", dims, theta, x, y, train_mask=mask, dropout=dr)
    np.testing.assert_allclose(gm, gf, rtol=1e-10, atol=1e-13)
    assert abs(sm["loss"] - sf["loss"]) < 1e-12
    g0, _ = step.train_step(part, "sage", dims, theta, x, y, minibatch=dict(seeds=seeds, fanouts=(64, 64, 64), sampler_seed=1, batch_id=6))
    assert np.abs(g0 - gm).max() > 1e-3 * np.abs(g0).max()


@pytest.mark.parametrize("arch", ["sage", "gat"])
def test_masks_follow_the_node_not_the_partition(arch):
    # with k hops of halo nodes a k-layer step is exact on the owned nodes; it stays exact with
    # dropout because a node's mask is keyed on its global id
    N, E, K, dims = 150, 900, 3, [5, 8, 6, 4]
    s, d = synth.uniform_graph(N, E, seed=8)
    s, d = s.numpy(), d.numpy()
    x = synth.normal_matrix(N, dims[0], 8).double().numpy()
    y = synth.labels(N, dims[-1], 8).numpy()
    theta = synth.model_weights(arch, dims, 8).double().numpy()
    whole = graph.partition(s, d, N, 1, 0, 0)
    own = graph.owner(N, K, 5)
    dr = dict(rate=0.5, seed=77, batch_id=4)
    for p in range(K):
        halo = graph.partition_halo(s, d, N, K, 5, p, hops=3)
        gh, sh = step.train_step(halo, arch, dims, theta, x[halo["l2g"]], y[halo["l2g"]],
                                 train_mask=halo["owned_mask"], dropout=dr)
        gw, sw = step.train_step(whole, arch, dims, theta, x, y, train_mask=(own == p), dropout=dr)
        np.testing.assert_allclose(gh, gw, rtol=1e-10, atol=1e-12)
        assert abs(sh["loss"] - sw["loss"]) < 1e-12
