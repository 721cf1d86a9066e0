"""Pins for oracle.gnn: textbook dense-adjacency forward passes written with Python
loops / dense matrices, central finite differences for every parameter, and the closed
forms of softmax cross-entropy."""
import math

import numpy as np
import pytest

import synth
from oracle import coverage, gnn, graph, step


def _tiny_graph(n=14, e=60, seed=5):
    s, d = synth.uniform_graph(n, e, seed=seed)
    s, d = s.numpy().copy(), d.numpy().copy()
    # adversarial structure: an isolated node, a self-loop, a duplicated edge, a hub
    keep = (s != 0) & (d != 0)
    s, d = s[keep], d[keep]
    s = np.concatenate([s, [3, 4, 4, 1, 2, 5, 6, 7, 8]])
    d = np.concatenate([d, [3, 9, 9, 2, 2, 2, 2, 2, 2]])
    return s, d, n


def _dense_adj(s, d, n):
    a = [[0.0] * n for _ in range(n)]
    for u, v in zip(s.tolist(), d.tolist()):
        a[v][u] += 1.0                       # row v aggregates from u
    return np.array(a)


def _dense_sage_logits(a, x, params):
    h = x
    k = len(params)
    for l, (ws, wn, b) in enumerate(params):
        n = a.shape[0]
        m = np.zeros_like(h)
        for v in range(n):
            dv = a[v].sum()
            if dv > 0:
                m[v] = (a[v][:, None] * h).sum(axis=0) / dv
        z = h @ ws + m @ wn + b
        h = z if l == k - 1 else np.where(z > 0, z, 0.0)
    return h


def _dense_gcn_logits(a, x, params, self_loops, residual):
    n = a.shape[0]
    at = a + np.eye(n) if self_loops else a.copy()
    din = at.sum(axis=1)
    dout = at.sum(axis=0)
    if not self_loops:
        din, dout = np.maximum(din, 1), np.maximum(dout, 1)
    ahat = at / np.sqrt(np.outer(din, dout))
    h = x
    k = len(params)
    for l, (w, _, b) in enumerate(params):
        z = ahat @ (h @ w) + b
        if l == k - 1:
            h = z
        else:
            a_ = np.where(z > 0, z, 0.0)
            h = h + a_ if (residual and h.shape[1] == a_.shape[1]) else a_
    return h


def _xent(logits, y, w, nodes):
    tot = 0.0
    for v in nodes:
        z = logits[v]
        tot += w[v] * (math.log(sum(math.exp(t - z.max()) for t in z)) + z.max() - z[y[v]])
    return tot / len(nodes)


def _setup(arch, dims, seed=1):
    s, d, n = _tiny_graph()
    part = graph.partition(s, d, n, 1, 0, 0)
    x = synth.normal_matrix(n, dims[0], seed).double().numpy()
    y = synth.labels(n, dims[-1], seed).numpy()
    theta = synth.model_weights("sage" if arch == "sage" else "gcn", dims, seed).double().numpy()
    return s, d, n, part, x, y, theta


@pytest.mark.parametrize("arch,dims,sl", [
    ("sage", [5, 7, 3], True), ("sage", [4, 6, 6, 3], True),
    ("gcn", [5, 7, 3], True), ("gcn", [5, 7, 3], False),
    ("gcn_res", [5, 6, 6, 6, 3], True),
])
def test_forward_matches_dense_textbook(arch, dims, sl):
    s, d, n, part, x, y, theta = _setup(arch, dims)
    a = _dense_adj(s, d, n)
    params = gnn.unpack_params(theta, arch, dims)
    if arch == "sage":
        want = _dense_sage_logits(a, x, params)
    else:
        want = _dense_gcn_logits(a, x, params, sl, arch == "gcn_res")
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    nodes = [1, 2, 3, 9, 11]
    w = np.linspace(0.2, 1.5, n)
    loss, _, logits = gnn.forward_backward(arch, dims, theta, x, [blk] * (len(dims) - 1), y, w,
                                           np.array(nodes), sl, return_logits=True)
    np.testing.assert_allclose(logits, want, rtol=1e-12, atol=1e-12)
    assert abs(loss - _xent(want, y, w, nodes)) < 1e-12


@pytest.mark.parametrize("arch,dims,sl", [
    ("sage", [4, 5, 3], True), ("sage", [3, 4, 4, 2], True),
    ("gcn", [4, 5, 3], True), ("gcn", [4, 5, 3], False),
    ("gcn_res", [4, 5, 5, 5, 3], True),
])
def test_gradient_matches_central_finite_differences(arch, dims, sl):
    s, d, n, part, x, y, theta = _setup(arch, dims, seed=3)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    blocks = [blk] * (len(dims) - 1)
    nodes = np.array([0, 1, 2, 5, 9, 13])
    w = np.linspace(0.1, 2.0, n)

    def f(t):
        return gnn.forward_backward(arch, dims, t, x, blocks, y, w, nodes, sl)[0]

    _, g = gnn.forward_backward(arch, dims, theta, x, blocks, y, w, nodes, sl)
    assert g.shape == theta.shape
    h = 1e-6
    fd = np.zeros_like(theta)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        fd[i] = (f(tp) - f(tm)) / (2 * h)
    assert np.abs(g).max() > 1e-3
    np.testing.assert_allclose(g, fd, rtol=2e-6, atol=2e-8)


def test_param_layout_is_layer_major_self_neigh_bias():
    dims = [2, 3, 2]
    p = gnn.param_count("sage", dims)
    assert p == 2 * 2 * 3 + 3 + 2 * 3 * 2 + 2
    theta = np.arange(p, dtype=np.float64)
    (ws0, wn0, b0), (ws1, wn1, b1) = gnn.unpack_params(theta, "sage", dims)
    assert ws0.tolist() == [[0, 1, 2], [3, 4, 5]]
    assert wn0[0, 0] == 6 and b0.tolist() == [12, 13, 14]
    assert ws1[0, 0] == 15 and wn1[0, 0] == 21 and b1.tolist() == [27, 28]
    assert gnn.param_count("gcn", dims) == 2 * 3 + 3 + 3 * 2 + 2
    g = gnn.pack_grads([(ws0, wn0, b0), (ws1, wn1, b1)])
    assert g.tolist() == theta.tolist()


def test_softmax_xent_closed_forms():
    C, n = 6, 9
    z = np.full((n, C), 0.37)
    y = np.arange(n) % C
    nodes = np.array([0, 2, 3, 7])
    w = np.ones(n)
    loss, dz = gnn.softmax_xent(z, y, w, nodes)
    assert abs(loss - math.log(C)) < 1e-14
    for v in range(n):
        if v in nodes:
            want = np.full(C, 1.0 / C)
            want[y[v]] -= 1.0
            np.testing.assert_allclose(dz[v], want / 4, atol=1e-15)
        else:
            assert (dz[v] == 0).all()
    # weighted rows: each row of dZ sums to zero and scales with w_v
    z2 = synth.normal_matrix(n, C, 4).double().numpy() * 30.0       # large logits: stable
    w2 = np.linspace(0.0, 2.0, n)
    loss2, dz2 = gnn.softmax_xent(z2, y, w2, np.arange(n))
    assert np.isfinite(loss2)
    np.testing.assert_allclose(dz2.sum(axis=1), 0.0, atol=1e-15)
    assert (dz2[0] == 0).all()                                       # w = 0
    # empty S
    assert gnn.softmax_xent(z2, y, w2, np.array([], dtype=int))[0] == 0.0


def test_k1_train_step_is_the_whole_graph_model():
    dims = [5, 6, 4]
    s, d, n, part, x, y, theta = _setup("sage", dims, seed=7)
    g, st = step.train_step(part, "sage", dims, theta, x, y)
    a = _dense_adj(s, d, n)
    logits = _dense_sage_logits(a, x, gnn.unpack_params(theta, "sage", dims))
    assert abs(st["loss"] - _xent(logits, y, np.ones(n), list(range(n)))) < 1e-12
    assert st["S"] == n and st["R"] == 0.0 and abs(st["sum_ratio"] - n) < 1e-12
    assert st["nnz_used"] == len(s)


def test_node_level_estimator_is_weighted_sum_of_per_node_gradients():
    """The node-level estimator weights node v's whole gradient contribution by
    d_local/d_global; check against per-node gradients combined by hand."""
    dims = [4, 5, 3]
    N, K = 60, 3
    s, d = synth.uniform_graph(N, 400, seed=21)
    part = graph.partition(s.numpy(), d.numpy(), N, K, 2, 1)
    n = part["n"]
    x = synth.normal_matrix(n, 4, 2).double().numpy()
    y = synth.labels(n, 3, 2).numpy()
    theta = synth.model_weights("sage", dims, 2).double().numpy()
    g, st = step.train_step(part, "sage", dims, theta, x, y, estimator=coverage.NODE_LEVEL)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    acc = np.zeros_like(g)
    for v in range(n):
        _, gv = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, np.ones(n), np.array([v]))
        dg, dl = part["d_global_in"][v], part["d_local_in"][v]
        acc += (dl / dg if dg > 0 else 1.0) * gv
    np.testing.assert_allclose(g, acc / n, rtol=1e-10, atol=1e-14)


def test_train_mask_selects_loss_nodes():
    dims = [4, 3]
    s, d, n, part, x, y, theta = _setup("gcn", dims, seed=9)
    mask = np.zeros(n, dtype=np.uint8)
    mask[[2, 5, 6]] = 1
    g, st = step.train_step(part, "gcn", dims, theta, x, y, train_mask=mask)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    loss, g2 = gnn.forward_backward("gcn", dims, theta, x, [blk], y, np.ones(n), np.array([2, 5, 6]))
    assert st["S"] == 3 and st["loss"] == loss
    np.testing.assert_array_equal(g, g2)


def test_relu_kink_options_flip_exactly_one_derivative():
    """near_kink lists hidden pre-activations close to 0; relu_flip inverts the derivative of
    one element: the gradient changes by that element's contribution and nothing else."""
    dims = [4, 5, 3]
    s, d, n, part, x, y, theta = _setup("sage", dims, seed=3)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    nodes = np.arange(n)
    w = np.ones(n)
    loss, g0, near = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, near_kink=0.05)
    params = gnn.unpack_params(theta, "sage", dims)
    z0, _ = gnn._sage_forward(x, blk, *params[0])
    rms = np.sqrt((z0 ** 2).mean())
    want = sorted((0, int(r), int(c)) for r, c in zip(*np.nonzero(np.abs(z0) <= 0.05 * rms)))
    assert sorted(near) == want and len(near) > 0
    e = near[0]
    loss1, g1 = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, relu_flip=[e])
    assert loss1 == loss and not np.allclose(g1, g0)
    # flipping twice restores the gradient; flips of one layer add up
    _, g2 = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, relu_flip=[e, e])
    np.testing.assert_array_equal(g2, g0)
    if len(near) > 1:
        f = near[1]
        _, gf = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, relu_flip=[f])
        _, gef = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, relu_flip=[e, f])
        np.testing.assert_allclose(gef - g0, (g1 - g0) + (gf - g0), rtol=1e-9, atol=1e-15)
    # relu_set fixes a decision instead of inverting it: the element's own decision changes nothing,
    # the opposite one is the flip
    own = bool(z0[e[1], e[2]] > 0)
    _, gs = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, relu_set={e: own})
    np.testing.assert_array_equal(gs, g0)
    _, gs = gnn.forward_backward("sage", dims, theta, x, [blk] * 2, y, w, nodes, relu_set={e: not own})
    np.testing.assert_array_equal(gs, g1)
