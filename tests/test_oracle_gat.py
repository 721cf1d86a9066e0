"""Pins for oracle.gat: a dense N x N attention implementation written independently (masked
softmax over an adjacency-count matrix), central finite differences on every parameter, the
zero-attention-vector special case (uniform weights = mean over neighbours and self), and
rows of the attention weights summing to one."""
import numpy as np
import pytest

import synth
from oracle import gat, gnn, graph


def _setup(N=40, E=160, dims=(5, 6, 3), seed=1):
    s, d = synth.uniform_graph(N, E, seed=seed)
    part = graph.partition(s.numpy(), d.numpy(), N, 1, 0, 0)
    blk = gnn.block_from_csr(part["rowptr"], part["col"])
    x = synth.normal_matrix(N, dims[0], seed + 1).double().numpy()
    y = synth.labels(N, dims[-1], seed + 2).numpy()
    rng = np.random.default_rng(seed)
    theta = rng.normal(size=gat.param_count(dims)) * 0.5
    return blk, x, y, theta, s.numpy(), d.numpy()


def _dense_forward(dims, theta, x, src, dst, N):
    cnt = np.zeros((N, N))
    np.add.at(cnt, (dst, src), 1.0)            # cnt[v, u] = multiplicity of u -> v
    cnt += np.eye(N)                           # the self term
    h = x
    params = gat.unpack_params(theta, dims)
    for l, (w, a_s, a_d, b) in enumerate(params):
        t = h @ w
        pre = (t @ a_d)[:, None] + (t @ a_s)[None, :]
        e = np.where(pre > 0, pre, 0.2 * pre)
        e = np.where(cnt > 0, e, -np.inf)
        e = e - e.max(axis=1, keepdims=True)
        num = cnt * np.exp(e)
        alpha = num / num.sum(axis=1, keepdims=True)
        z = alpha @ t + b
        h = z if l == len(params) - 1 else np.maximum(z, 0)
    return h


@pytest.mark.parametrize("dims", [(5, 6, 3), (4, 3), (6, 5, 4, 3)])
def test_forward_matches_dense_attention(dims):
    blk, x, y, theta, s, d = _setup(dims=dims)
    N = blk["n_dst"]
    _, _, logits = gat.forward_backward(dims, theta, x, blk, y, np.ones(N), np.arange(N), return_logits=True)
    np.testing.assert_allclose(logits, _dense_forward(dims, theta, x, s, d, N), rtol=1e-11, atol=1e-12)


def test_gradient_matches_finite_differences():
    dims = (4, 5, 3)
    blk, x, y, theta, s, d = _setup(N=24, E=90, dims=dims, seed=4)
    N = blk["n_dst"]
    w = np.linspace(0.5, 1.5, N)
    nodes = np.arange(0, N, 2)
    loss, grad = gat.forward_backward(dims, theta, x, blk, y, w, nodes)
    h = 1e-6
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        lp = gat.forward_backward(dims, tp, x, blk, y, w, nodes)[0]
        lm = gat.forward_backward(dims, tm, x, blk, y, w, nodes)[0]
        assert abs((lp - lm) / (2 * h) - grad[i]) < 2e-7 * max(1.0, abs(grad[i])), i


def test_zero_attention_vectors_give_the_uniform_mean():
    dims = (5, 4)
    blk, x, y, theta, s, d = _setup(dims=dims)
    N = blk["n_dst"]
    w, a_s, a_d, b = [p.copy() for p in gat.unpack_params(theta, dims)[0]]
    theta0 = np.concatenate([w.reshape(-1), 0 * a_s, 0 * a_d, b])
    _, _, logits = gat.forward_backward(dims, theta0, x, blk, y, np.ones(N), np.arange(N), return_logits=True)
    t = x @ w
    deg = np.bincount(blk["edst"], minlength=N) + 1.0
    want = (gnn._scatter_rows(N, blk["edst"], t[blk["esrc"]]) + t) / deg[:, None] + b
    np.testing.assert_allclose(logits, want, rtol=1e-12, atol=1e-13)


def test_attention_rows_sum_to_one_and_isolated_nodes_keep_themselves():
    dims = (3, 4)
    blk, x, y, theta, s, d = _setup(N=30, E=40, dims=dims, seed=9)
    N = blk["n_dst"]
    w, a_s, a_d, b = gat.unpack_params(theta, dims)[0]
    out, (t, pre_e, pre_s, al_e, al_s) = gat._layer_forward(x, blk["esrc"], blk["edst"], N, w, a_s, a_d, b)
    np.testing.assert_allclose(al_s + np.bincount(blk["edst"], weights=al_e, minlength=N), 1.0, rtol=1e-13)
    iso = np.flatnonzero(np.bincount(blk["edst"], minlength=N) == 0)
    assert iso.size > 0
    np.testing.assert_allclose(out[iso], t[iso] + b, rtol=1e-13)
    assert gat.param_count((3, 4)) == 3 * 4 + 12
