"""Graph attention layers (oracle; test infrastructure).

The third model of the paper's experimental setup: every layer applies a linear map to the
hidden states and combines a node's neighbours' states with learned attention weights.  The
paper only names the model; the layer is the published one (Velickovic et al., "Graph
Attention Networks", their equations 1-4), with these readings:

  * one attention head;
  * a node attends over its in-neighbours in the local subgraph (with multiplicity) and over
    itself (one self term, added analytically; explicit self-loop edges still count as edges),
    so the softmax is never empty;
  * score  e_uv = LeakyReLU_{0.2}(a_src . t_u + a_dst . t_v)  with  t = h W,
    alpha_uv = softmax over u of e_uv,  out_v = sum_u alpha_uv t_u + b,
    h'_v = ReLU(out_v) on hidden layers (the other two models' activation), logits = out_v on
    the last layer;
  * flat parameters, layer-major: W row-major [Fin x Fout], a_src [Fout], a_dst [Fout], b [Fout];
  * full-graph mode only (n_src = n_dst = n).

All arithmetic is float64 numpy; the reverse pass is written out by hand.
"""
from __future__ import annotations

import numpy as np

from .gnn import _scatter_rows, softmax_xent

SLOPE = 0.2


def param_count(dims) -> int:
    return int(sum(dims[l] * dims[l + 1] + 3 * dims[l + 1] for l in range(len(dims) - 1)))


def unpack_params(theta, dims):
    theta = np.asarray(theta, dtype=np.float64)
    if theta.size != param_count(dims):
        raise ValueError("parameter vector has the wrong length")
    out, off = [], 0
    for l in range(len(dims) - 1):
        fin, fout = dims[l], dims[l + 1]
        w = theta[off:off + fin * fout].reshape(fin, fout); off += fin * fout
        a_s = theta[off:off + fout]; off += fout
        a_d = theta[off:off + fout]; off += fout
        b = theta[off:off + fout]; off += fout
        out.append((w, a_s, a_d, b))
    return out


def _layer_forward(h, esrc, edst, n, w, a_s, a_d, b):
    t = h @ w
    p = t @ a_s                      # source-side score part, per node
    q = t @ a_d                      # destination-side score part, per node
    pre_e = p[esrc] + q[edst]        # one per edge
    pre_s = p + q                    # the self term of every node
    e_e = np.where(pre_e > 0, pre_e, SLOPE * pre_e)
    e_s = np.where(pre_s > 0, pre_s, SLOPE * pre_s)
    mx = e_s.copy()
    np.maximum.at(mx, edst, e_e)
    x_e = np.exp(e_e - mx[edst])
    x_s = np.exp(e_s - mx)
    zsum = x_s + np.bincount(edst, weights=x_e, minlength=n)
    al_e = x_e / zsum[edst]
    al_s = x_s / zsum
    out = _scatter_rows(n, edst, t[esrc] * al_e[:, None]) + t * al_s[:, None] + b
    return out, (t, pre_e, pre_s, al_e, al_s)


def _layer_backward(h, esrc, edst, n, w, a_s, a_d, saved, dout, need_dh):
    t, pre_e, pre_s, al_e, al_s = saved
    gb = dout.sum(axis=0)
    dt = _scatter_rows(n, esrc, dout[edst] * al_e[:, None]) + dout * al_s[:, None]
    dal_e = np.einsum("ef,ef->e", dout[edst], t[esrc])
    dal_s = np.einsum("nf,nf->n", dout, t)
    c = al_s * dal_s + np.bincount(edst, weights=al_e * dal_e, minlength=n)      # sum_u alpha dalpha per row
    de_e = al_e * (dal_e - c[edst])
    de_s = al_s * (dal_s - c)
    dpre_e = de_e * np.where(pre_e > 0, 1.0, SLOPE)
    dpre_s = de_s * np.where(pre_s > 0, 1.0, SLOPE)
    dp = dpre_s + np.bincount(esrc, weights=dpre_e, minlength=n)
    dq = dpre_s + np.bincount(edst, weights=dpre_e, minlength=n)
    dt += np.outer(dp, a_s) + np.outer(dq, a_d)
    ga_s = t.T @ dp
    ga_d = t.T @ dq
    gw = h.T @ dt
    dh = dt @ w.T if need_dh else None
    return (gw, ga_s, ga_d, gb), dh


def forward_backward(dims, theta, x, blk, labels, node_w, loss_nodes, return_logits=False,
                     relu_flip=None, near_kink=None, drop=None, relu_set=None, keep_z=None):
    """Loss and flat gradient of a k-layer GAT on the full local graph ``blk`` (n_src = n_dst).

    ``relu_flip`` / ``near_kink`` / ``drop`` as in ``gnn.forward_backward`` (dropout acts on the
    layer outputs only; the attention coefficients are not dropped).
    """
    if blk["n_src"] != blk["n_dst"]:
        raise ValueError("GAT layers are defined on the full local graph only")
    n, esrc, edst = blk["n_dst"], blk["esrc"], blk["edst"]
    k = len(dims) - 1
    params = unpack_params(theta, dims)
    h = np.asarray(x, dtype=np.float64)
    hs, saved, zs = [], [], []
    for l in range(k):
        w, a_s, a_d, b = params[l]
        hs.append(h)
        z, sv = _layer_forward(h, esrc, edst, n, w, a_s, a_d, b)
        saved.append(sv)
        zs.append(z)
        h = z if l == k - 1 else np.maximum(z, 0.0)
        if drop and l < k - 1:
            h = h * drop[l]
    logits = h
    if keep_z is not None:          # for checkers that look at individual pre-activations
        keep_z.extend(zs)
    loss, dz = softmax_xent(logits, labels, node_w, loss_nodes)
    grads = [None] * k
    dh_next = None
    for l in range(k - 1, -1, -1):
        w, a_s, a_d, b = params[l]
        if l == k - 1:
            dzl = dz
        else:
            mask = zs[l] > 0.0
            for (fl, fr, fc) in (relu_flip or ()):
                if fl == l:
                    mask[fr, fc] = not mask[fr, fc]
            for (fl, fr, fc), decision in (relu_set or {}).items():
                if fl == l:
                    mask[fr, fc] = bool(decision)
            dzl = dh_next * mask
            if drop:
                dzl = dzl * drop[l]
        g, dh = _layer_backward(hs[l], esrc, edst, n, w, a_s, a_d, saved[l], dzl, l > 0)
        grads[l] = g
        dh_next = dh
    flat = np.concatenate([np.concatenate([gw.reshape(-1), gas, gad, gb]) for (gw, gas, gad, gb) in grads])
    out = (loss, flat)
    if return_logits:
        out = out + (logits,)
    if near_kink is not None:
        near = []
        for l in range(k - 1):
            rms = float(np.sqrt(np.mean(zs[l] ** 2))) if zs[l].size else 0.0
            rr, cc = np.nonzero(np.abs(zs[l]) <= near_kink * rms)
            near += [(l, int(r), int(c)) for r, c in zip(rr, cc)]
        out = out + (near,)
    return out
