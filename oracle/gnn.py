"""GNN layers, loss and hand-derived gradients in fp64 numpy (oracle; test infrastructure).

What is computed follows the paper's model descriptions (experimental setup, "GNN
Models"): GraphSAGE averages the neighbours' states, combines them with the node's own
previous state and multiplies by a matrix; GCN applies a linear map and averages
neighbours with degree-based weights.  The gradient is that of the mean per-node loss
(the paper's true-gradient equation restricted to the partition's local neighbourhoods,
as its "Isolated Training" paragraph prescribes).

Readings where the paper is silent:
  * SAGE-mean:   m_v = mean_{u in N_v} h_u  (0 for an empty N_v),
                 z_v = h_v W_self + m_v W_neigh + b,  h'_v = ReLU(z_v); the last layer
                 outputs z_v (logits).  N_v is the multiset of in-neighbours present in
                 the block (all local in-edges in full-graph mode, the sampled ones in
                 mini-batch mode).  With edge weights (block key "ew", the general
                 non-uniform neighbour distribution) the mean is the weighted mean
                 m_v = sum_u w_uv h_u / sum_u w_uv over the same multiset.
  * GCN:         z_v = sum_u Ahat[v,u] (h_u W) + b with the symmetric normalisation
                 Ahat[v,u] = (A[v,u] + [u==v]) / sqrt((d_in(v)+1) (d_out(u)+1)) over
                 local degrees; with ``self_loops=False`` the identity is not added and
                 degrees are clamped to at least 1.
  * residual GCN: h^{l+1} = h^l + ReLU(z^l) where the two widths agree (never on the
                 last layer); not in the paper, defined by the workload list.
  * dropout (off unless factors are passed in): the activation of hidden layer l is multiplied
    elementwise by ``drop[l]`` = keep / (1 - rate) before a residual skip is added; see
    ``dropout.py`` for how keep is drawn.
  * the derivative of ReLU is 1 where the pre-activation z > 0 and 0 elsewhere.  A
    pre-activation within rounding distance of 0 makes that decision depend on the
    precision and summation order of whoever computes z, so ``forward_backward`` can list
    the hidden pre-activations with |z| <= guard (``near_kink``) and can be asked to take
    the opposite decision for chosen elements (``relu_flip``) or a given decision (``relu_set``); a
    checker uses them to accept either decision exactly at a kink and nothing else.
  * parameters are one flat vector: layer-major; per layer W_self (GCN: W) row-major
    [Fin x Fout], then W_neigh (SAGE only), then b.
  * loss = (1/|S|) sum_{v in S} w_v (logsumexp(z_v) - z_v[y_v]); S empty -> loss 0 and a
    zero gradient.

A "block" is a bipartite message-passing layer: ``n_src`` input nodes, ``n_dst`` output
nodes which are the first ``n_dst`` input nodes, and edge arrays ``esrc -> edst``.  In
full-graph mode every layer uses the same block with n_src = n_dst = n.
"""
from __future__ import annotations

import numpy as np

ARCHS = ("sage", "gcn", "gcn_res")


def param_count(arch: str, dims) -> int:
    per = 2 if arch == "sage" else 1
    return int(sum(per * dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1)))


def unpack_params(theta, arch: str, dims):
    """Split the flat parameter vector into per-layer (W_self, W_neigh or None, b) in fp64."""
    theta = np.asarray(theta, dtype=np.float64)
    if theta.size != param_count(arch, dims):
        raise ValueError("parameter vector has the wrong length")
    out, off = [], 0
    for l in range(len(dims) - 1):
        fin, fout = dims[l], dims[l + 1]
        ws = theta[off:off + fin * fout].reshape(fin, fout); off += fin * fout
        wn = None
        if arch == "sage":
            wn = theta[off:off + fin * fout].reshape(fin, fout); off += fin * fout
        b = theta[off:off + fout]; off += fout
        out.append((ws, wn, b))
    return out


def pack_grads(grads) -> np.ndarray:
    parts = []
    for (gws, gwn, gb) in grads:
        parts.append(gws.reshape(-1))
        if gwn is not None:
            parts.append(gwn.reshape(-1))
        parts.append(gb.reshape(-1))
    return np.concatenate(parts)


def block_from_csr(rowptr, col, n_src=None, ew=None) -> dict:
    rowptr = np.asarray(rowptr, dtype=np.int64)
    n_dst = rowptr.size - 1
    edst = np.repeat(np.arange(n_dst, dtype=np.int64), np.diff(rowptr))
    blk = dict(n_dst=n_dst, n_src=n_dst if n_src is None else int(n_src),
               esrc=np.asarray(col, dtype=np.int64), edst=edst)
    if ew is not None:
        blk["ew"] = np.asarray(ew, dtype=np.float64)
    return blk


def _scatter_rows(n_out: int, index, rows) -> np.ndarray:
    """out[index[e], :] += rows[e, :] (plain accumulation in edge order)."""
    out = np.zeros((n_out, rows.shape[1]), dtype=np.float64)
    np.add.at(out, index, rows)
    return out


# --------------------------------------------------------------------------- loss

def softmax_xent(logits, labels, node_w, loss_nodes):
    """Weighted mean softmax cross-entropy over ``loss_nodes`` and its logit gradient.

    Returns (loss, dZ) with dZ zero outside ``loss_nodes``.
    """
    z = np.asarray(logits, dtype=np.float64)
    dz = np.zeros_like(z)
    s = np.asarray(loss_nodes, dtype=np.int64)
    if s.size == 0:
        return 0.0, dz
    zs = z[s]
    y = np.asarray(labels, dtype=np.int64)[s]
    w = np.asarray(node_w, dtype=np.float64)[s]
    mx = zs.max(axis=1, keepdims=True)
    ex = np.exp(zs - mx)
    lse = np.log(ex.sum(axis=1)) + mx[:, 0]
    per_node = lse - zs[np.arange(s.size), y]
    loss = float((w * per_node).sum() / s.size)
    p = ex / ex.sum(axis=1, keepdims=True)
    p[np.arange(s.size), y] -= 1.0
    dz[s] = p * (w / s.size)[:, None]
    return loss, dz


# --------------------------------------------------------------------------- layers

def _sage_forward(h, blk, ws, wn, b):
    if "ew" in blk:
        mass = np.bincount(blk["edst"], weights=blk["ew"], minlength=blk["n_dst"])
        inv = np.where(mass > 0, 1.0 / np.where(mass > 0, mass, 1.0), 0.0)
        m = _scatter_rows(blk["n_dst"], blk["edst"], h[blk["esrc"]] * blk["ew"][:, None]) * inv[:, None]
        z = h[:blk["n_dst"]] @ ws + m @ wn + b
        return z, (m, inv)
    deg = np.bincount(blk["edst"], minlength=blk["n_dst"]).astype(np.float64)
    inv = 1.0 / np.maximum(deg, 1.0)
    m = _scatter_rows(blk["n_dst"], blk["edst"], h[blk["esrc"]]) * inv[:, None]
    z = h[:blk["n_dst"]] @ ws + m @ wn + b
    return z, (m, inv)


def _sage_backward(h, blk, ws, wn, saved, dz, need_dh):
    m, inv = saved
    gws = h[:blk["n_dst"]].T @ dz
    gwn = m.T @ dz
    gb = dz.sum(axis=0)
    dh = None
    if need_dh:
        dh = np.zeros_like(h)
        dh[:blk["n_dst"]] += dz @ ws.T
        dm = (dz @ wn.T) * inv[:, None]
        per_edge = dm[blk["edst"]]
        if "ew" in blk:
            per_edge = per_edge * blk["ew"][:, None]
        dh += _scatter_rows(blk["n_src"], blk["esrc"], per_edge)
    return (gws, gwn, gb), dh


def _gcn_coeffs(blk, self_loops):
    if "ew" in blk:
        raise ValueError("edge weights are defined for the GraphSAGE mean aggregator only")
    if blk["n_src"] != blk["n_dst"]:
        raise ValueError("GCN layers are defined on the full local graph only")
    n = blk["n_dst"]
    din = np.bincount(blk["edst"], minlength=n).astype(np.float64)
    dout = np.bincount(blk["esrc"], minlength=n).astype(np.float64)
    if self_loops:
        din, dout = din + 1.0, dout + 1.0
    else:
        din, dout = np.maximum(din, 1.0), np.maximum(dout, 1.0)
    r = 1.0 / np.sqrt(din)       # destination side
    s = 1.0 / np.sqrt(dout)      # source side
    return r, s


def _gcn_forward(h, blk, w, b, self_loops):
    r, s = _gcn_coeffs(blk, self_loops)
    t = h @ w
    ce = r[blk["edst"]] * s[blk["esrc"]]
    z = _scatter_rows(blk["n_dst"], blk["edst"], t[blk["esrc"]] * ce[:, None])
    if self_loops:
        z += t * (r * s)[:, None]
    return z + b, (r, s, ce)


def _gcn_backward(h, blk, w, saved, dz, need_dh, self_loops):
    r, s, ce = saved
    dt = _scatter_rows(blk["n_src"], blk["esrc"], dz[blk["edst"]] * ce[:, None])
    if self_loops:
        dt += dz * (r * s)[:, None]
    gw = h.T @ dt
    gb = dz.sum(axis=0)
    dh = dt @ w.T if need_dh else None
    return (gw, None, gb), dh


def forward_backward(arch, dims, theta, x, blocks, labels, node_w, loss_nodes,
                     gcn_self_loops=True, return_logits=False, relu_flip=None, near_kink=None, drop=None, relu_set=None,
                     keep_z=None):
    """Loss and flat parameter gradient of a k-layer model.

    ``blocks`` has one block per layer (input side first); pass the same block k times for
    full-graph mode.  ``x`` is [n_src of block 0, dims[0]]; ``labels``/``node_w`` are indexed by
    the last block's destination ids, and ``loss_nodes`` lists the destinations in the loss.
    ``relu_flip``: iterable of (layer, row, col) whose ReLU derivative is inverted.
    ``near_kink``: a guard g; the call then also returns the list of (layer, row, col) of
    hidden pre-activations with |z| <= g * rms(z of that layer).
    ``relu_set``: {(layer, row, col): bool} fixes the ReLU derivative decision of the listed elements
    (a checker passes the decisions another implementation took for the ``near_kink`` elements).
    ``drop``: per hidden layer the factor array keep / (1 - rate) of its output ([] or None: no dropout).
    ``keep_z``: a list that receives the pre-activation array of every layer (for checkers that look at
    individual elements).
    """
    if arch not in ARCHS:
        raise ValueError("unknown arch")
    k = len(dims) - 1
    if len(blocks) != k:
        raise ValueError("need one block per layer")
    params = unpack_params(theta, arch, dims)
    h = np.asarray(x, dtype=np.float64)
    hs, saved, zs = [], [], []
    for l in range(k):
        ws, wn, b = params[l]
        blk = blocks[l]
        hs.append(h)
        if arch == "sage":
            z, sv = _sage_forward(h, blk, ws, wn, b)
        else:
            z, sv = _gcn_forward(h, blk, ws, b, gcn_self_loops)
        saved.append(sv)
        zs.append(z)
        if l == k - 1:
            h = z
        else:
            a = np.maximum(z, 0.0)
            if drop:
                a = a * drop[l]
            if arch == "gcn_res" and dims[l] == dims[l + 1]:
                a = h[:blk["n_dst"]] + a
            h = a
    logits = h
    if keep_z is not None:
        keep_z.extend(zs)
    loss, dz = softmax_xent(logits, labels, node_w, loss_nodes)

    grads = [None] * k
    dh_next = None          # gradient w.r.t. the output of layer l (post-activation)
    for l in range(k - 1, -1, -1):
        ws, wn, b = params[l]
        blk = blocks[l]
        skip = None
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
            if arch == "gcn_res" and dims[l] == dims[l + 1]:
                skip = dh_next
        need_dh = l > 0
        if arch == "sage":
            g, dh = _sage_backward(hs[l], blk, ws, wn, saved[l], dzl, need_dh)
        else:
            g, dh = _gcn_backward(hs[l], blk, ws, saved[l], dzl, need_dh, gcn_self_loops)
        if need_dh and skip is not None:
            dh = dh.copy()
            dh[:blk["n_dst"]] += skip
        grads[l] = g
        dh_next = dh
    flat = pack_grads(grads)
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
