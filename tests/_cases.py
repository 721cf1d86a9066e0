"""Shared helpers for the GPU parity tests: seeded workloads and the tolerance rule.

Tolerance (per output tensor: each layer's dW and db, the loss, G, each c_p):
    max|a - b| / max(max|b|, 1e-30) <= tol,   tol = 1e-4 (fp32), 2e-2 (bf16-stored features).
A gradient tensor that is zero in exact arithmetic (the oracle returns it at fp64 rounding level, below
1e-12 of the largest gradient entry; e.g. the destination attention vector of a GAT layer whose scores
all fall on one branch of the LeakyReLU) has no scale of its own: it is measured against 1e-2 of the
largest gradient entry instead, i.e. its absolute error must stay below tol * 1e-2 * max|gradient|.
"""
from __future__ import annotations

import numpy as np
import torch

import synth

TOL_FP32 = 1e-4
TOL_BF16 = 2e-2


def rel_err(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if b.size == 0:
        return 0.0
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def split_flat(flat, arch: str, dims):
    """Per-layer named views of a flat parameter/gradient vector (layout only)."""
    out, off = {}, 0
    for l in range(len(dims) - 1):
        fin, fout = dims[l], dims[l + 1]
        out[f"W{l}"] = flat[off:off + fin * fout]; off += fin * fout
        if arch == "sage":
            out[f"Wn{l}"] = flat[off:off + fin * fout]; off += fin * fout
        if arch == "gat":
            out[f"as{l}"] = flat[off:off + fout]; off += fout
            out[f"ad{l}"] = flat[off:off + fout]; off += fout
        out[f"b{l}"] = flat[off:off + fout]; off += fout
    assert off == len(flat)
    return out


def assert_grads_close(got, want, arch, dims, tol):
    g, w = split_flat(np.asarray(got), arch, dims), split_flat(np.asarray(want), arch, dims)
    worst = {}
    for k in w:
        worst[k] = rel_err(g[k], w[k])
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"gradient tensors beyond tol {tol}: {bad} (all: {worst})"


KINK_GUARD = 4e-6      # |z| <= guard * rms(z): fp32 rounding of z can decide ReLU'(z) either way


def grad_errors(got, want, arch, dims):
    want = np.asarray(want, dtype=np.float64)
    g, w = split_flat(np.asarray(got), arch, dims), split_flat(want, arch, dims)
    top = float(np.abs(want).max()) if want.size else 0.0
    out = {}
    for k in w:
        own = float(np.abs(w[k]).max()) if w[k].size else 0.0
        if top > 0.0 and own < 1e-12 * top:         # zero in exact arithmetic: see the module docstring
            out[k] = float(np.abs(np.asarray(g[k], dtype=np.float64) - w[k]).max() / (1e-2 * top))
        else:
            out[k] = rel_err(g[k], w[k])
    return out


def assert_step_grads_close(got, oracle_fn, arch, dims, tol):
    """Compare a gradient with the oracle, accepting either ReLU-derivative decision for the
    hidden pre-activations the oracle finds within KINK_GUARD of zero and nothing else.

    ``oracle_fn(relu_flip=..., near_kink=...)`` returns (grad, stats).  The set of flipped
    decisions is found by least squares on the residual and must come out as 0/1 choices;
    the gradient is then recomputed by the oracle with exactly that set and compared to tol.
    Returns the oracle's (grad, stats) that matched.
    """
    got = np.asarray(got, dtype=np.float64)
    og, ost = oracle_fn(relu_flip=None, near_kink=KINK_GUARD)
    errs = grad_errors(got, og, arch, dims)
    if all(v <= tol for v in errs.values()):
        return og, ost
    near = ost["near_kink"]
    assert 0 < len(near) <= 64, f"beyond tol {tol} with {len(near)} near-kink elements: {errs}"
    D = np.stack([oracle_fn(relu_flip=[e], near_kink=None)[0] - og for e in near], axis=1)
    coef, *_ = np.linalg.lstsq(D, got - og, rcond=None)
    pick = np.rint(coef)
    assert np.all((pick == 0) | (pick == 1)) and np.abs(coef - pick).max() < 0.1, \
        f"residual is not a set of kink decisions: coef={coef}, errs={errs}"
    flips = [e for e, p in zip(near, pick) if p == 1]
    og2, ost2 = oracle_fn(relu_flip=flips, near_kink=None)
    errs2 = grad_errors(got, og2, arch, dims)
    assert all(v <= tol for v in errs2.values()), f"beyond tol {tol} after kink decisions {flips}: {errs2}"
    return og2, ost2


def make_inputs(n, dims, arch, seed, bf16=False, n_classes=None):
    x = synth.normal_matrix(n, dims[0], seed)
    if bf16:
        x = synth.to_bf16_rne(x)
    y = synth.labels(n, dims[-1], seed)
    theta = synth.model_weights(arch if arch in ("sage", "gat") else "gcn", dims, seed)
    return x, y, theta


def assert_blocks_equal(g, part, model, opts, ws, oracle_part, seeds, fanouts, sampler_seed, batch_id):
    """The sampled blocks the step left in its workspace against the oracle's, bit for bit: per layer the
    row pointer, the source index of every edge, the destination nodes and the source list."""
    from oracle import sampling as osampling
    blocks, input_nodes = osampling.sample_blocks(oracle_part, np.asarray(seeds, dtype=np.int64), fanouts, sampler_seed, batch_id)
    k = len(fanouts)
    dst_nodes = np.asarray(seeds, dtype=np.int64)
    for l in range(k - 1, -1, -1):
        got, want = g.read_block(part, model, opts, ws, l), blocks[l]
        assert got["n_dst"] == want["n_dst"] and got["nnz"] == want["edst"].size, (l, got["n_dst"], got["nnz"])
        ptr = np.zeros(want["n_dst"] + 1, dtype=np.int64)
        np.cumsum(np.bincount(want["edst"], minlength=want["n_dst"]), out=ptr[1:])
        assert np.array_equal(got["rowptr"], ptr), f"layer {l}: row pointer"
        assert np.array_equal(got["dst_nodes"].astype(np.int64), dst_nodes), f"layer {l}: destination nodes"
        if l == 0:          # the input layer keeps partition-local ids and has no source list of its own
            assert got["src_nodes"] is None and got["n_src"] == oracle_part["n"]
            assert np.array_equal(got["col"].astype(np.int64), want["src_nodes"][want["esrc"]]), "layer 0: sources"
        else:
            assert got["n_src"] == want["n_src"]
            assert np.array_equal(got["col"].astype(np.int64), want["esrc"]), f"layer {l}: sources"
            assert np.array_equal(got["src_nodes"].astype(np.int64), want["src_nodes"]), f"layer {l}: source list"
        dst_nodes = want["src_nodes"]
    return blocks


def library_relu_decisions(g, part, model, opts, ws, dims, near, zs, factors=None, n_sample=100_000, seed=11):
    """The ReLU-derivative decisions the library took at the oracle's near-kink elements, read from its stored
    activations - after proving that they are legitimate: at every near-kink element the library's stored value
    must lie within KINK_GUARD * rms of the oracle's max(z, 0) (so either decision is within rounding), and on a
    seeded sample of other elements the sign of the stored value must be the oracle's.  ``zs``: the oracle's
    pre-activations per layer; ``factors``: per hidden layer the dropout factor array (stored value =
    max(z, 0) * factor), or None.  Elements dropped by dropout are stored as 0 and need no decision."""
    decisions = {}
    for l in range(len(dims) - 2):
        z = zs[l]
        rms = float(np.sqrt(np.mean(z ** 2)))
        fac = factors[l] if factors else None
        el = [e for e in near if e[0] == l]
        if el:
            rr, cc = np.array([e[1] for e in el]), np.array([e[2] for e in el])
            vals = g.read_activation(part, model, opts, ws, l, rr, cc).astype(np.float64)
            f = fac[rr, cc] if fac is not None else np.ones(len(el))
            want = np.maximum(z[rr, cc], 0.0) * f
            assert np.all(np.abs(vals - want) <= KINK_GUARD * rms * np.maximum(f, 1.0)), \
                f"layer {l}: a stored activation at a near-kink element is not within rounding of the oracle's"
            decisions.update({e: bool(v > 0) for e, v, kept in zip(el, vals, f > 0) if kept})
        idx = torch.arange(n_sample, dtype=torch.int64)
        rr = ((synth.stream_bits(seed, 50 + l, idx) >> 1) % z.shape[0]).numpy()
        cc = ((synth.stream_bits(seed, 60 + l, idx) >> 1) % z.shape[1]).numpy()
        vals = g.read_activation(part, model, opts, ws, l, rr, cc)
        zz = z[rr, cc]
        far = np.abs(zz) > KINK_GUARD * rms
        if fac is not None:
            far &= fac[rr, cc] > 0
        assert np.array_equal(vals[far] > 0, zz[far] > 0), f"layer {l}: a ReLU decision away from the kink differs"
    return decisions
