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
