"""Shared helpers for the GPU parity tests: seeded workloads and the tolerance rule.

Tolerance (per output tensor: each layer's dW and db, the loss, G, each c_p):
    max|a - b| / max(max|b|, 1e-30) <= tol,   tol = 1e-4 (fp32), 2e-2 (bf16-stored features).
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


def make_inputs(n, dims, arch, seed, bf16=False, n_classes=None):
    x = synth.normal_matrix(n, dims[0], seed)
    if bf16:
        x = synth.to_bf16_rne(x)
    y = synth.labels(n, dims[-1], seed)
    theta = synth.model_weights("sage" if arch == "sage" else "gcn", dims, seed)
    return x, y, theta
