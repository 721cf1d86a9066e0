"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This module produces *data only*: graphs (COO edge lists), feature matrices, labels,
model weights and stand-in global degrees.  It contains none of the method's
arithmetic (no partition hash, no layers, no estimators); both implementations
receive the tensors it returns and share nothing else.

Every generator is counter based: element ``i`` of stream ``s`` under seed ``k`` is a
pure function ``mix(k, s, i)`` of integers, evaluated with wrapping 64-bit integer
arithmetic in torch, so the same call gives the same integers on the CPU and on a GPU.
Floating-point outputs (normal deviates) go through ``log``/``cos`` whose last bit may
differ between devices, so a test generates them once and hands the same copy to both
sides.

The graphs stand in for the datasets the paper trains on (its dataset table: OGBN
ArXiv / Products / Papers100M, Reddit and Graph500 R-MAT graphs): only their sizes and
degree skew are reproduced.
"""
from __future__ import annotations

import torch

_M1 = -0x00AE502812AA7333  # 0xff51afd7ed558ccd as a signed 64-bit value
_M2 = -0x3B314601E57A13AD  # 0xc4ceb9fe1a85ec53 as a signed 64-bit value
_G1 = 0x2545F4914F6CDD1D
_G2 = 0x106689D45497FDB5


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor holding uint64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _fmix(x: torch.Tensor) -> torch.Tensor:
    """64-bit finaliser of MurmurHash3 (a public-domain avalanche mixer)."""
    x = x ^ _lsr(x, 33)
    x = x * _M1
    x = x ^ _lsr(x, 33)
    x = x * _M2
    x = x ^ _lsr(x, 33)
    return x


def _wrap64(v: int) -> int:
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def stream_bits(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits (as int64) for each counter in ``idx``."""
    key = _wrap64(seed * _G1 + stream * _G2 + 0x1234567)
    base = torch.full((), key, dtype=torch.int64, device=idx.device)
    return _fmix(_fmix(base + idx * _G1) ^ idx)


def _unit(bits: torch.Tensor) -> torch.Tensor:
    """Map 64 random bits to a float64 in (0, 1)."""
    return (_lsr(bits, 11).to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform_graph(n_nodes: int, n_edges: int, seed: int, device="cpu"):
    """``n_edges`` i.i.d. uniform directed (src, dst) pairs; duplicates and self-loops kept."""
    e = torch.arange(n_edges, dtype=torch.int64, device=device)
    src = _lsr(stream_bits(seed, 1, e), 1) % n_nodes
    dst = _lsr(stream_bits(seed, 2, e), 1) % n_nodes
    return src, dst


def _rmat_range(scale: int, lo: int, hi: int, seed: int, n_nodes: int, a: float = 0.57, b: float = 0.19,
                c: float = 0.19, device="cpu"):
    """Edges number lo .. hi-1 of the R-MAT stream (see rmat_graph)."""
    ta = int(a * 65536)
    tb = int((a + b) * 65536)
    tc = int((a + b + c) * 65536)
    e = torch.arange(lo, hi, dtype=torch.int64, device=device)
    s = torch.zeros_like(e)
    d = torch.zeros_like(e)
    bits = None
    for lvl in range(scale):
        if lvl % 4 == 0:
            bits = stream_bits(seed, 16 + lvl // 4, e)
        r = _lsr(bits, 16 * (lvl % 4)) & 0xFFFF
        sbit = (r >= tb).to(torch.int64)                  # quadrants c, d: src bit set
        dbit = ((r >= ta) & (r < tb) | (r >= tc)).to(torch.int64)  # quadrants b, d
        s = (s << 1) | sbit
        d = (d << 1) | dbit
    scr = _wrap64(seed * _G2 + 99)
    s = _lsr(_fmix(s ^ scr), 1) % n_nodes
    d = _lsr(_fmix(d ^ scr), 1) % n_nodes
    return s, d


def rmat_graph(scale: int, n_edges: int, seed: int, n_nodes: int | None = None,
               a: float = 0.57, b: float = 0.19, c: float = 0.19, device="cpu",
               chunk: int = 1 << 26, progress=None):
    """Graph500-style R-MAT edge list with 2**scale raw ids.

    Each of the ``scale`` recursion levels picks a quadrant with probabilities
    (a, b, c, 1-a-b-c) from 16 fresh random bits.  Raw ids are then scrambled by a
    fixed bijection-free mixer and folded ``mod n_nodes`` (default 2**scale) so that
    hubs are not clustered at small ids.  Duplicates and self-loops are kept.
    Edges are generated ``chunk`` at a time (``progress(done, total)`` is called after each).
    """
    if n_nodes is None:
        n_nodes = 1 << scale
    src_parts, dst_parts = [], []
    for lo in range(0, n_edges, chunk):
        hi = min(n_edges, lo + chunk)
        s, d = _rmat_range(scale, lo, hi, seed, n_nodes, a, b, c, device)
        src_parts.append(s)
        dst_parts.append(d)
        if progress is not None:
            progress(hi, n_edges)
    if len(src_parts) == 1:
        return src_parts[0], dst_parts[0]
    return torch.cat(src_parts), torch.cat(dst_parts)


def rmat_local_csr(scale: int, n_edges: int, seed: int, n_nodes: int | None = None, device="cpu",
                   chunk: int = 1 << 28, slice_edges: int = 1 << 28, progress=None, **rmat):
    """The edges of ``rmat_graph`` (same arguments, same multiset) as rows of in-edges: ``rowptr`` int64
    [n_nodes + 1] and ``col`` int32 [n_edges], row v listing the sources of the edges into v in ascending
    order, duplicates kept.  For shares too large to hold as an edge list next to a sort of it (2**32 edges):
    the edges are generated ``chunk`` at a time and kept only as sorted 64-bit keys (dst << 32 | src), then
    merged one range of destinations of about ``slice_edges`` edges at a time."""
    if n_nodes is None:
        n_nodes = 1 << scale
    sorted_chunks = []
    for lo in range(0, n_edges, chunk):
        hi = min(n_edges, lo + chunk)
        s, d = _rmat_range(scale, lo, hi, seed, n_nodes, device=device, **rmat)
        key = (d << 32) | s
        del s, d
        sorted_chunks.append(torch.sort(key)[0])
        del key
        if progress is not None:
            progress(hi, n_edges)
    col = torch.empty(n_edges, dtype=torch.int32, device=device)
    deg = torch.zeros(n_nodes, dtype=torch.int64, device=device)
    n_slices = max(1, -(-n_edges // slice_edges))
    bounds = [n_nodes * i // n_slices for i in range(n_slices + 1)]
    at = 0
    for i in range(n_slices):
        d0, d1 = bounds[i], bounds[i + 1]
        lim = torch.tensor([d0 << 32, d1 << 32], dtype=torch.int64, device=device)
        pieces = []
        for c in sorted_chunks:
            a, b = torch.searchsorted(c, lim).tolist()
            pieces.append(c[a:b])
        keys = torch.sort(torch.cat(pieces))[0] if len(pieces) > 1 else pieces[0]
        del pieces
        cnt = int(keys.numel())
        col[at:at + cnt] = (keys & 0xFFFFFFFF).to(torch.int32)
        if cnt:
            deg[d0:d1] = torch.bincount((keys >> 32) - d0, minlength=d1 - d0)
        at += cnt
        del keys
    assert at == n_edges
    rowptr = torch.zeros(n_nodes + 1, dtype=torch.int64, device=device)
    torch.cumsum(deg, 0, out=rowptr[1:])
    return rowptr, col


def normal_matrix(rows: int, cols: int, seed: int, stream: int = 3, std: float = 1.0,
                  device="cpu", dtype=torch.float32) -> torch.Tensor:
    """rows x cols matrix of N(0, std^2) deviates (Box-Muller on two counter streams)."""
    i = torch.arange(rows * cols, dtype=torch.int64, device=device)
    u1 = _unit(stream_bits(seed, stream, i))
    u2 = _unit(stream_bits(seed, stream + 1000, i))
    z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(6.283185307179586 * u2)
    return (z * std).to(dtype).reshape(rows, cols)


def labels(n: int, n_classes: int, seed: int, device="cpu") -> torch.Tensor:
    """Uniform random class labels in [0, n_classes) as int32."""
    i = torch.arange(n, dtype=torch.int64, device=device)
    return (_lsr(stream_bits(seed, 5, i), 1) % n_classes).to(torch.int32)


def planted_labels(x: torch.Tensor, n_classes: int, seed: int) -> torch.Tensor:
    """Learnable int32 labels: the arg-max of a seeded random linear map of the features."""
    r = normal_matrix(x.shape[1], n_classes, seed, stream=9, device=x.device, dtype=torch.float32)
    return torch.argmax(x.to(torch.float32) @ r, dim=1).to(torch.int32)


def train_mask(n: int, frac: float, seed: int, device="cpu") -> torch.Tensor:
    """uint8 mask selecting about ``frac`` of the nodes."""
    i = torch.arange(n, dtype=torch.int64, device=device)
    return (_unit(stream_bits(seed, 6, i)) < frac).to(torch.uint8)


def edge_weights(n_edges: int, seed: int, lo: float = 0.25, hi: float = 4.0, device="cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """float32 edge weights, log-uniform in [lo, hi) (a stand-in for similarity / frequency weights)."""
    out = torch.empty(n_edges, dtype=torch.float32, device=device)
    for b in range(0, n_edges, chunk):
        e = torch.arange(b, min(n_edges, b + chunk), dtype=torch.int64, device=device)
        u = _unit(stream_bits(seed, 9, e))
        out[b:b + e.numel()] = (lo * (hi / lo) ** u).to(torch.float32)
    return out


def stand_in_global_degree(d_local: torch.Tensor, gids: torch.Tensor, seed: int,
                           mean_missing_shares: int) -> torch.Tensor:
    """Global in-degree for a directly generated local subgraph.

    ``d_global = d_local + extra`` with ``extra`` uniform in
    ``[0, 2 * mean_missing_shares * max(d_local, 1)]`` so that on average the node
    misses ``mean_missing_shares`` times its local degree (the other partitions'
    shares).  Purely an input: the method only ever reads the two degree arrays.
    """
    dl = d_local.to(torch.int64)
    span = 2 * mean_missing_shares * torch.clamp(dl, min=1) + 1
    extra = _lsr(stream_bits(seed, 7, gids.to(torch.int64)), 1) % span
    return dl + extra


def layer_dims_param_count(arch: str, dims) -> int:
    """Number of floats in the flat parameter vector (layout: per layer W_self, W_neigh, b;
    "gat": per layer W, a_src, a_dst, b)."""
    if arch == "gat":
        return sum(dims[l] * dims[l + 1] + 3 * dims[l + 1] for l in range(len(dims) - 1))
    per = 2 if arch == "sage" else 1
    return sum(per * dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))


def model_weights(arch: str, dims, seed: int, device="cpu") -> torch.Tensor:
    """Flat fp32 parameter vector: weights ~ N(0, 1/Fin), biases ~ N(0, 0.01)."""
    out = []
    per = 2 if arch == "sage" else 1
    for l in range(len(dims) - 1):
        fin, fout = dims[l], dims[l + 1]
        for m in range(per):
            out.append(normal_matrix(fin, fout, seed, stream=100 + 10 * l + m,
                                     std=fin ** -0.5, device=device).reshape(-1))
        if arch == "gat":            # the two attention vectors ~ N(0, 1/Fout)
            for m in (5, 6):
                out.append(normal_matrix(1, fout, seed, stream=100 + 10 * l + m, std=fout ** -0.5,
                                         device=device).reshape(-1))
        out.append(normal_matrix(1, fout, seed, stream=100 + 10 * l + 9, std=0.1,
                                 device=device).reshape(-1))
    return torch.cat(out).contiguous()


def to_bf16_rne(x: torch.Tensor) -> torch.Tensor:
    """Round an fp32 tensor to bfloat16 storage (round to nearest even)."""
    return x.to(torch.bfloat16)
