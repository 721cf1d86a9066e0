"""Configuration 5 at its stated size: one share of the trillion-edge run, 2^24 nodes and 2^32 local edges
(int32 indices, int64 offsets), features 64-dim bf16, GraphSAGE-mean 64-128-16.

The share is generated directly as sorted rows (an edge list of it would need 69 GB before any sort) and
adopted by grp_partition_from_csr.  The oracle cannot run at this size, so everything is checked through
what determines it:
  * the transposed structure: colptr must equal the prefix sum of the sources' histogram, every row of it
    must ascend, and the multiset of (source, destination) pairs must be that of the input (a 64-bit hash
    summed over all edges of both structures) - together these fix the canonical CSC bit for bit;
  * the mean aggregation, forward and transposed: a seeded sample of output rows recomputed exactly by the
    oracle from the input rows alone - among them the rows that hold edge offsets 2^31 - 1, 2^31 and
    2^32 - 1, and one row of several hundred chunks - and the column-sum identity over all 2^32 edges;
  * the train step: the integer statistics exactly, and the logits of sampled nodes against the oracle's
    forward pass over their complete two-hop neighbourhoods."""
import numpy as np
import pytest
import torch

import synth
from oracle import gnn as ognn
from tests._cases import TOL_FP32

import time

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED, F = 2602018725, 64
_T0 = time.time()


def _note(msg):
    print(f"[case {time.time() - _T0:7.1f}s] {msg}", flush=True)


def _halves_sum(h):
    """Sum of 64-bit patterns mod 2^64, from two sums that cannot overflow."""
    lo = int((h & 0xFFFFFFFF).sum())
    hi = int(((h >> 32) & 0xFFFFFFFF).sum())
    return (lo + (hi << 32)) & ((1 << 64) - 1)


def _row_of(ptr, pos):
    return torch.searchsorted(ptr, pos, right=True) - 1


def _oracle_rows(ptr_rows, nb_lists, x):
    """Exact mean rows from explicit neighbour lists (fp64, the oracle's scatter)."""
    lens = np.array([len(a) for a in nb_lists], dtype=np.int64)
    esrc_g = np.concatenate(nb_lists) if lens.sum() else np.zeros(0, np.int64)
    nbs, inv = np.unique(esrc_g, return_inverse=True)
    xn = x[torch.from_numpy(nbs).to(DEV)].to(torch.float32).cpu().double().numpy()
    edst = np.repeat(np.arange(len(nb_lists)), lens)
    return ognn._scatter_rows(len(nb_lists), edst, xn[inv]) / np.maximum(lens, 1)[:, None].astype(np.float64)


def test_config5_full_size():
    """2^24 nodes, 2^32 edges."""
    _run(24, 1 << 24, 1 << 32, 1 << 28)


def test_config5_same_checks_at_a_small_scale():
    """The same code path with 2^18 nodes and 2^26 edges (the same edge factor), 16 passes of 2^22 edges."""
    _run(18, 1 << 18, 1 << 26, 1 << 22)


def _run(SCALE, N, E, CH):
    import paper_2602_01872_amd as g
    g.load()
    sh = CH.bit_length() - 1
    _note(f"configuration 5 with {N} nodes: generating {E} edges as sorted rows")
    rowptr, col = synth.rmat_local_csr(SCALE, E, seed=SEED, n_nodes=N, device=DEV, chunk=CH, slice_edges=CH,
                                       progress=lambda done, total: _note(f"generated {done >> sh} of {total >> sh} chunks"))
    deg_in = rowptr[1:] - rowptr[:-1]
    d_global = synth.stand_in_global_degree(deg_in, torch.arange(N, device=DEV), SEED, 255)
    _note("adopting the share")
    g.grp_set_slice_policy(1, 25)          # the reduced-size run takes the sliced schedule too (default: 2^19 nodes and more)
    try:
        part = g.grp_partition_from_csr(rowptr, col, N, d_global_in=d_global, slice_edges=CH)
    finally:
        g.grp_set_slice_policy()
    _note("adopted")
    assert part.n == N and part.nnz == E
    assert part.view.rowptr == rowptr.data_ptr() and part.view.col == col.data_ptr()

    # ---- the transposed structure
    deg_out = torch.zeros(N, dtype=torch.int64, device=DEV)
    for a in range(0, E, CH):
        deg_out += torch.bincount(col[a:a + CH], minlength=N)
    colptr = torch.zeros(N + 1, dtype=torch.int64, device=DEV)
    torch.cumsum(deg_out, 0, out=colptr[1:])
    assert torch.equal(part.device_array("colptr"), colptr)
    assert torch.equal(part.device_array("d_local_in"), deg_in.to(torch.int32))
    assert torch.equal(part.device_array("d_local_out"), deg_out.to(torch.int32))
    assert torch.equal(part.device_array("d_global_in"), d_global)
    assert torch.equal(part.device_array("l2g"), torch.arange(N, device=DEV))
    row = part.device_array("row")
    _note(f"max in-degree {int(deg_in.max())}, max out-degree {int(deg_out.max())}, rows over 512 edges: "
          f"{int((deg_in > 512).sum())} / {int((deg_out > 512).sum())}")

    # rows to recompute exactly: a seeded sample of moderate rows, the rows holding the offsets around 2^31 and
    # the last offset, and a row of several hundred chunks
    def picks(ptr, deg, stream):
        cand = (synth.stream_bits(SEED, stream, torch.arange(4096, dtype=torch.int64)) >> 1) % N
        cand = torch.unique(cand).to(DEV)
        cand = cand[deg[cand] <= 100_000]
        marks = _row_of(ptr, torch.tensor([E // 2 - 1, E // 2, E - 1], dtype=torch.int64, device=DEV))
        big = torch.where(deg <= 300_000, deg, torch.zeros_like(deg)).argmax().reshape(1)     # a row of several hundred chunks
        return torch.unique(torch.cat([cand, marks, big])), marks
    pick_f, marks_f = picks(rowptr, deg_in, 21)
    pick_t, marks_t = picks(colptr, deg_out, 22)
    for ptr, marks in ((rowptr, marks_f), (colptr, marks_t)):
        m = marks.tolist()
        assert any(int(ptr[r]) < E // 2 < int(ptr[r + 1]) for r in m[:2]), "no sampled row straddles the middle offset (2^31 at full size)"
        assert int(ptr[m[2] + 1]) == E

    inv_in = 1.0 / deg_in.clamp(min=1).to(torch.float64)
    inv_out = 1.0 / deg_out.clamp(min=1).to(torch.float64)
    w_fwd = torch.zeros(N, dtype=torch.float64, device=DEV)      # sum over the out-edges u->v of 1/deg_in(v)
    w_bwd = torch.zeros(N, dtype=torch.float64, device=DEV)      # sum over the in-edges u->v of 1/deg_out(u)
    h_csr = h_csc = 0
    t_src, t_dst = [], []                                        # the out-edges of pick_t, from the input rows
    for a in range(0, E, CH):
        b = min(E, a + CH)
        lo = max(a - 1, 0)
        pos = torch.arange(lo, b, dtype=torch.int64, device=DEV)
        dst = _row_of(rowptr, pos[a - lo:])
        src = col[a:b].to(torch.int64)
        h_csr = (h_csr + _halves_sum(synth.stream_bits(SEED, 77, (src << 32) | dst))) & ((1 << 64) - 1)
        # per-node sums as differences of a prefix sum over the pass's edges grouped by node (floating-point
        # atomics on one address per hub edge are far too slow): the destinations of a pass are sorted as they are,
        r0, r1 = int(dst[0]), int(dst[-1])
        cs = torch.zeros(b - a + 1, dtype=torch.float64, device=DEV)
        torch.cumsum(inv_out[src], 0, out=cs[1:])
        cut = (rowptr[r0:r1 + 2] - a).clamp(0, b - a)
        w_bwd[r0:r1 + 1] += cs[cut[1:]] - cs[cut[:-1]]
        del cut
        # the sources are sorted first
        by_src, perm = torch.sort(src)
        torch.cumsum(inv_in[dst[perm]], 0, out=cs[1:])
        del perm
        cut = torch.searchsorted(by_src, torch.arange(N + 1, dtype=torch.int64, device=DEV))
        w_fwd += cs[cut[1:]] - cs[cut[:-1]]
        del cs, cut, by_src
        at = torch.searchsorted(pick_t, src).clamp(max=pick_t.numel() - 1)
        hit = pick_t[at] == src
        t_src.append(src[hit])
        t_dst.append(dst[hit])
        del dst, src, at, hit
        src2 = _row_of(colptr, pos)
        dst2 = row[lo:b].to(torch.int64)
        assert not bool(((dst2[1:] < dst2[:-1]) & (src2[1:] == src2[:-1])).any()), f"a CSC row descends near offset {a}"
        h_csc = (h_csc + _halves_sum(synth.stream_bits(SEED, 77, (src2[a - lo:] << 32) | dst2[a - lo:]))) & ((1 << 64) - 1)
        del src2, dst2, pos
        _note(f"structure pass {b >> sh} of {E >> sh}")
    assert h_csr == h_csc, "the CSC does not hold the multiset of edges of the CSR"
    del row
    t_src, t_dst = torch.cat(t_src), torch.cat(t_dst)

    # ---- mean aggregation, forward and transposed
    x = synth.to_bf16_rne(synth.normal_matrix(N, F, SEED, device=DEV))
    y = torch.empty(N, F, device=DEV)
    for transposed in (False, True):
        y.fill_(float("nan"))
        g.grp_spmm(part, transposed, g.SCALE_MEAN, False, F, x, F, g.DTYPE_BF16, y, F)
        torch.cuda.synchronize()
        if not transposed:
            rows = pick_f
            lists = [col[int(rowptr[v]):int(rowptr[v + 1])].cpu().numpy().astype(np.int64) for v in rows.tolist()]
        else:
            rows = pick_t
            order = torch.argsort(t_src, stable=True)
            ts, td = t_src[order].cpu().numpy(), t_dst[order].cpu().numpy()
            cuts = np.searchsorted(ts, rows.cpu().numpy(), side="left").tolist() + [len(ts)]
            lists = [td[cuts[i]:cuts[i + 1]] for i in range(rows.numel())]
            assert [len(a) for a in lists] == deg_out[rows].tolist()
        want = _oracle_rows(rows, lists, x)
        got = y[rows].cpu().double().numpy()
        err = np.abs(got - want).max() / max(np.abs(want).max(), 1e-30)
        worst = int(np.abs(got - want).max(axis=1).argmax())
        _note(f"transposed={transposed}: {rows.numel()} sampled rows (longest {max(len(a) for a in lists)}, "
              f"{sum(len(a) == 0 for a in lists)} empty) rel err {err:.2e} (largest at row {int(rows[worst])} "
              f"of {len(lists[worst])} edges)")
        assert err <= TOL_FP32
        lhs = y.sum(dim=0, dtype=torch.float64)
        w = w_bwd if transposed else w_fwd
        rhs = torch.zeros(F, dtype=torch.float64, device=DEV)
        for lo in range(0, N, 1 << 20):
            rhs += (w[lo:lo + (1 << 20), None] * x[lo:lo + (1 << 20)].to(torch.float64)).sum(dim=0)
        cerr = float((lhs - rhs).abs().max() / rhs.abs().max())
        _note(f"transposed={transposed}: checksum over all edges rel err {cerr:.2e}")
        assert cerr <= TOL_FP32
        assert not torch.isnan(y).any()
    del y, w_fwd, w_bwd, t_src, t_dst

    # ---- the train step
    dims = [64, 128, 16]
    labels = synth.labels(N, dims[-1], SEED, device=DEV)
    theta = synth.model_weights("sage", dims, SEED, device=DEV)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims, feat_dtype=g.DTYPE_BF16)
    opts = g.step_opts(estimator=g.EST_SHRINKAGE)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    _note(f"train step, workspace {ws.numel() / 1e9:.1f} GB")
    g.grp_train_step(part, model, opts, x, labels, None, theta, ws, grad, stats)
    torch.cuda.synchronize()
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == N and int(st["nnz_used"]) == E
    assert float(st["R"]) == float(int((d_global - deg_in).sum()))               # dropped in-edges: an exact integer
    ratio = torch.where(d_global > 0, deg_in.to(torch.float64) / d_global.clamp(min=1).to(torch.float64),
                        torch.ones(N, dtype=torch.float64, device=DEV))
    assert abs(float(st["sum_ratio"]) - float(ratio.sum())) <= 1e-9 * float(ratio.sum())
    assert np.isfinite(float(st["loss"])) and bool(torch.isfinite(grad).all())

    # logits of a few nodes whose complete two-hop neighbourhood is small enough for the oracle
    lim = min(N, 400_000)
    cand = torch.nonzero((deg_in[:lim] >= 1) & (deg_in[:lim] <= 6)).flatten()
    cpos = torch.cat([torch.arange(int(rowptr[v]), int(rowptr[v + 1]), device=DEV) for v in cand[:3000].tolist()])
    cost = torch.zeros(N, dtype=torch.int64, device=DEV).index_add_(0, _row_of(rowptr, cpos), deg_in[col[cpos].to(torch.int64)])
    cand = cand[:3000]
    cand = cand[cost[cand] <= 200_000][:8]
    assert cand.numel() >= 4, "no sampled node has a small two-hop neighbourhood"
    nb = lambda v: col[int(rowptr[v]):int(rowptr[v + 1])].cpu().numpy().astype(np.int64)
    d1 = cand.cpu().numpy()
    l1 = [nb(v) for v in d1.tolist()]
    src1 = np.concatenate([d1, np.setdiff1d(np.unique(np.concatenate(l1)), d1)])
    l0 = [nb(v) for v in src1.tolist()]
    src0 = np.concatenate([src1, np.setdiff1d(np.unique(np.concatenate(l0)), src1)])

    def block(dst_nodes, lists, src_nodes):
        order = np.argsort(src_nodes, kind="stable")
        esrc = order[np.searchsorted(src_nodes[order], np.concatenate(lists))]
        edst = np.repeat(np.arange(len(dst_nodes)), [len(a) for a in lists])
        return dict(n_dst=len(dst_nodes), n_src=len(src_nodes), esrc=esrc, edst=edst)
    blocks = [block(src1, l0, src0), block(d1, l1, src1)]
    _note(f"oracle forward over {len(d1)} nodes: {len(src1)} one-hop and {len(src0)} two-hop nodes, "
          f"{blocks[0]['esrc'].size} edges")
    xs = x[torch.from_numpy(src0).to(DEV)].to(torch.float32).cpu().double().numpy()
    _, _, logits = ognn.forward_backward("sage", dims, theta.cpu().double().numpy(), xs, blocks,
                                         labels[cand].cpu().numpy(), np.ones(len(d1)), np.arange(len(d1)), return_logits=True)
    rows = np.repeat(d1, dims[-1])
    cols = np.tile(np.arange(dims[-1]), len(d1))
    got = g.read_activation(part, model, opts, ws, 1, rows, cols).reshape(len(d1), dims[-1])
    err = np.abs(got - logits).max() / np.abs(logits).max()
    _note(f"logits of {len(d1)} nodes against the oracle: rel err {err:.2e}")
    assert err <= TOL_FP32
    part.destroy()
