"""Full-size cases.  Workload 2, in the launch configuration bench.py times: partition 0 of 8 of the
2.4 M-node / 62 M-edge R-MAT graph, 3-layer 100-256-256-47 models (GraphSAGE-mean, the headline; the
attention model; GraphSAGE on weighted edges with dropout), and the SpMM of workloads 4 and 5.

The partition arrays must be bit-exact; the loss, the statistics and every gradient tensor must hold
1e-4.  The lower layers contain ~1.5e8 hidden pre-activations, of which a few hundred lie within fp32
rounding of 0, where the ReLU derivative can be decided either way: the oracle lists those elements,
the decisions the library took there are read from its stored activations, and the oracle is rerun with
them (and with its own decisions everywhere else)."""
import numpy as np
import pytest
import torch

import synth
from oracle import dropout as odropout
from oracle import graph as ograph
from oracle import step as ostep
from tests._cases import KINK_GUARD, TOL_FP32, assert_blocks_equal, grad_errors, library_relu_decisions

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_workload2_partition0_full_size():
    import paper_2602_01872_amd as g
    g.load()
    print("[case] workload 2 full size", flush=True)
    N, E, K, dims = 2_400_000, 62_000_000, 8, [100, 256, 256, 47]
    seed = 2602018722
    s, d = synth.rmat_graph(22, E, seed=seed, n_nodes=N, device=DEV)
    part = g.grp_partition(s, d, N, K, 1, 0)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)
    del s, d
    assert part.n == op["n"] and part.nnz == op["nnz"]
    for key in ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in"):
        assert np.array_equal(part.array(key), op[key]), key
    l2g = torch.from_numpy(op["l2g"]).to(DEV)
    x = synth.normal_matrix(N, dims[0], seed, device=DEV)[l2g].contiguous()
    y = synth.labels(N, dims[-1], seed, device=DEV)[l2g].contiguous()
    theta = synth.model_weights("sage", dims, seed, device=DEV)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    opts = g.step_opts(estimator=g.EST_SHRINKAGE)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x, y, None, theta, ws, grad, stats)
    torch.cuda.synchronize()
    zs = []
    og, ost = ostep.train_step(op, "sage", dims, theta.cpu().double().numpy(), x.cpu().double().numpy(),
                               y.cpu().numpy(), near_kink=KINK_GUARD, keep_z=zs)
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == ost["S"] and int(st["nnz_used"]) == ost["nnz_used"] and float(st["R"]) == ost["R"]
    assert abs(float(st["sum_ratio"]) - ost["sum_ratio"]) <= 1e-9 * ost["sum_ratio"]
    assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    errs = grad_errors(grad.cpu().numpy(), og, "sage", dims)
    near = ost["near_kink"]
    print("[case] per-tensor errors before the kink decisions are matched", {k: f"{v:.2e}" for k, v in errs.items()},
          "near-kink", len(near), flush=True)
    for k in ("W2", "Wn2", "b2"):                       # the last layer's gradients involve no ReLU decision
        assert errs[k] <= TOL_FP32, (k, errs[k])
    # Hidden pre-activations within rounding distance of 0 (the oracle lists them) may take either
    # ReLU-derivative decision; the oracle is rerun with the decisions the library took there (read
    # from its stored activations) and with its own decisions everywhere else.
    assert len(near) < 5000
    decisions = library_relu_decisions(g, part, model, opts, ws, dims, near, zs)
    del zs
    og2, _ = ostep.train_step(op, "sage", dims, theta.cpu().double().numpy(), x.cpu().double().numpy(),
                              y.cpu().numpy(), relu_set=decisions)
    errs2 = grad_errors(grad.cpu().numpy(), og2, "sage", dims)
    print("[case] per-tensor errors with matched decisions", {k: f"{v:.2e}" for k, v in errs2.items()}, flush=True)
    for k, v in errs2.items():
        assert v <= TOL_FP32, (k, v)


def test_workload2_partition0_full_size_gat():
    """The attention model on the headline workload's partition at full size (the configuration
    `bench.py --workload c2-gat-step` times), gradients against the oracle with the library's
    ReLU decisions at the near-kink elements."""
    import paper_2602_01872_amd as g
    g.load()
    print("[case] workload 2 full size, GAT", flush=True)
    N, E, K, dims = 2_400_000, 62_000_000, 8, [100, 256, 256, 47]
    seed = 2602018722
    s, d = synth.rmat_graph(22, E, seed=seed, n_nodes=N, device=DEV)
    part = g.grp_partition(s, d, N, K, 1, 0)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)      # the oracle's own arrays
    assert part.n == op["n"] and part.nnz == op["nnz"]
    del s, d
    l2g = torch.from_numpy(op["l2g"]).to(DEV)
    x = synth.normal_matrix(N, dims[0], seed, device=DEV)[l2g].contiguous()
    y = synth.labels(N, dims[-1], seed, device=DEV)[l2g].contiguous()
    theta = synth.model_weights("gat", dims, seed, device=DEV)
    model = g.model_desc(g.ARCH_GAT, dims)
    opts = g.step_opts(estimator=g.EST_SHRINKAGE)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x, y, None, theta, ws, grad, stats)
    torch.cuda.synchronize()
    th, xh, yh = theta.cpu().double().numpy(), x.cpu().double().numpy(), y.cpu().numpy()
    print("[case] oracle pass 1 (lists the near-kink elements)", flush=True)
    zs = []
    og, ost = ostep.train_step(op, "gat", dims, th, xh, yh, near_kink=KINK_GUARD, keep_z=zs)
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == ost["S"] and float(st["R"]) == ost["R"]
    assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    near = ost["near_kink"]
    errs = grad_errors(grad.cpu().numpy(), og, "gat", dims)
    print("[case] per-tensor errors before the kink decisions are matched", {k: f"{v:.2e}" for k, v in errs.items()},
          "near-kink", len(near), flush=True)
    assert len(near) < 5000
    decisions = library_relu_decisions(g, part, model, opts, ws, dims, near, zs)
    del zs
    print("[case] oracle pass 2 (the library's decisions at those elements)", flush=True)
    og2, _ = ostep.train_step(op, "gat", dims, th, xh, yh, relu_set=decisions)
    errs2 = grad_errors(grad.cpu().numpy(), og2, "gat", dims)
    print("[case] per-tensor errors with matched decisions", {k: f"{v:.2e}" for k, v in errs2.items()}, flush=True)
    for k, v in errs2.items():
        assert v <= TOL_FP32, (k, v)
    part.destroy()


def test_workload2_partition0_full_size_weighted_with_dropout():
    """Weighted edges and hidden-layer dropout together on the headline workload's partition at full
    size: the weighted partition arrays bit for bit, then the GraphSAGE step against the oracle."""
    import paper_2602_01872_amd as g
    g.load()
    print("[case] workload 2 full size, weighted edges + dropout", flush=True)
    N, E, K, dims = 2_400_000, 62_000_000, 8, [100, 256, 256, 47]
    seed = 2602018722
    s, d = synth.rmat_graph(22, E, seed=seed, n_nodes=N, device=DEV)
    w = synth.edge_weights(E, seed, device=DEV)
    part = g.grp_partition_weighted(s, d, w, N, K, 1, 0)
    print("[case] oracle partition", flush=True)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0, weights=w.cpu().numpy())
    del s, d, w
    for key in ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_global_in"):
        assert np.array_equal(part.array(key), op[key]), key
    got = part.weights()
    for key in ("csr_w", "csc_w", "w_local_in", "w_global_in"):
        assert np.array_equal(got[key], op[key]), key
    l2g = torch.from_numpy(op["l2g"]).to(DEV)
    x = synth.normal_matrix(N, dims[0], seed, device=DEV)[l2g].contiguous()
    y = synth.labels(N, dims[-1], seed, device=DEV)[l2g].contiguous()
    theta = synth.model_weights("sage", dims, seed, device=DEV)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    opts = g.step_opts(estimator=g.EST_NODE_LEVEL, batch_id=5, dropout_rate=0.5, dropout_seed=99)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x, y, None, theta, ws, grad, stats)
    torch.cuda.synchronize()
    th, xh, yh = theta.cpu().double().numpy(), x.cpu().double().numpy(), y.cpu().numpy()
    dr = dict(rate=0.5, seed=99, batch_id=5)
    print("[case] oracle pass 1 (lists the near-kink elements)", flush=True)
    zs = []
    og, ost = ostep.train_step(op, "sage", dims, th, xh, yh, estimator=1, near_kink=KINK_GUARD, dropout=dr, keep_z=zs)
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == ost["S"]
    assert abs(float(st["R"]) - ost["R"]) <= 1e-9 * ost["R"]
    assert abs(float(st["sum_ratio"]) - ost["sum_ratio"]) <= 1e-9 * ost["sum_ratio"]
    assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    # a dropped element is stored as 0 by the library and needs no decision; the others are matched
    near = ost["near_kink"]
    factors = odropout.layer_factors(99, 5, op["l2g"], dims, 0.5)
    decisions = library_relu_decisions(g, part, model, opts, ws, dims, near, zs, factors=factors)
    del zs, factors
    print(f"[case] near-kink {len(near)}, kept by dropout {len(decisions)}; oracle pass 2", flush=True)
    og2, _ = ostep.train_step(op, "sage", dims, th, xh, yh, estimator=1, relu_set=decisions, dropout=dr)
    errs2 = grad_errors(grad.cpu().numpy(), og2, "sage", dims)
    print("[case] per-tensor errors with matched decisions", {k: f"{v:.2e}" for k, v in errs2.items()}, flush=True)
    for k, v in errs2.items():
        assert v <= TOL_FP32, (k, v)
    part.destroy()


def test_workload3_minibatch_full_size():
    """Workload 3 at full size (`bench.py --workload c3-step`): a 7 M-node / 100 M-edge store with hub
    rows of 10^5 in-edges, isolated 3-hop sampling with fanouts (15, 10, 5) from 1024 seeds, bf16
    features.  The library builds its store from the edge list; the oracle samples and trains on the
    same edges generated independently as sorted rows (the two stores must agree bit for bit), and the
    sampled blocks are compared bit for bit before the gradients."""
    import paper_2602_01872_amd as g
    g.load()
    print("[case] workload 3 full size, mini-batch", flush=True)
    scale, n, E, seed, dims, fanouts = 23, 7_000_000, 100_000_000, 2602018720 + 3, [128, 256, 256, 172], (15, 10, 5)
    src, dst = synth.rmat_graph(scale, E, seed=seed, n_nodes=n, device=DEV, chunk=1 << 28)
    d_local = torch.bincount(dst, minlength=n)
    d_global = synth.stand_in_global_degree(d_local, torch.arange(n, device=DEV), seed, 15)
    part = g.grp_partition_from_local_coo(src, dst, n, d_global_in=d_global)
    assert part.n == n and part.nnz == E
    del src, dst
    # the oracle's store is built without the library: the same edges generated as sorted rows
    rowptr, col = synth.rmat_local_csr(scale, E, seed=seed, n_nodes=n, device=DEV, chunk=1 << 26, slice_edges=1 << 26)
    assert torch.equal(rowptr[1:] - rowptr[:-1], d_local) and int(rowptr[-1]) == E
    assert int(d_local.max()) > 50_000                        # hub rows: the sampler's whole-workgroup scan
    assert torch.equal(part.device_array("rowptr"), rowptr) and torch.equal(part.device_array("col"), col)
    op = dict(n=n, nnz=E, l2g=np.arange(n, dtype=np.int64), rowptr=rowptr.cpu().numpy(), col=col.cpu().numpy(),
              d_local_in=d_local.cpu().numpy().astype(np.int32), d_global_in=d_global.cpu().numpy())
    del rowptr, col
    x = synth.to_bf16_rne(synth.normal_matrix(n, dims[0], seed, device=DEV))
    y = synth.labels(n, dims[-1], seed, device=DEV)
    theta = synth.model_weights("sage", dims, seed, device=DEV)
    train = torch.nonzero(synth.train_mask(n, 0.05, seed, device=DEV)).flatten().to(torch.int32)
    seeds = train[:1024].contiguous()
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims, feat_dtype=g.DTYPE_BF16)
    opts = g.step_opts(estimator=g.EST_BATCH_MIN_DIST, full_graph=False, seeds=seeds, fanouts=fanouts, sampler_seed=7,
                       batch_id=0)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x, y, None, theta, ws, grad, stats)
    torch.cuda.synchronize()
    th, yh = theta.cpu().double().numpy(), y.cpu().numpy()
    xh = x.cpu().to(torch.float32).numpy()                    # the oracle widens the rows it gathers
    mb = dict(seeds=seeds.cpu().numpy(), fanouts=fanouts, sampler_seed=7, batch_id=0)
    print("[case] oracle pass 1 (sampling, lists the near-kink elements)", flush=True)
    assert_blocks_equal(g, part, model, opts, ws, op, mb["seeds"], fanouts, 7, 0)
    zs = []
    og, ost = ostep.train_step(op, "sage", dims, th, xh, yh, estimator=2, minibatch=mb, near_kink=KINK_GUARD, keep_z=zs)
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == ost["S"] == 1024
    assert int(st["nnz_used"]) == ost["nnz_used"]             # the sampled edge multiset has the same size
    assert abs(float(st["R"]) - ost["R"]) <= 1e-9 * max(1.0, ost["R"])
    assert abs(float(st["sum_ratio"]) - ost["sum_ratio"]) <= 1e-9 * ost["sum_ratio"]
    assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
    near = ost["near_kink"]
    decisions = library_relu_decisions(g, part, model, opts, ws, dims, near, zs, n_sample=20_000)
    del zs
    print(f"[case] edges used {ost['nnz_used']}, near-kink {len(near)}; oracle pass 2", flush=True)
    og2, _ = ostep.train_step(op, "sage", dims, th, xh, yh, estimator=2, minibatch=mb, relu_set=decisions)
    errs2 = grad_errors(grad.cpu().numpy(), og2, "sage", dims)
    print("[case] per-tensor errors with matched decisions", {k: f"{v:.2e}" for k, v in errs2.items()}, flush=True)
    for k, v in errs2.items():
        assert v <= TOL_FP32, (k, v)
    part.destroy()


def _sampled_rows_and_checksum(g, scale, n, E, seed, F, bf16, n_sample=4096):
    """Mean aggregation (forward over in-edges, transposed over out-edges) of a directly generated
    local subgraph at full size.  The oracle cannot run at this size, so (a) a seeded sample of
    output rows is recomputed exactly (each row needs only its own neighbour list, taken from the
    edge list itself, not from the library's CSR), and (b) the column sums of the whole output are
    checked against the identity  1^T (D^-1 A X) = sum_u (sum_{v: u->v} 1/deg(v)) X[u,:], which
    holds at any size and involves every edge."""
    from oracle import gnn as ognn
    src, dst = synth.rmat_graph(scale, E, seed=seed, n_nodes=n, device=DEV, chunk=1 << 28)
    part = g.grp_partition_from_local_coo(src, dst, n)
    assert part.n == n and part.nnz == E
    x = synth.normal_matrix(n, F, seed, device=DEV)
    if bf16:
        x = synth.to_bf16_rne(x)
    y = torch.empty(n, F, device=DEV)
    pick = (synth.stream_bits(seed, 21, torch.arange(n_sample, dtype=torch.int64)) >> 1) % n
    pick = torch.unique(pick).to(DEV)
    for transposed in (False, True):
        a, b = (dst, src) if transposed else (src, dst)       # row owner = b, neighbour = a
        y.fill_(float("nan"))
        g.grp_spmm(part, transposed, g.SCALE_MEAN, False, F, x, F, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, y, F)
        torch.cuda.synchronize()
        # (a) sampled rows, exact
        sel = torch.isin(b, pick)
        e_row, e_nb = b[sel], a[sel]
        nbs, inv = torch.unique(e_nb, return_inverse=True)
        rows, rinv = torch.unique(torch.cat([pick, e_row]), return_inverse=True)     # = pick, sorted
        blk = dict(n_dst=int(rows.numel()), n_src=int(nbs.numel()), esrc=inv.cpu().numpy(),
                   edst=rinv[pick.numel():].cpu().numpy())
        xn = x[nbs].cpu().double().numpy()
        deg = np.bincount(blk["edst"], minlength=blk["n_dst"]).astype(np.float64)
        want = ognn._scatter_rows(blk["n_dst"], blk["edst"], xn[blk["esrc"]]) / np.maximum(deg, 1.0)[:, None]
        got = y[rows].cpu().double().numpy()
        scale_ref = max(np.abs(want).max(), 1e-30)
        err = np.abs(got - want).max() / scale_ref
        print(f"[case] transposed={transposed} sampled rows {rows.numel()} (max degree {int(deg.max())}, "
              f"{int((deg == 0).sum())} empty) rel err {err:.2e}", flush=True)
        assert err <= TOL_FP32
        # (b) column checksum over every edge, in float64
        degb = torch.bincount(b, minlength=n).to(torch.float64)
        w = torch.zeros(n, dtype=torch.float64, device=DEV).index_add_(0, a, 1.0 / degb[b])
        lhs = y.sum(dim=0, dtype=torch.float64)
        rhs = torch.zeros(F, dtype=torch.float64, device=DEV)
        step = 1 << 20
        for lo in range(0, n, step):                       # chunked: keeps the float64 copy of X small
            rhs += (w[lo:lo + step, None] * x[lo:lo + step].to(torch.float64)).sum(dim=0)
        cerr = float((lhs - rhs).abs().max() / rhs.abs().max())
        print(f"[case] transposed={transposed} checksum rel err {cerr:.2e}", flush=True)
        assert cerr <= TOL_FP32
        assert not torch.isnan(y).any()
    part.destroy()


def test_config4_spmm_full_size():
    import paper_2602_01872_amd as g
    g.load()
    print("[case] configuration 4 SpMM full size (n=2^22, 1e8 edges, F=256 fp32)", flush=True)
    _sampled_rows_and_checksum(g, 22, 1 << 22, 100_000_000, 2602018724, 256, False)


def test_config5_spmm_quarter_size():
    import paper_2602_01872_amd as g
    g.load()
    print("[case] configuration 5 SpMM at a quarter of its edges (n=2^24, 2^30 edges, F=64 bf16)", flush=True)
    _sampled_rows_and_checksum(g, 24, 1 << 24, 1 << 30, 2602018725, 64, True)
