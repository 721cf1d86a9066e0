"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded
inputs.  Integer outputs (partition, local indices, degrees, |S|, the full-graph shrinkage
sum) must be bit-exact; floating point within the tolerances in tests/_cases.py."""
import numpy as np
import pytest
import torch

import synth
from oracle import coverage as ocov
from oracle import gnn as ognn
from oracle import graph as ograph
from oracle import sampling as osampling
from oracle import step as ostep
from tests._cases import TOL_BF16, TOL_FP32, assert_blocks_equal, assert_grads_close, assert_step_grads_close, make_inputs, rel_err, split_flat

pytestmark = pytest.mark.gpu

DEV = "cuda"


@pytest.fixture(scope="module")
def g():
    import paper_2602_01872_amd as lib
    lib.load()
    return lib


def _note(msg):
    print(f"[case] {msg}", flush=True)


PART_KEYS = ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in")


def _assert_partition_equal(part, want):
    assert part.n == want["n"] and part.nnz == want["nnz"]
    for k in PART_KEYS:
        got = part.array(k)
        assert got.dtype == want[k].dtype, k
        assert np.array_equal(got, want[k]), f"{k} differs"


# ----------------------------------------------------------------------------- partition
@pytest.mark.parametrize("kind,N,E,K,seed", [
    ("uniform", 10000, 100000, 4, 1),
    ("uniform", 1000, 5000, 1, 0),
    ("uniform", 50, 400, 64, 3),
    ("rmat", 1 << 14, 300000, 8, 1),
    ("rmat", 1 << 12, 200000, 3, 12345678901234567),
])
def test_partition_bit_exact(g, kind, N, E, K, seed):
    _note(f"partition {kind} N={N} E={E} K={K} seed={seed}")
    if kind == "uniform":
        s, d = synth.uniform_graph(N, E, seed=2602018721, device=DEV)
    else:
        s, d = synth.rmat_graph(N.bit_length() - 1, E, seed=2602018722, device=DEV)
    sh, dh = s.cpu().numpy(), d.cpu().numpy()
    parts = sorted(set([0, K - 1, K // 2]))
    for p in parts:
        part = g.grp_partition(s, d, N, K, seed, p)
        _assert_partition_equal(part, ograph.partition(sh, dh, N, K, seed, p))
        part.destroy()


@pytest.mark.parametrize("N,K,seed", [(100003, 8, 1), (5000, 1, 9), (70000, 3000, 2**63 + 5), (1, 4, 0)])
def test_node_owners_bit_exact(g, N, K, seed):
    _note(f"node owners N={N} K={K}")
    owner = torch.full((N,), -1, dtype=torch.int32, device=DEV)
    count = torch.full((K,), -7, dtype=torch.int64, device=DEV)
    g.grp_node_owners(N, K, seed, owner, count)
    torch.cuda.synchronize()
    want = ograph.owner(N, K, seed)
    assert np.array_equal(owner.cpu().numpy(), want)
    assert np.array_equal(count.cpu().numpy(), np.bincount(want, minlength=K))
    g.grp_node_owners(N, K, seed, owner, None)            # the histogram is optional
    with pytest.raises(g.GrappaError):
        g.grp_node_owners(N, 0, seed, owner, count)


def test_partition_edge_cases_and_errors(g):
    _note("partition edge cases")
    part = g.grp_partition(None, None, 10, 3, 0, 1)
    e = np.zeros(0, dtype=np.int64)
    _assert_partition_equal(part, ograph.partition(e, e, 10, 3, 0, 1))
    part = g.grp_partition(None, None, 0, 2, 0, 0)
    assert part.n == 0 and part.nnz == 0
    s = torch.tensor([0, 1, 12], dtype=torch.int64, device=DEV)
    d = torch.tensor([1, 2, 3], dtype=torch.int64, device=DEV)
    with pytest.raises(g.GrappaError) as ei:
        g.grp_partition(s, d, 10, 2, 0, 0)
    assert ei.value.status == g.ERANGE
    for K, p in ((0, 0), (2, 2), (2, -1)):
        with pytest.raises(g.GrappaError) as ei:
            g.grp_partition(s[:2], d[:2], 10, K, 0, p)
        assert ei.value.status == g.EINVAL


def test_partition_from_local_coo(g):
    _note("partition_from_local_coo")
    n, E = 3000, 40000
    s, d = synth.rmat_graph(12, E, seed=5, n_nodes=n, device=DEV)
    part0 = g.grp_partition_from_local_coo(s, d, n)
    want = ograph.local_graph_from_edges(s.cpu().numpy(), d.cpu().numpy(), n)
    _assert_partition_equal(part0, want)
    dg = synth.stand_in_global_degree(torch.from_numpy(want["d_local_in"]), torch.arange(n), 9, 15).to(DEV)
    part = g.grp_partition_from_local_coo(s, d, n, d_global_in=dg)
    assert np.array_equal(part.array("d_global_in"), dg.cpu().numpy())
    with pytest.raises(g.GrappaError) as ei:
        g.grp_partition_from_local_coo(s, d, n - 2000)
    assert ei.value.status == g.ERANGE


# ----------------------------------------------------------------------------- SpMM
def _oracle_spmm(part, transposed, scale, self_term, x):
    n = part["n"]
    if transposed:
        ptr, idx = part["colptr"], part["row"]
    else:
        ptr, idx = part["rowptr"], part["col"]
    blk = ognn.block_from_csr(ptr, idx)
    y = ognn._scatter_rows(n, blk["edst"], x[blk["esrc"]])
    deg = np.diff(ptr).astype(np.float64)
    if self_term:
        y += x
    if scale == 1:
        y *= (1.0 / np.maximum(deg, 1.0))[:, None]
    elif scale == 2:
        y *= (1.0 / np.sqrt(np.maximum(deg + (1 if self_term else 0), 1.0)))[:, None]
    return y


@pytest.mark.parametrize("F,ld,bf16", [(8, 8, False), (47, 48, False), (47, 47, False), (64, 64, True), (100, 100, False),
                                       (128, 128, True), (256, 256, False), (300, 300, False), (5, 8, True)])
def test_spmm_matches_oracle(g, F, ld, bf16):
    _note(f"spmm F={F} ld={ld} bf16={bf16}")
    N, E, K = 1 << 13, 200000, 2
    s, d = synth.rmat_graph(13, E, seed=77, device=DEV)
    part = g.grp_partition(s, d, N, K, 5, 1)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 5, 1)
    n = part.n
    assert int(op["d_local_in"].max()) > 2 * 512      # a hub row that is split into chunks (rows over 512 edges are)
    assert int(op["d_local_out"].max()) > 2 * 512
    assert (op["d_local_in"] == 0).any()
    xf = synth.normal_matrix(n, ld, 3)
    xf[:, F:] = 0
    x = (synth.to_bf16_rne(xf) if bf16 else xf).to(DEV)
    x64 = x.cpu().double().numpy()[:, :F]
    tol = TOL_FP32
    for transposed in (False, True):
        for scale, self_term in ((g.SCALE_NONE, False), (g.SCALE_MEAN, False), (g.SCALE_RSQRT, True), (g.SCALE_RSQRT, False)):
            y = torch.full((n, ld), float("nan"), device=DEV)
            g.grp_spmm(part, transposed, scale, self_term, F, x, ld, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, y, ld)
            torch.cuda.synchronize()
            want = _oracle_spmm(op, transposed, scale, self_term, x64)
            got = y.cpu().numpy()[:, :F]
            assert rel_err(got, want) <= tol, (transposed, scale, self_term, rel_err(got, want))


@pytest.mark.parametrize("F,bf16", [(16, False), (64, True), (47, False), (256, False), (300, False)])
def test_spmm_with_the_sliced_schedule_matches_oracle(g, F, bf16):
    """The source-sliced schedule of the long rows (built for large partitions) forced on a small one: rows cut
    into 64 source ranges and pieces of at most 128 edges, partial rows combined per row."""
    _note(f"spmm sliced schedule F={F} bf16={bf16}")
    n, E = 5000, 700000
    s, d = synth.rmat_graph(13, E, seed=78, n_nodes=n, device=DEV)
    plain = g.grp_partition_from_local_coo(s, d, n)        # 5000 nodes: below the default policy's size
    g.grp_set_slice_policy(1, 0)
    try:
        part = g.grp_partition_from_local_coo(s, d, n)
    finally:
        g.grp_set_slice_policy()
    # the sliced handle keeps a partial row per piece of at most 128 edges, the plain one per chunk of 512
    assert g.grp_spmm_workspace_bytes(part, False, F) > 2 * g.grp_spmm_workspace_bytes(plain, False, F) > 0
    plain.destroy()
    op = ograph.local_graph_from_edges(s.cpu().numpy(), d.cpu().numpy(), n)
    assert int(op["d_local_in"].max()) > 15000 and int((op["d_local_in"] > 512).sum()) > 100      # hub rows of many pieces per range
    assert g.grp_spmm_workspace_bytes(part, False, F) > 0
    ld = (F + 3) // 4 * 4
    xf = synth.normal_matrix(n, ld, 3)
    xf[:, F:] = 0
    x = (synth.to_bf16_rne(xf) if bf16 else xf).to(DEV)
    x64 = x.cpu().double().numpy()[:, :F]
    for transposed in (False, True):
        for scale, self_term in ((g.SCALE_MEAN, False), (g.SCALE_RSQRT, True)):
            y = torch.full((n, ld), float("nan"), device=DEV)
            g.grp_spmm(part, transposed, scale, self_term, F, x, ld, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, y, ld)
            torch.cuda.synchronize()
            want = _oracle_spmm(op, transposed, scale, self_term, x64)
            assert rel_err(y.cpu().numpy()[:, :F], want) <= TOL_FP32, (transposed, scale, rel_err(y.cpu().numpy()[:, :F], want))
    # a train step on the same handle (every aggregation of the step takes the sliced path), GCN for the per-source scale
    for arch, name, dims in ((g.ARCH_SAGE_MEAN, "sage", [24, 40, 6]), (g.ARCH_GCN, "gcn", [24, 16, 6])):
        xs, ys, theta = make_inputs(n, dims, name, 9)
        model = g.model_desc(arch, dims)
        opts = g.step_opts(estimator=g.EST_SHRINKAGE)
        P = g.grp_param_count(model)
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
        grad = torch.full((P,), float("nan"), device=DEV)
        stats = g.new_stats(1)
        g.grp_train_step(part, model, opts, xs.to(DEV), ys.to(DEV), None, theta.to(DEV), ws, grad, stats)
        torch.cuda.synchronize()
        fn = lambda relu_flip=None, near_kink=None: ostep.train_step(op, name, dims, theta.double().numpy(), xs.double().numpy(),
                                                                      ys.numpy(), estimator=3, relu_flip=relu_flip, near_kink=near_kink)
        assert_step_grads_close(grad.cpu().numpy(), fn, name, dims, TOL_FP32)
    part.destroy()


# ----------------------------------------------------------------------------- GEMMs
@pytest.mark.parametrize("M,N,K,bf16", [(1000, 256, 256, False), (777, 47, 100, False), (129, 8, 64, False),
                                        (5000, 172, 128, True), (333, 130, 33, False), (64, 64, 256, False)])
def test_gemm_nn_matches_numpy(g, M, N, K, bf16):
    _note(f"gemm_nn M={M} N={N} K={K} bf16={bf16}")
    a = synth.normal_matrix(M, K, 1)
    a = (synth.to_bf16_rne(a) if bf16 else a).to(DEV)
    b = synth.normal_matrix(K, N, 2).to(DEV)
    c = torch.full((M, N), float("nan"), device=DEV)
    g.grp_gemm_nn(M, N, K, a, K, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, b, N, c, N)
    torch.cuda.synchronize()
    want = a.cpu().double().numpy() @ b.cpu().double().numpy()
    assert rel_err(c.cpu().numpy(), want) <= TOL_FP32


@pytest.mark.parametrize("M,K,N,bf16", [(10000, 256, 256, False), (70001, 100, 47, False), (513, 64, 8, False),
                                        (30000, 128, 172, True), (31, 33, 130, False), (0, 16, 16, False),
                                        (20000, 64, 128, True), (9001, 48, 47, False), (40000, 17, 64, False)])
def test_gemm_tn_matches_numpy(g, M, K, N, bf16):
    _note(f"gemm_tn M={M} K={K} N={N} bf16={bf16}")
    a = synth.normal_matrix(max(M, 1), K, 3)[:M]
    a = (synth.to_bf16_rne(a) if bf16 else a).to(DEV)
    b = synth.normal_matrix(max(M, 1), N, 4)[:M].to(DEV)
    c = torch.full((K, N), float("nan"), device=DEV)
    ws = torch.empty(max(g.grp_gemm_tn_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device=DEV)
    g.grp_gemm_tn(M, K, N, a, K, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, b, N, c, N, ws)
    torch.cuda.synchronize()
    want = a.cpu().double().numpy().T @ b.cpu().double().numpy()
    got = c.cpu().numpy()
    if M == 0:
        assert (got == 0).all()
    else:
        assert rel_err(got, want) <= TOL_FP32


# ----------------------------------------------------------------------------- train step + aggregate
ARCH = {"sage": 0, "gcn": 1, "gcn_res": 2}


def _run_step(g, part, arch, dims, x, y, theta, mask=None, est=0, bf16=False, self_loops=True):
    model = g.model_desc(ARCH[arch], dims, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, self_loops)
    opts = g.step_opts(estimator=est, full_graph=True)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x, y, mask, theta, ws, grad, stats)
    torch.cuda.synchronize()
    return grad, stats


def _check_stats(st_gpu, st_cpu, tol):
    assert int(st_gpu["S"]) == st_cpu["S"]
    assert int(st_gpu["nnz_used"]) == st_cpu["nnz_used"]
    assert float(st_gpu["R"]) == st_cpu["R"]                          # integer count in full-graph mode
    assert abs(float(st_gpu["sum_ratio"]) - st_cpu["sum_ratio"]) <= 1e-9 * max(1.0, st_cpu["sum_ratio"])
    assert abs(float(st_gpu["loss"]) - st_cpu["loss"]) <= tol * max(abs(st_cpu["loss"]), 1e-30)


@pytest.mark.parametrize("est", [0, 1])
def test_config1_gcn2_four_partitions_and_aggregate(g, est):
    """Workload 1: 2-layer GCN, uniform graph N=10,000 / E=100,000, 4 hash partitions,
    features 64, hidden 64, 8 classes; one step per partition, then every aggregation variant."""
    _note(f"config 1 est={est}")
    N, E, K, dims = 10000, 100000, 4, [64, 64, 8]
    s, d = synth.uniform_graph(N, E, seed=2602018721, device=DEV)
    sh, dh = s.cpu().numpy(), d.cpu().numpy()
    xg = synth.normal_matrix(N, 64, 2602018721)
    yg = synth.labels(N, 8, 2602018721)
    theta = synth.model_weights("gcn", dims, 2602018721)
    P = theta.numel()
    ldg = ((P + 3) // 4) * 4
    grads = torch.zeros(K, ldg, device=DEV)
    stats = g.new_stats(K)
    o_grads, o_stats = [], []
    for p in range(K):
        part = g.grp_partition(s, d, N, K, 1, p)
        op = ograph.partition(sh, dh, N, K, 1, p)
        _assert_partition_equal(part, op)
        x = xg[op["l2g"]].contiguous()
        y = yg[op["l2g"]].contiguous()
        model = g.model_desc(g.ARCH_GCN, dims)
        opts = g.step_opts(estimator=est)
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
        g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grads[p],
                         stats[p * g.STATS_BYTES:(p + 1) * g.STATS_BYTES])
        torch.cuda.synchronize()
        def oracle_fn(relu_flip=None, near_kink=None):
            return ostep.train_step(op, "gcn", dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                    estimator=est, relu_flip=relu_flip, near_kink=near_kink)
        og, ost = assert_step_grads_close(grads[p, :P].cpu().numpy(), oracle_fn, "gcn", dims, TOL_FP32)
        _check_stats(g.read_stats(stats)[p], ost, TOL_FP32)
        o_grads.append(og)
        o_stats.append(ost)
    for variant in (0, 1, 2, 3):
        upd = torch.full((P,), float("nan"), device=DEV)
        c = torch.zeros(K, device=DEV)
        g.grp_aggregate(grads, ldg, stats, K, P, variant, upd, c)
        torch.cuda.synchronize()
        G, oc = ocov.aggregate(o_grads, o_stats, variant)
        assert rel_err(c.cpu().numpy(), oc) <= TOL_FP32
        assert_grads_close(upd.cpu().numpy(), G, "gcn", dims, TOL_FP32)


@pytest.mark.parametrize("arch,dims,bf16,self_loops,masked", [
    ("sage", [100, 256, 256, 47], False, True, False),
    ("sage", [64, 128, 16], True, True, True),
    ("sage", [128, 256, 256, 172], True, True, False),
    ("sage", [36, 20, 52, 7], False, True, True),
    ("gcn", [128, 256, 64], False, False, True),
    ("gcn", [40, 72, 72, 10], False, True, False),
])
def test_train_step_rmat_matches_oracle(g, arch, dims, bf16, self_loops, masked):
    """R-MAT partition (degree skew, empty rows, multi-edges) at sizes the oracle finishes in
    seconds: several 128-row tiles plus a ragged tail."""
    _note(f"train_step {arch} dims={dims} bf16={bf16} sl={self_loops} masked={masked}")
    scale, E, K = 14, 400000, 3
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018722, device=DEV)
    part = g.grp_partition(s, d, N, K, 1, 0)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)
    n = part.n
    assert n % 128 != 0
    x, y, theta = make_inputs(n, dims, arch, 11, bf16=bf16)
    mask = synth.train_mask(n, 0.3, 4) if masked else None
    tol = TOL_BF16 if bf16 else TOL_FP32
    for est in (0, 1):
        grad, stats = _run_step(g, part, arch, dims, x.to(DEV), y.to(DEV), theta.to(DEV),
                                None if mask is None else mask.to(DEV), est, bf16, self_loops)
        def oracle_fn(relu_flip=None, near_kink=None, est=est):
            return ostep.train_step(op, arch, dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                    train_mask=None if mask is None else mask.numpy(), estimator=est,
                                    gcn_self_loops=self_loops, relu_flip=relu_flip, near_kink=near_kink)
        og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, arch, dims, min(tol, TOL_FP32))
        _check_stats(g.read_stats(stats)[0], ost, TOL_FP32)


def test_train_step_is_bit_reproducible(g):
    _note("determinism")
    scale, E, K, dims = 13, 150000, 2, [64, 96, 10]
    s, d = synth.rmat_graph(scale, E, seed=9, device=DEV)
    part = g.grp_partition(s, d, 1 << scale, K, 1, 1)
    x, y, theta = make_inputs(part.n, dims, "sage", 5)
    a, sa = _run_step(g, part, "sage", dims, x.to(DEV), y.to(DEV), theta.to(DEV))
    b, sb = _run_step(g, part, "sage", dims, x.to(DEV), y.to(DEV), theta.to(DEV))
    assert torch.equal(a, b) and torch.equal(sa, sb)


def test_train_step_degenerate_partitions(g):
    _note("degenerate partitions")
    dims = [8, 12, 3]
    theta = synth.model_weights("sage", dims, 1).to(DEV)
    # empty partition: zero gradient, S = 0, loss 0
    part = g.grp_partition(None, None, 0, 1, 0, 0)
    grad, stats = _run_step(g, part, "sage", dims, torch.zeros(1, 8, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV), theta)
    st = g.read_stats(stats)[0]
    assert (grad == 0).all() and st["S"] == 0 and st["loss"] == 0.0
    # no edges at all; every node isolated
    part = g.grp_partition(None, None, 300, 1, 0, 0)
    x, y, _ = make_inputs(300, dims, "sage", 2)
    grad, stats = _run_step(g, part, "sage", dims, x.to(DEV), y.to(DEV), theta)
    op = ograph.partition(np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64), 300, 1, 0, 0)
    og, ost = ostep.train_step(op, "sage", dims, theta.cpu().double().numpy(), x.double().numpy(), y.numpy())
    assert_grads_close(grad.cpu().numpy(), og, "sage", dims, TOL_FP32)
    # empty loss set
    mask = torch.zeros(300, dtype=torch.uint8, device=DEV)
    grad, stats = _run_step(g, part, "sage", dims, x.to(DEV), y.to(DEV), theta, mask=mask)
    assert (grad == 0).all() and g.read_stats(stats)[0]["S"] == 0


def test_error_paths(g):
    _note("error paths")
    part = g.grp_partition(None, None, 100, 1, 0, 0)
    dims = [8, 4]
    model = g.model_desc(g.ARCH_GCN, dims)
    opts = g.step_opts()
    need = g.grp_step_workspace_bytes(part, model, opts)
    x, y, theta = make_inputs(100, dims, "gcn", 1)
    x, y, theta = x.to(DEV), y.to(DEV), theta.to(DEV)
    grad = torch.zeros(theta.numel(), device=DEV)
    stats = g.new_stats(1)
    small = torch.empty(max(need - 256, 1), dtype=torch.uint8, device=DEV)
    with pytest.raises(g.GrappaError) as ei:
        g.grp_train_step(part, model, opts, x, y, None, theta, small, grad, stats)
    assert ei.value.status == g.EWORKSPACE
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    with pytest.raises(g.GrappaError) as ei:
        g.grp_train_step(part, model, opts, x, y, None, None, ws, grad, stats)
    assert ei.value.status == g.EINVAL
    bad = g.model_desc(g.ARCH_GCN, [8, -1])
    with pytest.raises(g.GrappaError) as ei:
        g.grp_step_workspace_bytes(part, bad, opts)
    assert ei.value.status == g.EINVAL
    with pytest.raises(g.GrappaError) as ei:
        g.grp_aggregate(grad, 8, stats, 0, 4, 0, grad)
    assert ei.value.status == g.EINVAL
    with pytest.raises(g.GrappaError) as ei:
        g.grp_aggregate(grad, 8, stats, 1, 4, 9, grad)
    assert ei.value.status == g.EINVAL
    assert "variant" in str(ei.value)


def test_aggregate_invariants(g):
    """Full coverage -> plain average for every variant; K = 256 shrinkage against the oracle."""
    _note("aggregate invariants")
    K, P = 256, 20624
    ld = P
    grads = synth.normal_matrix(K, ld, 8).to(DEV)
    recs = np.zeros(K, dtype=g.STATS_DTYPE)
    recs["S"] = 1000
    recs["sum_ratio"] = 1000.0
    recs["R"] = 0.0
    stats = torch.from_numpy(recs.view(np.uint8)).to(DEV)
    plain = grads.cpu().double().numpy().mean(axis=0)
    for variant in (0, 1, 2, 3):
        upd = torch.zeros(P, device=DEV)
        g.grp_aggregate(grads, ld, stats, K, P, variant, upd)
        torch.cuda.synchronize()
        assert rel_err(upd.cpu().numpy(), plain) <= TOL_FP32
    recs["sum_ratio"] = np.linspace(3.0, 900.0, K)
    recs["R"] = np.arange(K) * 17.0                                  # R_0 = 0 -> c = 1
    recs["S"][5] = 0
    stats = torch.from_numpy(recs.view(np.uint8)).to(DEV)
    ost = [dict(S=int(r["S"]), sum_ratio=float(r["sum_ratio"]), R=float(r["R"])) for r in recs]
    og = [grads[p].cpu().double().numpy() for p in range(K)]
    for variant in (2, 3):
        upd = torch.zeros(P, device=DEV)
        c = torch.zeros(K, device=DEV)
        g.grp_aggregate(grads, ld, stats, K, P, variant, upd, c)
        torch.cuda.synchronize()
        G, oc = ocov.aggregate(og, ost, variant)
        assert rel_err(c.cpu().numpy(), oc) <= TOL_FP32
        assert rel_err(upd.cpu().numpy(), G) <= TOL_FP32


@pytest.mark.parametrize("K,P", [(4, 4680), (13, 1001), (256, 20624), (9, 3)])
def test_aggregate_over_separately_owned_buffers(g, K, P):
    """grp_aggregate_ptrs: K gradient buffers of their own (some deliberately misaligned) against the oracle, and
    bit for bit against the slab form on the same values."""
    _note(f"aggregate_ptrs K={K} P={P}")
    vals = synth.normal_matrix(K, P, 12)
    aligned = [vals[p].clone().to(DEV) for p in range(K)]
    odd = []
    for p in range(K):                                      # every other buffer starts 4 bytes off a 16-byte boundary
        buf = torch.zeros(P + 4, device=DEV)
        view = buf[1:P + 1] if p % 2 else buf[:P]
        view.copy_(vals[p])
        odd.append(view)
    recs = np.zeros(K, dtype=g.STATS_DTYPE)
    recs["S"] = 100 + np.arange(K)
    recs["sum_ratio"] = np.linspace(3.0, 90.0, K)
    recs["R"] = np.arange(K) * 3.0
    stats = torch.from_numpy(recs.view(np.uint8)).to(DEV)
    ost = [dict(S=int(r["S"]), sum_ratio=float(r["sum_ratio"]), R=float(r["R"])) for r in recs]
    og = [vals[p].double().numpy() for p in range(K)]
    ld = (P + 3) // 4 * 4
    slab = torch.zeros(K, ld, device=DEV)
    slab[:, :P] = vals.to(DEV)
    for variant in (0, 2, 3):
        want = torch.zeros(P, device=DEV)
        g.grp_aggregate(slab, ld, stats, K, P, variant, want)
        G, oc = ocov.aggregate(og, ost, variant)
        for bufs in (aligned, odd):
            upd = torch.full((P,), float("nan"), device=DEV)
            c = torch.zeros(K, device=DEV)
            keep = g.grp_aggregate_ptrs(bufs, stats, P, variant, upd, c)
            torch.cuda.synchronize()
            assert rel_err(upd.cpu().numpy(), G) <= TOL_FP32 and rel_err(c.cpu().numpy(), oc) <= TOL_FP32
            assert torch.equal(upd, want)
            del keep


@pytest.mark.gpu
def test_partition_that_keeps_far_more_edges_than_a_random_one(g):
    """Every edge lies inside partition 0 (a graph drawn on its nodes only), so the one-pass build's key
    buffer, sized for about E / K^2 kept edges, overflows and the keys are written by the second pass."""
    _note("partition with all edges kept")
    N, K, E = 6000, 4, 1_600_000
    owner = torch.empty(N, dtype=torch.int32, device=DEV)
    g.grp_node_owners(N, K, 5, owner)
    mine = torch.nonzero(owner == 0).flatten().cpu()
    a, b = synth.uniform_graph(int(mine.numel()), E, seed=97)
    s, d = mine[a], mine[b]
    assert E > 2 * (E // K // K) + (1 << 20)                   # beyond the first buffer
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 5, 0)
    want = ograph.partition(s.numpy(), d.numpy(), N, K, 5, 0)
    assert want["nnz"] == E
    _assert_partition_equal(part, want)
    part.destroy()
    other = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 5, 1)     # and a partition that keeps none of them
    assert other.nnz == 0 and int(other.array("d_global_in").sum()) == 0
    other.destroy()


# ----------------------------------------------------------------------------- mini-batch + residual GCN
@pytest.mark.parametrize("dims,fanouts,bf16,n_seeds", [
    ([32, 48, 6], (4, 3), False, 200),
    ([128, 256, 256, 172], (15, 10, 5), True, 1024),
    ([40, 24, 24, 5], (6, 5, 64), False, 333),
    ([24, 32, 32, 4], (7, 64, 1), False, 97),          # run on the graph with star hubs (below); fanouts 64 and 1 are the limits
])
def test_minibatch_train_step_matches_oracle(g, dims, fanouts, bf16, n_seeds):
    """Isolated k-hop sampling + SAGE step on the sampled blocks: the sampled structure is
    integer work (edge count, |S|, per-seed sampled counts enter R), the gradient fp32."""
    _note(f"minibatch dims={dims} fanouts={fanouts} bf16={bf16} seeds={n_seeds}")
    scale, E, K = 14, 600000, 2
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018723, device=DEV)
    stars = n_seeds == 97
    if stars:       # eight nodes with 50 000 extra in-edges each: rows far longer than anything R-MAT gives at this size
        es, _ = synth.uniform_graph(N, 400000, seed=41, device=DEV)
        ed = 100 + torch.arange(400000, device=DEV) % 8
        s, d = torch.cat([s, es]), torch.cat([d, ed])
    part = g.grp_partition(s, d, N, K, 1, 0)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)
    n = part.n
    dl = op["d_local_in"]
    assert dl.max() > 4096                                     # a hub row among the seeds
    if stars:
        assert np.count_nonzero(dl > 20000) >= 2
    # seeds: the hub, an isolated node, and a seeded spread of others (distinct)
    order = np.argsort(synth.stream_bits(5, 77, torch.arange(n)).numpy(), kind="stable")
    hubs = [int(v) for v in np.flatnonzero(dl > 20000)] if stars else [int(dl.argmax())]
    iso = int(np.flatnonzero(dl == 0)[0])
    rest = [int(v) for v in order if v not in hubs and v != iso][:n_seeds - 1 - len(hubs)]
    seeds = np.array(hubs + [iso] + rest, dtype=np.int32)
    x, y, theta = make_inputs(n, dims, "sage", 21, bf16=bf16)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32)
    for est, batch in ((0, 0), (1, 3)):
        seeds_dev = torch.from_numpy(seeds).to(DEV)
        opts = g.step_opts(estimator=est, full_graph=False, seeds=seeds_dev, fanouts=fanouts, sampler_seed=7, batch_id=batch)
        P = g.grp_param_count(model)
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
        grad = torch.full((P,), float("nan"), device=DEV)
        stats = g.new_stats(1)
        g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grad, stats)
        torch.cuda.synchronize()
        mb = dict(seeds=seeds, fanouts=fanouts, sampler_seed=7, batch_id=batch)
        assert_blocks_equal(g, part, model, opts, ws, op, seeds, fanouts, 7, batch)      # the sampled structure, bit for bit

        def oracle_fn(relu_flip=None, near_kink=None, est=est, mb=mb):
            return ostep.train_step(op, "sage", dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                    estimator=est, minibatch=mb, relu_flip=relu_flip, near_kink=near_kink)
        og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, "sage", dims, TOL_FP32)
        st = g.read_stats(stats)[0]
        assert int(st["S"]) == ost["S"] == n_seeds
        assert int(st["nnz_used"]) == ost["nnz_used"]           # same sampled edge multiset size
        assert abs(float(st["R"]) - ost["R"]) <= 1e-9 * max(1.0, ost["R"])
        assert abs(float(st["sum_ratio"]) - ost["sum_ratio"]) <= 1e-9 * max(1.0, ost["sum_ratio"])
        assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])


def test_minibatch_flags_seeds_outside_the_partition(g):
    """A mini-batch step is queued without waiting for the device, so a bad seed list cannot fail the call:
    the step runs with node 0 in the bad seeds' place (nothing outside the partition is read) and the record
    says how many there were."""
    _note("minibatch bad seeds")
    n, dims = 500, [8, 8, 3]
    s, d = synth.uniform_graph(n, 4000, seed=3, device=DEV)
    part = g.grp_partition_from_local_coo(s, d, n)
    x, y, theta = make_inputs(n, dims, "sage", 2)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    P = g.grp_param_count(model)
    for fanouts in ((3, 3), (3,)):
        m = g.model_desc(g.ARCH_SAGE_MEAN, dims[:len(fanouts)] + [dims[-1]])
        th = synth.model_weights("sage", dims[:len(fanouts)] + [dims[-1]], 2).to(DEV)
        for bad, count in (([n], 1), ([-1], 1), ([2**31 - 1, -5], 2)):
            seeds = torch.tensor([1, 2] + bad + [7], dtype=torch.int32, device=DEV)
            opts = g.step_opts(full_graph=False, seeds=seeds, fanouts=fanouts, sampler_seed=1)
            ws = torch.empty(g.grp_step_workspace_bytes(part, m, opts), dtype=torch.uint8, device=DEV)
            grad = torch.zeros(g.grp_param_count(m), device=DEV)
            stats = g.new_stats(1)
            g.grp_train_step(part, m, opts, x.to(DEV), y.to(DEV), None, th, ws, grad, stats)
            torch.cuda.synchronize()
            assert int(g.read_stats(stats)[0]["nnz_used"]) == -count, (fanouts, bad)
            blk = g.read_block(part, m, opts, ws, len(fanouts) - 1)
            want = [1, 2] + [0] * count + [7]
            assert blk["dst_nodes"].tolist() == want, (fanouts, bad)
    # and the same call with valid seeds reports its edges again
    seeds = torch.tensor([1, 2, 3, 7], dtype=torch.int32, device=DEV)
    opts = g.step_opts(full_graph=False, seeds=seeds, fanouts=(3, 3), sampler_seed=1)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, torch.zeros(P, device=DEV), stats)
    torch.cuda.synchronize()
    assert int(g.read_stats(stats)[0]["nnz_used"]) > 0


def test_minibatch_block_with_a_source_shared_by_thousands_of_seeds(g):
    """One node feeds 1500 seeds: its row of the transposed block is far beyond the length at which the
    backward aggregation splits a row into chunks (the split schedule is built on the device)."""
    _note("minibatch transposed long row")
    scale, E, K = 13, 100000, 2
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018731, device=DEV)
    op0 = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)
    quiet = np.flatnonzero(op0["d_local_in"] <= 20)[:1500]
    assert quiet.size == 1500
    feeder = int(op0["l2g"][int(np.flatnonzero(op0["d_local_in"] > 20)[0])])
    es = torch.full((1500,), feeder, dtype=torch.int64, device=DEV)
    ed = torch.from_numpy(op0["l2g"][quiet].astype(np.int64)).to(DEV)
    s, d = torch.cat([s, es]), torch.cat([d, ed])
    part = g.grp_partition(s, d, N, K, 1, 0)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 0)
    assert np.array_equal(op["l2g"], op0["l2g"])              # same nodes, same local ids
    seeds = quiet.astype(np.int32)
    dims, fanouts = [16, 24, 24, 5], (5, 6, 64)
    oblocks, _ = osampling.sample_blocks(op, seeds, fanouts, 11, 2)
    assert np.bincount(oblocks[2]["esrc"]).max() >= 1500       # the feeder, kept by every seed
    assert np.bincount(oblocks[1]["esrc"]).max() > 512         # and again one hop further in
    x, y, theta = make_inputs(part.n, dims, "sage", 23)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    opts = g.step_opts(estimator=3, full_graph=False, seeds=torch.from_numpy(seeds).to(DEV), fanouts=fanouts,
                       sampler_seed=11, batch_id=2)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((g.grp_param_count(model),), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grad, stats)
    torch.cuda.synchronize()
    mb = dict(seeds=seeds, fanouts=fanouts, sampler_seed=11, batch_id=2)

    def oracle_fn(relu_flip=None, near_kink=None):
        return ostep.train_step(op, "sage", dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                estimator=3, minibatch=mb, relu_flip=relu_flip, near_kink=near_kink)
    og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, "sage", dims, TOL_FP32)
    st = g.read_stats(stats)[0]
    assert int(st["nnz_used"]) == ost["nnz_used"]
    assert abs(float(st["R"]) - ost["R"]) <= 1e-9 * max(1.0, ost["R"])


def test_minibatch_of_isolated_seeds_has_empty_blocks(g):
    """Seeds without local in-edges: every block is empty (no sampled edge, no new source node) and
    only the self path carries gradient."""
    _note("minibatch isolated seeds")
    N, E, K = 600, 250, 2
    s, d = synth.uniform_graph(N, E, seed=2602018741)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, 1)
    op = ograph.partition(s.numpy(), d.numpy(), N, K, 1, 1)
    seeds = np.flatnonzero(op["d_local_in"] == 0)[:37].astype(np.int32)
    assert seeds.size == 37
    dims, fanouts = [9, 12, 12, 4], (3, 2, 5)
    x, y, theta = make_inputs(part.n, dims, "sage", 29)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    opts = g.step_opts(estimator=2, full_graph=False, seeds=torch.from_numpy(seeds).to(DEV), fanouts=fanouts,
                       sampler_seed=3, batch_id=0)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((g.grp_param_count(model),), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grad, stats)
    torch.cuda.synchronize()
    mb = dict(seeds=seeds, fanouts=fanouts, sampler_seed=3, batch_id=0)

    def oracle_fn(relu_flip=None, near_kink=None):
        return ostep.train_step(op, "sage", dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                estimator=2, minibatch=mb, relu_flip=relu_flip, near_kink=near_kink)
    og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, "sage", dims, TOL_FP32)
    st = g.read_stats(stats)[0]
    assert int(st["nnz_used"]) == ost["nnz_used"] == 0 and int(st["S"]) == 37
    wn = split_flat(grad.cpu().numpy(), "sage", dims)
    assert all(np.all(wn[f"Wn{l}"] == 0.0) for l in range(3))           # no neighbour ever contributes


def test_minibatch_is_bit_reproducible_and_batch_dependent(g):
    _note("minibatch determinism")
    scale, E = 13, 200000
    s, d = synth.rmat_graph(scale, E, seed=3, device=DEV)
    part = g.grp_partition(s, d, 1 << scale, 2, 1, 1)
    dims = [16, 32, 4]
    x, y, theta = make_inputs(part.n, dims, "sage", 2)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    seeds = torch.arange(0, 512, dtype=torch.int32, device=DEV)
    outs = []
    for batch in (0, 0, 1):
        opts = g.step_opts(full_graph=False, seeds=seeds, fanouts=(5, 5), sampler_seed=9, batch_id=batch)
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
        grad = torch.zeros(g.grp_param_count(model), device=DEV)
        stats = g.new_stats(1)
        g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grad, stats)
        torch.cuda.synchronize()
        outs.append(grad.clone())
    assert torch.equal(outs[0], outs[1])
    assert not torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("dims,self_loops", [([24, 40, 40, 40, 6], True), ([32, 32, 32, 5], False),
                                             ([128, 256, 256, 256, 64], True),
                                             ([13, 13, 13, 13, 6], True)])   # a residual first layer on 52-byte feature rows
def test_residual_gcn_matches_oracle(g, dims, self_loops):
    _note(f"residual gcn dims={dims} sl={self_loops}")
    scale, E, K = 13, 250000, 2
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018724, device=DEV)
    part = g.grp_partition(s, d, N, K, 1, 1)
    op = ograph.partition(s.cpu().numpy(), d.cpu().numpy(), N, K, 1, 1)
    x, y, theta = make_inputs(part.n, dims, "gcn_res", 31)
    grad, stats = _run_step(g, part, "gcn_res", dims, x.to(DEV), y.to(DEV), theta.to(DEV), self_loops=self_loops)

    def oracle_fn(relu_flip=None, near_kink=None):
        return ostep.train_step(op, "gcn_res", dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                gcn_self_loops=self_loops, relu_flip=relu_flip, near_kink=near_kink)
    og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, "gcn_res", dims, TOL_FP32)
    _check_stats(g.read_stats(stats)[0], ost, TOL_FP32)


@pytest.mark.parametrize("M,N,K,bf16", [(1000, 256, 256, False), (777, 47, 100, False), (4097, 172, 36, True),
                                        (333, 130, 33, False), (129, 512, 48, False), (5000, 95, 256, False),
                                        (700, 96, 100, False), (1031, 80, 52, True), (256, 72, 16, False)])
def test_gemm_nt_matches_numpy(g, M, N, K, bf16):
    _note(f"gemm_nt M={M} N={N} K={K} bf16={bf16}")
    a = synth.normal_matrix(M, K, 1)
    a = (synth.to_bf16_rne(a) if bf16 else a).to(DEV)
    bt = synth.normal_matrix(N, K, 2).to(DEV)
    c = torch.full((M, N), float("nan"), device=DEV)
    g.grp_gemm_nt(M, N, K, a, K, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32, bt, K, c, N)
    torch.cuda.synchronize()
    want = a.cpu().double().numpy() @ bt.cpu().double().numpy().T
    assert rel_err(c.cpu().numpy(), want) <= TOL_FP32


# ------------------------------------------------------------------ optimizer step and the phase-parallel loop
@pytest.mark.gpu
@pytest.mark.parametrize("P", [1, 7, 4096, 100003])
@pytest.mark.parametrize("kind", ["adam", "sgd"])
def test_optimizer_step_matches_oracle(g, P, kind):
    from oracle import optim as ooptim
    _note(f"optimizer {kind} P={P}")
    rng = np.random.default_rng(P)
    theta = rng.normal(size=P)
    m = np.zeros(P)
    v = np.zeros(P)
    th_d = torch.tensor(theta, dtype=torch.float32, device=DEV)
    m_d = torch.zeros(P, device=DEV)
    v_d = torch.zeros(P, device=DEV)
    theta = th_d.cpu().double().numpy()
    opt = g.optimizer_desc(g.OPT_ADAM if kind == "adam" else g.OPT_SGD, lr=0.003)
    # the ABI carries the hyper-parameters as fp32: the oracle gets the same (rounded) values
    lr, b1, b2, eps = (float(np.float32(h)) for h in (0.003, 0.9, 0.999, 1e-8))
    for t in range(1, 6):
        grad = (rng.normal(size=P) * 10.0 ** rng.integers(-3, 2, size=P)).astype(np.float32)
        grad[::5] = 0.0                                            # exact zeros stay put under Adam
        g_d = torch.tensor(grad, device=DEV)
        g.grp_optimizer_step(opt, P, t, th_d, g_d, m_d, v_d)
        if kind == "adam":
            theta, m, v = ooptim.adam_step(theta, grad.astype(np.float64), m, v, t, lr, b1, b2, eps)
            assert rel_err(m_d.cpu().numpy(), m) < 2e-6
            assert rel_err(v_d.cpu().numpy(), v) < 2e-6
        else:
            theta = ooptim.sgd_step(theta, grad.astype(np.float64), lr)
        # the update is lr * O(1) per step: compare absolutely against lr
        assert np.abs(th_d.cpu().double().numpy() - theta).max() < 0.003 * 2e-4


@pytest.mark.gpu
def test_optimizer_step_error_paths(g):
    t = torch.zeros(8, device=DEV)
    with pytest.raises(g.GrappaError):
        g.grp_optimizer_step(g.optimizer_desc(g.OPT_ADAM), 8, 1, t, t, None, None)      # Adam without moments
    with pytest.raises(g.GrappaError):
        g.grp_optimizer_step(g.optimizer_desc(g.OPT_SGD), 8, 0, t, t)                   # step < 1
    with pytest.raises(g.GrappaError):
        g.grp_optimizer_step(g.optimizer_desc(g.OPT_SGD, lr=0.0), 8, 1, t, t)
    with pytest.raises(g.GrappaError):
        g.grp_optimizer_step(g.optimizer_desc(7), 8, 1, t, t)
    g.grp_optimizer_step(g.optimizer_desc(g.OPT_SGD), 0, 1, t, t)                       # P = 0 is a no-op


@pytest.mark.gpu
@pytest.mark.parametrize("M", [1, 2, 4])
@pytest.mark.parametrize("kind", ["sgd", "adam"])
def test_phase_parallel_loop_matches_oracle(g, M, kind):
    """Algorithm 1 with K = 4 partitions, M per phase, two epochs: theta after every epoch and the
    loss history against the oracle loop.  SGD is linear in the gradient (tight bound); Adam
    normalises every coordinate, so coordinates whose gradient is at rounding level move by
    up to lr per step in either run and the bound is lr-sized."""
    from oracle import optim as ooptim
    _note(f"phase-parallel loop M={M} {kind}")
    N, E, K = 2000, 20000, 4
    s, d = synth.uniform_graph(N, E, seed=77)
    dims = [16, 32, 5]
    x = synth.normal_matrix(N, dims[0], 78)
    y = synth.planted_labels(x, dims[-1], 79)
    theta0 = synth.model_weights("sage", dims, 80)
    oparts = [ograph.partition(s.numpy(), d.numpy(), N, K, 1, p) for p in range(K)]
    oxs = [x.double().numpy()[p["l2g"]] for p in oparts]
    oys = [y.numpy()[p["l2g"]] for p in oparts]
    parts = [g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, p) for p in range(K)]
    xs = [x.to(DEV)[torch.from_numpy(p["l2g"]).to(DEV)].contiguous() for p in oparts]
    ys = [y.to(DEV)[torch.from_numpy(p["l2g"]).to(DEV)].contiguous() for p in oparts]
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    lr = 0.05 if kind == "sgd" else 0.003
    opt = g.optimizer_desc(g.OPT_SGD if kind == "sgd" else g.OPT_ADAM, lr=lr)
    tr = g.PhaseParallelTrainer(parts, model, xs, ys, [None] * K, theta0.to(DEV), g.EST_BATCH_MIN_DIST, M, opt)
    n_epochs = 2
    for _ in range(n_epochs):
        tr.run_epoch()
    want, hist = ooptim.train_epochs(oparts, "sage", dims, theta0.double().numpy(), oxs, oys, [None] * K, n_epochs, M,
                                     ocov.BATCH_MIN_DIST, optimizer=ooptim.SGD if kind == "sgd" else ooptim.ADAM, lr=lr)
    got = tr.theta.cpu().double().numpy()
    steps = len(hist)
    assert tr.step_count == steps == n_epochs * -(-K // M)
    np.testing.assert_allclose(tr.losses(), hist, rtol=2e-4)
    if kind == "sgd":
        assert rel_err(got, want) < TOL_FP32
    else:
        assert np.abs(got - want).max() < 0.5 * lr * steps          # no coordinate drifts by more than half its travel
        assert np.mean(np.abs(got - want) < 1e-3 * lr * steps) > 0.99   # and almost all agree closely
    for p in parts:
        p.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("arch", ["sage", "gat"])
def test_phase_steps_on_several_streams_give_the_same_bits(g, arch):
    """The partitions of a phase are independent: spread over three streams (with M = 4, so one stream
    takes two steps in a row on its workspace) the loop must reproduce the one-stream run bit for bit."""
    _note(f"phase-parallel loop on several streams {arch}")
    N, E, K, M = 3000, 40000, 4, 4
    s, d = synth.rmat_graph(12, E, seed=91, n_nodes=N)
    dims = [24, 32, 6]
    x = synth.normal_matrix(N, dims[0], 92)
    y = synth.planted_labels(x, dims[-1], 93)
    theta0 = synth.model_weights(arch, dims, 94)
    parts = [g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, p) for p in range(K)]
    l2gs = [torch.from_numpy(p.array("l2g")).to(DEV) for p in parts]
    xs = [x.to(DEV)[i].contiguous() for i in l2gs]
    ys = [y.to(DEV)[i].contiguous() for i in l2gs]
    model = g.model_desc(g.ARCH_SAGE_MEAN if arch == "sage" else g.ARCH_GAT, dims)
    runs = []
    for streams in (1, 3):
        tr = g.PhaseParallelTrainer(parts, model, xs, ys, [None] * K, theta0.to(DEV), g.EST_SHRINKAGE, M,
                                    g.optimizer_desc(g.OPT_ADAM, lr=0.003), dropout_rate=0.25, dropout_seed=5,
                                    streams=streams)
        for _ in range(3):
            tr.run_epoch()
        torch.cuda.synchronize()
        runs.append((tr.theta.clone(), tr.losses()))
    assert torch.equal(runs[0][0], runs[1][0])
    assert runs[0][1] == runs[1][1]
    for p in parts:
        p.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,cols", [(torch.float32, 100), (torch.float32, 13), (torch.bfloat16, 128), (torch.bfloat16, 7),
                                        (torch.int32, 0), (torch.uint8, 0), (torch.uint8, 5)])
def test_gather_rows_bit_exact(g, dtype, cols):
    """Rows of a global tensor by a partition's node list (16-, 4- and 1-byte moves; with and without the
    keep mask; out-of-range indices zero-filled)."""
    _note(f"gather rows {dtype} cols={cols}")
    n_src, n = 5000, 1777
    base = synth.stream_bits(9, 3, torch.arange(n_src * max(cols, 1)))
    if dtype in (torch.float32, torch.bfloat16):
        src = ((base % 2001).to(torch.float32) / 7.0 - 100.0).to(dtype)
    else:
        src = (base % 251).to(dtype)
    src = src.reshape(n_src, cols) if cols else src.reshape(n_src)
    idx = (synth.stream_bits(9, 4, torch.arange(n)) % n_src).abs()
    idx[5], idx[6] = -1, n_src                                 # outside: zero rows
    keep = (synth.stream_bits(9, 5, torch.arange(n)) % 3 != 0).to(torch.uint8)
    for kp in (None, keep):
        got = g.grp_gather_rows(src.to(DEV), idx.to(DEV), None if kp is None else kp.to(DEV)).cpu()
        want = src[idx.clamp(0, n_src - 1)].clone()
        dead = (idx < 0) | (idx >= n_src)
        if kp is not None:
            dead = dead | (kp == 0)
        want[dead] = 0
        assert got.dtype == src.dtype and got.shape == want.shape
        assert torch.equal(got.view(torch.uint8) if dtype == torch.bfloat16 else got,
                           want.view(torch.uint8) if dtype == torch.bfloat16 else want)
    assert g.grp_gather_rows(src.to(DEV), idx[:0].to(DEV)).shape[0] == 0


@pytest.mark.gpu
def test_epoch_seed_order_bit_exact(g):
    _note("epoch seed order")
    N, E, K = 5000, 30000, 3
    s, d = synth.uniform_graph(N, E, seed=61)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, 2)
    op = ograph.partition(s.numpy(), d.numpy(), N, K, 1, 2)
    n = part.n
    third = (synth.stream_bits(3, 1, torch.arange(n)).numpy() % 3 == 0).astype(np.uint8)
    out = torch.full((n,), -1, dtype=torch.int32, device=DEV)
    for mask in (None, third, np.zeros(n, dtype=np.uint8), np.ones(n, dtype=np.uint8)):
        for seed, epoch in ((7, 0), (7, 1), (2 ** 63 + 5, 12345678901)):
            out.fill_(-1)
            md = None if mask is None else torch.from_numpy(mask).to(DEV)
            cnt = g.grp_epoch_seeds(part, md, seed, epoch, out)
            want = osampling.epoch_seed_order(op, mask, seed, epoch)
            assert cnt == want.size
            assert np.array_equal(out[:cnt].cpu().numpy(), want.astype(np.int32))
            assert bool((out[cnt:] == -1).all())                   # nothing is written past the count
    part.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("M", [1, 2])
def test_minibatch_phase_parallel_loop_matches_oracle(g, M):
    """Two epochs of the mini-batch loop (K = 3 partitions of unequal training sets, so one runs out of
    seeds before the others and takes part with empty batches): theta and the loss history."""
    from oracle import optim as ooptim
    _note(f"mini-batch loop M={M}")
    N, E, K = 1500, 18000, 3
    s, d = synth.rmat_graph(11, E, seed=71, n_nodes=N)
    dims = [12, 24, 4]
    x = synth.normal_matrix(N, dims[0], 72)
    y = synth.planted_labels(x, dims[-1], 73)
    theta0 = synth.model_weights("sage", dims, 74)
    oparts = [ograph.partition(s.numpy(), d.numpy(), N, K, 1, p) for p in range(K)]
    masks = [None, (np.arange(oparts[1]["n"]) % 3 == 0).astype(np.uint8), None]
    oxs = [x.double().numpy()[p["l2g"]] for p in oparts]
    oys = [y.numpy()[p["l2g"]] for p in oparts]
    parts = [g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, p) for p in range(K)]
    xs = [x.to(DEV)[torch.from_numpy(p["l2g"]).to(DEV)].contiguous() for p in oparts]
    ys = [y.to(DEV)[torch.from_numpy(p["l2g"]).to(DEV)].contiguous() for p in oparts]
    dmasks = [None if mk is None else torch.from_numpy(mk).to(DEV) for mk in masks]
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    B, fan, lr, n_epochs = 128, (4, 3), 0.05, 2
    tr = g.MiniBatchTrainer(parts, model, xs, ys, dmasks, theta0.to(DEV), g.EST_SHRINKAGE, M, B, fan, 9,
                            g.optimizer_desc(g.OPT_SGD, lr=lr))
    for _ in range(n_epochs):
        tr.run_epoch()
    want, hist = ooptim.train_epochs_minibatch(oparts, "sage", dims, theta0.double().numpy(), oxs, oys, masks, n_epochs, M,
                                               ocov.SHRINKAGE, B, fan, 9, optimizer=ooptim.SGD, lr=lr)
    iters = max(-(-(p["n"] if mk is None else int(mk.sum())) // B) for p, mk in zip(oparts, masks))
    assert tr.iters == iters and tr.step_count == len(hist) == n_epochs * iters * -(-K // M)
    np.testing.assert_allclose(tr.losses(), hist, rtol=2e-4)
    assert rel_err(tr.theta.cpu().double().numpy(), want) < TOL_FP32
    for p in parts:
        p.destroy()


@pytest.mark.gpu
def test_minibatch_steps_driven_by_several_host_threads_give_the_same_bits(g):
    """The steps of a phase on three host threads, each with its stream and workspace (one thread takes two
    of the four steps), and as captured graphs replayed on three streams by one thread: same theta and losses
    as the one-thread loop, bit for bit."""
    _note("mini-batch loop on several host threads")
    N, E, K, M = 2000, 24000, 4, 4
    s, d = synth.rmat_graph(11, E, seed=81, n_nodes=N)
    dims = [12, 24, 24, 4]
    x = synth.normal_matrix(N, dims[0], 82)
    y = synth.planted_labels(x, dims[-1], 83)
    theta0 = synth.model_weights("sage", dims, 84)
    parts = [g.grp_partition(s.to(DEV), d.to(DEV), N, K, 1, p) for p in range(K)]
    l2gs = [torch.from_numpy(p.array("l2g")).to(DEV) for p in parts]
    xs = [x.to(DEV)[i].contiguous() for i in l2gs]
    ys = [y.to(DEV)[i].contiguous() for i in l2gs]
    masks = [None, (torch.arange(parts[1].n, device=DEV) % 2 == 0).to(torch.uint8), None, None]
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    runs = []
    for lanes, graphs in ((1, False), (3, False), (3, True)):
        # graphs: every partition's full-batch step is captured once and replayed with the seeds and the batch
        # id rewritten in device memory (the batches shorter than 100 seeds run uncaptured)
        tr = g.MiniBatchTrainer(parts, model, xs, ys, masks, theta0.to(DEV), g.EST_SHRINKAGE, M, 100, (4, 3, 5), 21,
                                g.optimizer_desc(g.OPT_ADAM, lr=0.003), dropout_rate=0.3, dropout_seed=2, lanes=lanes,
                                graphs=graphs)
        for _ in range(2):
            tr.run_epoch()
        torch.cuda.synchronize()
        runs.append((tr.theta.clone(), tr.losses()))
        if graphs:
            assert len(tr.captured) == K
    for other in runs[1:]:
        assert torch.equal(runs[0][0], other[0])
        assert runs[0][1] == other[1] and len(runs[0][1]) > 8
    for p in parts:
        p.destroy()


# ------------------------------------------------------------------ chunks and sweeping partitions
@pytest.mark.gpu
@pytest.mark.parametrize("kind,N,E,c", [("uniform", 3000, 40000, 4), ("rmat", 1 << 12, 150000, 3), ("uniform", 500, 0, 2),
                                         ("uniform", 2000, 30000, 1), ("rmat", 1 << 13, 300000, 8)])
def test_partition_from_chunks_bit_exact(g, kind, N, E, c):
    from oracle import chunks as ochunks
    _note(f"chunks {kind} N={N} E={E} c={c}")
    if E == 0:
        s = d = torch.zeros(0, dtype=torch.int64)
    elif kind == "uniform":
        s, d = synth.uniform_graph(N, E, seed=41)
    else:
        s, d = synth.rmat_graph(int(np.log2(N)), E, seed=41)
    ck = g.grp_chunks_build(s.to(DEV), d.to(DEV), N, c, 13)
    sched = ochunks.sweep_schedule(c)
    pairs = [(b, b) for b in range(c)] + [p for t in (0, len(sched) - 1) for p in sched[t]][:2 * c]
    for base, swept in pairs:
        part = g.grp_partition_from_chunks(ck, base, swept)
        want = ochunks.partition_from_chunks(s.numpy(), d.numpy(), N, c, 13, base, swept)
        _assert_partition_equal(part, want)
        assert np.array_equal(part.base_mask(), want["base_mask"])
        part.destroy()
    # the base chunk alone is the plain hash partition
    part = g.grp_partition_from_chunks(ck, 0, 0)
    plain = g.grp_partition(s.to(DEV), d.to(DEV), N, c, 13, 0)
    for k in PART_KEYS:
        assert np.array_equal(part.array(k), plain.array(k)), k
    assert plain.base_mask_ptr() == 0
    with pytest.raises(g.GrappaError):
        g.grp_partition_from_chunks(ck, c, 0)
    with pytest.raises(g.GrappaError):
        g.grp_chunks_build(s.to(DEV), d.to(DEV), N, 65, 13)
    if E:
        bad = s.clone(); bad[0] = N
        with pytest.raises(g.GrappaError):
            g.grp_chunks_build(bad.to(DEV), d.to(DEV), N, c, 13)
    part.destroy(); plain.destroy(); ck.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("arch,dims", [("sage", [24, 40, 12]), ("gcn", [16, 32, 32, 6]), ("gcn_res", [16, 32, 32, 32, 6])])
def test_step_activation_view_matches_oracle_logits(g, arch, dims):
    """grp_step_activation: the last layer's stored output is the logits matrix, the first hidden
    layer's is ReLU of the oracle's pre-activations; error paths."""
    from oracle import gnn as ognn
    _note(f"activation view {arch}")
    N, E = 3000, 30000
    s, d = synth.uniform_graph(N, E, seed=31)
    part = g.grp_partition(s.to(DEV), d.to(DEV), N, 2, 4, 1)
    op = ograph.partition(s.numpy(), d.numpy(), N, 2, 4, 1)
    n, k = part.n, len(dims) - 1
    x, y, theta = make_inputs(n, dims, arch, 3)
    model = g.model_desc(ARCH[arch], dims, g.DTYPE_FP32, True)
    opts = g.step_opts(full_graph=True)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.zeros(g.grp_param_count(model), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None, theta.to(DEV), ws, grad, stats)
    torch.cuda.synchronize()
    blk = ognn.block_from_csr(op["rowptr"], op["col"])
    _, _, logits = ognn.forward_backward(arch, dims, theta.double().numpy(), x.double().numpy(), [blk] * k, y.numpy(),
                                         np.ones(n), np.arange(n), True, return_logits=True)
    rows = np.repeat(np.arange(n), dims[-1])
    cols = np.tile(np.arange(dims[-1]), n)
    got = g.read_activation(part, model, opts, ws, k - 1, rows, cols).reshape(n, dims[-1])
    assert rel_err(got, logits) <= TOL_FP32
    # the first hidden layer against the oracle's layer function
    params = ognn.unpack_params(theta.double().numpy(), arch, dims)
    if arch == "sage":
        z0, _ = ognn._sage_forward(x.double().numpy(), blk, *params[0])
    else:
        z0, _ = ognn._gcn_forward(x.double().numpy(), blk, params[0][0], params[0][2], True)
    rows = np.repeat(np.arange(n), dims[1])
    cols = np.tile(np.arange(dims[1]), n)
    hid = g.read_activation(part, model, opts, ws, 0, rows, cols).reshape(n, dims[1])
    assert rel_err(hid, np.maximum(z0, 0.0)) <= TOL_FP32
    with pytest.raises(g.GrappaError):
        g.grp_step_activation(part, model, opts, ws, k)
    with pytest.raises(g.GrappaError):
        g.grp_step_activation(part, model, opts, ws[:256], 0)
    part.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("kind", ["ranges", "skewed", "hash"])
def test_partition_from_assigned_chunks_bit_exact(g, kind):
    """Chunks given by the caller (the output of any partitioner): contiguous id ranges, a skewed
    assignment with an empty chunk, and the library's own random split handed back in."""
    from oracle import chunks as ochunks
    _note(f"assigned chunks {kind}")
    N, E, c = 5000, 90000, 5
    s, d = synth.rmat_graph(13, E, seed=61, n_nodes=N)
    if kind == "ranges":
        assign = (np.arange(N) * c // N).astype(np.int32)
    elif kind == "skewed":
        assign = np.minimum(np.arange(N) % 7, 3).astype(np.int32)          # chunk 4 is empty, chunk 3 is large
    else:
        assign = ochunks.chunk_of(N, c, 13).astype(np.int32)
    ck = g.grp_chunks_build_assigned(s.to(DEV), d.to(DEV), N, c, torch.from_numpy(assign).to(DEV))
    for base, swept in [(0, 1), (3, 3), (4, 2), (2, 4), (1, 3)]:
        part = g.grp_partition_from_chunks(ck, base, swept)
        want = ochunks.partition_from_chunks(s.numpy(), d.numpy(), N, c, 0, base, swept, assignment=assign)
        _assert_partition_equal(part, want)
        assert np.array_equal(part.base_mask(), want["base_mask"])
        part.destroy()
    if kind == "hash":                                    # the same handle as the random split's
        ck2 = g.grp_chunks_build(s.to(DEV), d.to(DEV), N, c, 13)
        a, b = g.grp_partition_from_chunks(ck, 1, 2), g.grp_partition_from_chunks(ck2, 1, 2)
        for k in PART_KEYS:
            assert np.array_equal(a.array(k), b.array(k)), k
        a.destroy(); b.destroy(); ck2.destroy()
    bad = assign.copy()
    bad[17] = c
    with pytest.raises(g.GrappaError):
        g.grp_chunks_build_assigned(s.to(DEV), d.to(DEV), N, c, torch.from_numpy(bad).to(DEV))
    ck.destroy()


@pytest.mark.gpu
def test_calls_run_on_the_stream_they_are_given(g):
    """Partition build, train step (full-graph and mini-batch), aggregation and optimizer step on a
    second stream (default priority) give the bits of the default stream."""
    _note("explicit stream")
    N, E, dims = 6000, 80000, [32, 48, 8]
    s, d = synth.uniform_graph(N, E, seed=71)
    sd, dd = s.to(DEV), d.to(DEV)
    x, y, theta = make_inputs(N, dims, "sage", 9)
    xd, yd, td = x.to(DEV), y.to(DEV), theta.to(DEV)
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
    seeds = torch.arange(0, 256, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()

    def run():
        part = g.grp_partition(sd, dd, N, 1, 3, 0)
        outs = []
        for opts in (g.step_opts(estimator=1, full_graph=True),
                     g.step_opts(full_graph=False, seeds=seeds, fanouts=(4, 4), sampler_seed=2, batch_id=1)):
            P = g.grp_param_count(model)
            ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
            grads = torch.zeros(1, (P + 3) // 4 * 4, device=DEV)
            stats = g.new_stats(1)
            g.grp_train_step(part, model, opts, xd[:part.n], yd[:part.n], None, td, ws, grads[0], stats)
            upd = torch.zeros(P, device=DEV)
            g.grp_aggregate(grads, grads.shape[1], stats, 1, P, g.EST_BATCH_MIN_DIST, upd)
            th = td.clone()
            g.grp_optimizer_step(g.optimizer_desc(g.OPT_SGD, lr=0.1), P, 1, th, upd)
            outs += [grads.clone(), upd, th]
        torch.cuda.current_stream().synchronize()
        part.destroy()
        return outs

    base = run()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        other = run()
    torch.cuda.synchronize()
    for a, b in zip(base, other):
        assert torch.equal(a, b)
