"""grp_partition_from_csr: a share that exists as rows of in-edges is adopted as it is (the handle borrows
the arrays) and only the transposed structure, the degrees and the long-row schedules are built.  Every
array of the handle must equal the oracle's canonical arrays bit for bit, for any slice size of the
transpose; aggregation and a train step on the adopted handle must match the oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import gnn as ognn
from oracle import graph as ograph
from oracle import step as ostep
from tests._cases import TOL_FP32, assert_step_grads_close, make_inputs, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"
PART_KEYS = ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in")


@pytest.fixture(scope="module")
def g():
    import paper_2602_01872_amd as lib
    lib.load()
    return lib


def _note(msg):
    print(f"[case] {msg}", flush=True)


def _adopt(g, want, slice_edges=0, d_global=None, l2g=None):
    rowptr = torch.from_numpy(want["rowptr"]).to(DEV)
    col = torch.from_numpy(want["col"]).to(DEV)
    return g.grp_partition_from_csr(rowptr, col, want["n"], d_global_in=d_global, l2g=l2g, slice_edges=slice_edges)


def _assert_equal(part, want):
    assert part.n == want["n"] and part.nnz == want["nnz"]
    for k in PART_KEYS:
        got = part.array(k)
        assert got.dtype == want[k].dtype, k
        assert np.array_equal(got, want[k]), f"{k} differs"


@pytest.mark.parametrize("kind,n,E,slice_edges", [
    ("uniform", 5000, 60000, 0),            # one slice
    ("uniform", 5000, 60000, 7000),         # nine slices, each a run of whole histogram bins
    ("rmat", 1 << 13, 400000, 50000),       # hub rows of several thousand edges in both directions
    ("rmat", 1 << 13, 400000, 1),           # the bound is raised to the largest bin: a slice per bin
    ("rmat", 300000, 50000, 9000),          # far more rows than edges: tiles whose row window exceeds LDS
    ("uniform", 3, 5000, 100),              # three nodes, long duplicate runs
])
def test_from_csr_bit_exact(g, kind, n, E, slice_edges):
    _note(f"from_csr {kind} n={n} E={E} slice_edges={slice_edges}")
    if kind == "uniform":
        s, d = synth.uniform_graph(n, E, seed=31)
    else:
        s, d = synth.rmat_graph(max(2, (n - 1).bit_length()), E, seed=32, n_nodes=n)
    want = ograph.local_graph_from_edges(s.numpy(), d.numpy(), n)
    part = _adopt(g, want, slice_edges)
    _assert_equal(part, want)
    # the CSR is borrowed, not copied
    assert part.view.rowptr == part._borrowed[0].data_ptr() and part.view.col == part._borrowed[1].data_ptr()
    part.destroy()
    # with a stand-in global degree and a node list of its own
    dg = synth.stand_in_global_degree(torch.from_numpy(want["d_local_in"]), torch.arange(n), 9, 15)
    l2g = torch.arange(n, dtype=torch.int64) * 3 + 1
    part = _adopt(g, want, slice_edges, d_global=dg.to(DEV), l2g=l2g.to(DEV))
    assert np.array_equal(part.array("d_global_in"), dg.numpy()) and np.array_equal(part.array("l2g"), l2g.numpy())
    part.destroy()


def test_from_csr_matches_the_edge_list_builder(g):
    _note("from_csr against grp_partition_from_local_coo and the generator of sorted shares")
    n, E = 20000, 700000
    s, d = synth.rmat_graph(15, E, seed=8, n_nodes=n, device=DEV)
    ref = g.grp_partition_from_local_coo(s, d, n)
    rowptr, col = synth.rmat_local_csr(15, E, seed=8, n_nodes=n, device=DEV, chunk=100000, slice_edges=90000)
    assert np.array_equal(rowptr.cpu().numpy(), ref.array("rowptr")) and np.array_equal(col.cpu().numpy(), ref.array("col"))
    part = g.grp_partition_from_csr(rowptr, col, n, slice_edges=130000)
    for k in PART_KEYS:
        assert np.array_equal(part.array(k), ref.array(k)), k


def test_from_csr_edge_cases_and_errors(g):
    _note("from_csr edge cases")
    z64 = torch.zeros(1, dtype=torch.int64, device=DEV)
    part = g.grp_partition_from_csr(z64, None, 0)
    assert part.n == 0 and part.nnz == 0
    rp = torch.zeros(11, dtype=torch.int64, device=DEV)
    part = g.grp_partition_from_csr(rp, None, 10)                       # ten isolated nodes
    _assert_equal(part, ograph.local_graph_from_edges(np.zeros(0, np.int64), np.zeros(0, np.int64), 10))
    rowptr = torch.tensor([0, 2, 2, 5], dtype=torch.int64, device=DEV)
    ok = torch.tensor([0, 2, 0, 1, 1], dtype=torch.int32, device=DEV)
    part = g.grp_partition_from_csr(rowptr, ok, 3)
    _assert_equal(part, ograph.local_graph_from_edges(np.array([0, 2, 0, 1, 1]), np.array([0, 0, 2, 2, 2]), 3))
    for bad_col, status in ((torch.tensor([2, 0, 0, 1, 1], dtype=torch.int32), g.EINVAL),     # row 0 descends
                            (torch.tensor([0, 2, 0, 1, 3], dtype=torch.int32), g.ERANGE),     # source 3 of 3 nodes
                            (torch.tensor([0, 2, 0, -1, 1], dtype=torch.int32), g.ERANGE)):
        with pytest.raises(g.GrappaError) as ei:
            g.grp_partition_from_csr(rowptr, bad_col.to(DEV), 3)
        assert ei.value.status == status, ei.value
    for bad_ptr in ([1, 2, 2, 5], [0, 3, 2, 5], [0, 2, 2, 4], [0, 2, 2, 6]):
        with pytest.raises(g.GrappaError) as ei:
            g.grp_partition_from_csr(torch.tensor(bad_ptr, dtype=torch.int64, device=DEV), ok, 3)
        assert ei.value.status == g.EINVAL, (bad_ptr, ei.value)
    with pytest.raises(g.GrappaError) as ei:
        g.grp_partition_from_csr(None, ok, 3)
    assert ei.value.status == g.EINVAL


def _oracle_mean(ptr, idx, x):
    blk = ognn.block_from_csr(ptr, idx)
    y = ognn._scatter_rows(len(ptr) - 1, blk["edst"], x[blk["esrc"]])
    return y / np.maximum(np.diff(ptr).astype(np.float64), 1.0)[:, None]


def test_aggregation_and_step_on_an_adopted_share(g):
    _note("spmm + train step on an adopted share with long rows")
    n, E, dims = 6000, 500000, [64, 128, 16]
    s, d = synth.rmat_graph(13, E, seed=77, n_nodes=n)
    want = ograph.local_graph_from_edges(s.numpy(), d.numpy(), n)
    assert int(want["d_local_in"].max()) > 2048 and int(want["d_local_out"].max()) > 2048      # several chunks per hub
    dg = synth.stand_in_global_degree(torch.from_numpy(want["d_local_in"]), torch.arange(n), 9, 255)
    want["d_global_in"] = dg.numpy()
    part = _adopt(g, want, 60000, d_global=dg.to(DEV))
    x, y, theta = make_inputs(n, dims, "sage", 5, bf16=True)
    x64 = x.to(torch.float32).double().numpy()
    out = torch.full((n, dims[0]), float("nan"), device=DEV)
    xd = x.to(DEV)
    for transposed in (False, True):
        g.grp_spmm(part, transposed, g.SCALE_MEAN, False, dims[0], xd, dims[0], g.DTYPE_BF16, out, dims[0])
        torch.cuda.synchronize()
        ptr, idx = (want["colptr"], want["row"]) if transposed else (want["rowptr"], want["col"])
        assert rel_err(out.cpu().numpy(), _oracle_mean(ptr, idx, x64)) <= TOL_FP32, transposed
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims, feat_dtype=g.DTYPE_BF16)
    opts = g.step_opts(estimator=g.EST_SHRINKAGE)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, xd, y.to(DEV), None, theta.to(DEV), ws, grad, stats)
    torch.cuda.synchronize()
    fn = lambda relu_flip=None, near_kink=None: ostep.train_step(want, "sage", dims, theta.double().numpy(), x64, y.numpy(),
                                                                  estimator=3, relu_flip=relu_flip, near_kink=near_kink)
    og, ost = assert_step_grads_close(grad.cpu().numpy(), fn, "sage", dims, TOL_FP32)
    st = g.read_stats(stats)[0]
    assert int(st["S"]) == ost["S"] and int(st["nnz_used"]) == E and float(st["R"]) == ost["R"]
    assert abs(float(st["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
