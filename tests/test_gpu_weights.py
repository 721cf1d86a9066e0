"""GPU parity of weighted partitions (the general non-uniform neighbour weights): partition arrays
bit for bit, the weighted-mean GraphSAGE step and its coverage statistics against the oracle,
aggregation with the resulting factors, the uniform reduction and the error paths."""
import numpy as np
import pytest
import torch

import synth
from oracle import coverage as ocov
from oracle import graph as ograph
from oracle import step as ostep
from tests._cases import TOL_FP32, assert_step_grads_close, make_inputs, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.fixture(scope="module")
def g():
    import paper_2602_01872_amd as lib
    lib.load()
    return lib


def _weights(E, seed):
    rng = np.random.default_rng(seed)
    return torch.from_numpy(rng.uniform(0.05, 4.0, E).astype(np.float32))


@pytest.mark.parametrize("kind,N,E,K", [("uniform", 3000, 40000, 3), ("rmat", 1 << 13, 200000, 2), ("uniform", 64, 0, 2),
                                        ("dups", 50, 4000, 2)])
def test_weighted_partition_bit_exact(g, kind, N, E, K):
    print(f"[case] weighted partition {kind} N={N} E={E} K={K}", flush=True)
    if kind == "rmat":
        s, d = synth.rmat_graph(13, E, seed=41)
    else:
        s, d = synth.uniform_graph(N, E, seed=41)        # "dups": many equal (dst, src) pairs with different weights
    w = _weights(E, 42)
    for p in range(K):
        part = g.grp_partition_weighted(s.to(DEV), d.to(DEV), w.to(DEV), N, K, 7, p)
        want = ograph.partition(s.numpy(), d.numpy(), N, K, 7, p, weights=w.numpy())
        for key in ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in"):
            assert np.array_equal(part.array(key), want[key]), key
        got = part.weights()
        assert got is not None
        for key in ("csr_w", "csc_w", "w_local_in", "w_global_in"):
            assert np.array_equal(got[key], want[key]), key
        part.destroy()
    plain = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 7, 0)
    assert plain.weights() is None
    plain.destroy()


def test_weight_masses_of_hub_rows_over_twenty_binades(g):
    """Rows of more than 1024 weights are summed by a workgroup (256 runs added in order, then combined in
    order) instead of one thread; with weights spread over twenty binades the fp64 partial sums round, so
    those masses agree with the serial sum to fp64 rounding (1e-14 relative), the shorter rows exactly,
    and everything else of the partition bit for bit."""
    print("[case] weighted partition with hub rows, wide-range weights", flush=True)
    N, K = 4000, 2
    s, d = synth.uniform_graph(N, 60000, seed=51)
    es, _ = synth.uniform_graph(N, 30000, seed=52)
    ed = 7 + torch.arange(30000) % 3                       # three hubs with 10 000 extra in-edges each
    s, d = torch.cat([s, es]), torch.cat([d, ed])
    w = synth.edge_weights(s.numel(), 53, lo=1e-3, hi=1e3)
    seen_long = 0
    for p in range(K):
        part = g.grp_partition_weighted(s.to(DEV), d.to(DEV), w.to(DEV), N, K, 7, p)
        want = ograph.partition(s.numpy(), d.numpy(), N, K, 7, p, weights=w.numpy())
        for key in ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in"):
            assert np.array_equal(part.array(key), want[key]), key
        got = part.weights()
        assert np.array_equal(got["csr_w"], want["csr_w"]) and np.array_equal(got["csc_w"], want["csc_w"])
        for key, deg in (("w_local_in", want["d_local_in"]), ("w_global_in", want["d_global_in"])):
            short = deg <= 1024
            seen_long += int((~short).sum())
            assert np.array_equal(got[key][short], want[key][short]), key
            np.testing.assert_allclose(got[key][~short], want[key][~short], rtol=1e-14, atol=0.0)
        part.destroy()
    assert seen_long >= 3


def _step(g, part, dims, x, y, theta, mask, est, bf16=False):
    model = g.model_desc(g.ARCH_SAGE_MEAN, dims, g.DTYPE_BF16 if bf16 else g.DTYPE_FP32)
    opts = g.step_opts(estimator=est, full_graph=True)
    P = g.grp_param_count(model)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=DEV)
    grad = torch.full((P,), float("nan"), device=DEV)
    stats = g.new_stats(1)
    g.grp_train_step(part, model, opts, x.to(DEV), y.to(DEV), None if mask is None else mask.to(DEV), theta.to(DEV), ws,
                     grad, stats)
    torch.cuda.synchronize()
    return grad, stats


@pytest.mark.parametrize("dims,bf16,masked", [
    ([100, 256, 256, 47], False, False),     # aggregate-first twice, then transform-first
    ([36, 20, 52, 7], False, True),
    ([64, 128, 16], True, True),
])
def test_weighted_sage_step_matches_oracle(g, dims, bf16, masked):
    print(f"[case] weighted sage step dims={dims} bf16={bf16} masked={masked}", flush=True)
    scale, E, K = 14, 400000, 3
    N = 1 << scale
    s, d = synth.rmat_graph(scale, E, seed=2602018731)
    w = _weights(E, 5)
    part = g.grp_partition_weighted(s.to(DEV), d.to(DEV), w.to(DEV), N, K, 1, 0)
    op = ograph.partition(s.numpy(), d.numpy(), N, K, 1, 0, weights=w.numpy())
    assert int(op["d_local_in"].max()) > 600            # long rows take the chunked path with values
    n = part.n
    x, y, theta = make_inputs(n, dims, "sage", 13, bf16=bf16)
    mask = synth.train_mask(n, 0.3, 4) if masked else None
    grads, stats = [], []
    for est in (ocov.NONE, ocov.NODE_LEVEL):
        grad, st = _step(g, part, dims, x, y, theta, mask, est, bf16)

        def oracle_fn(relu_flip=None, near_kink=None, est=est):
            return ostep.train_step(op, "sage", dims, theta.double().numpy(), x.double().numpy(), y.numpy(),
                                    train_mask=None if mask is None else mask.numpy(), estimator=est,
                                    relu_flip=relu_flip, near_kink=near_kink)
        og, ost = assert_step_grads_close(grad.cpu().numpy(), oracle_fn, "sage", dims, TOL_FP32)
        got = g.read_stats(st)[0]
        assert int(got["S"]) == ost["S"] and int(got["nnz_used"]) == ost["nnz_used"]
        assert abs(float(got["sum_ratio"]) - ost["sum_ratio"]) <= 1e-9 * max(1.0, ost["sum_ratio"])
        assert abs(float(got["R"]) - ost["R"]) <= 1e-9 * max(1.0, ost["R"])
        assert abs(float(got["loss"]) - ost["loss"]) <= TOL_FP32 * abs(ost["loss"])
        grads.append((grad, og))
        stats.append((st, ost))
    # the aggregation kernel derives its factors from these statistics records
    P = grads[0][0].numel()
    ld = (P + 3) // 4 * 4
    buf = torch.zeros(2, ld, device=DEV)
    buf[0, :P], buf[1, :P] = grads[0][0], grads[0][0]
    st2 = torch.cat([stats[0][0], stats[0][0]])
    for est in (ocov.BATCH_MIN_DIST, ocov.SHRINKAGE):
        out = torch.zeros(P, device=DEV)
        g.grp_aggregate(buf, ld, st2, 2, P, est, out)
        torch.cuda.synchronize()
        want, c = ocov.aggregate([grads[0][1], grads[0][1]], [stats[0][1], stats[0][1]], est)
        assert 0 < c[0] < 1
        assert rel_err(out.cpu().numpy(), want) <= TOL_FP32
    part.destroy()


def test_constant_weights_reduce_to_the_plain_step_and_bad_input_is_refused(g):
    print("[case] weighted: uniform reduction and errors", flush=True)
    N, E, K, dims = 4000, 50000, 2, [32, 48, 8]
    s, d = synth.uniform_graph(N, E, seed=9)
    ones = torch.full((E,), 2.0)
    a = g.grp_partition_weighted(s.to(DEV), d.to(DEV), ones.to(DEV), N, K, 3, 1)
    b = g.grp_partition(s.to(DEV), d.to(DEV), N, K, 3, 1)
    x, y, theta = make_inputs(a.n, dims, "sage", 2)
    ga, sa = _step(g, a, dims, x, y, theta, None, ocov.NODE_LEVEL)
    gb, sb = _step(g, b, dims, x, y, theta, None, ocov.NODE_LEVEL)
    assert rel_err(ga.cpu().numpy(), gb.cpu().numpy()) <= 1e-5
    ra, rb = g.read_stats(sa)[0], g.read_stats(sb)[0]
    assert abs(float(ra["sum_ratio"]) - float(rb["sum_ratio"])) < 1e-9 and abs(float(ra["R"]) - float(rb["R"])) < 1e-6
    bad = ones.clone()
    bad[17] = 0.0
    with pytest.raises(g.GrappaError):
        g.grp_partition_weighted(s.to(DEV), d.to(DEV), bad.to(DEV), N, K, 3, 1)
    bad[17] = float("inf")
    with pytest.raises(g.GrappaError):
        g.grp_partition_weighted(s.to(DEV), d.to(DEV), bad.to(DEV), N, K, 3, 1)
    # other models and mini-batch mode refuse a weighted handle
    for arch, dd in ((g.ARCH_GCN, dims), (g.ARCH_GAT, dims)):
        with pytest.raises(g.GrappaError):
            g.grp_step_workspace_bytes(a, g.model_desc(arch, dd), g.step_opts(full_graph=True))
    seeds = torch.arange(8, dtype=torch.int32, device=DEV)
    with pytest.raises(g.GrappaError):
        g.grp_step_workspace_bytes(a, g.model_desc(g.ARCH_SAGE_MEAN, dims),
                                   g.step_opts(full_graph=False, seeds=seeds, fanouts=(3, 3)))
    a.destroy()
    b.destroy()
