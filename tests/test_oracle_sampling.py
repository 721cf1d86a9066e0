"""Pins for oracle.sampling: structural invariants of the sampled blocks, a brute-force
per-row selection written with Python loops, reproducibility, near-uniform selection
frequencies, and the reduction to the full-graph step when the fanout covers every row."""
import numpy as np

import synth
from oracle import coverage as cov
from oracle import graph, sampling, step


def _part(N=300, E=6000, K=2, scale=None):
    if scale is None:
        s, d = synth.uniform_graph(N, E, seed=17)
    else:
        s, d = synth.rmat_graph(scale, E, seed=17)
        N = 1 << scale
    return graph.partition(s.numpy(), d.numpy(), N, K, 4, 0)


def test_layer_sample_matches_brute_force_selection():
    part = _part(scale=8, E=5000)
    dst = np.array([5, 0, 17, 3, 40, 41])
    f = 4
    edst, esrc = sampling.sample_layer(part, dst, f, sampler_seed=7, batch_id=2, layer=1)
    got = [[] for _ in dst]
    for e, u in zip(edst.tolist(), esrc.tolist()):
        got[e].append(u)
    for i, v in enumerate(dst.tolist()):
        b, e = int(part["rowptr"][v]), int(part["rowptr"][v + 1])
        row = part["col"][b:e].tolist()
        if len(row) <= f:
            want = row
        else:
            keys = [int(sampling.edge_keys(7, 2, 1, part["l2g"][v], j)) for j in range(len(row))]
            pick = sorted(sorted(range(len(row)), key=lambda j: (keys[j], j))[:f])
            want = [row[j] for j in pick]
        assert got[i] == want
        assert len(got[i]) == min(f, len(row))


def test_blocks_are_well_formed_and_reproducible():
    part = _part(scale=9, E=20000)
    seeds = np.array([3, 99, 100, 7, 200])
    fan = (6, 4, 2)
    blocks, inputs = sampling.sample_blocks(part, seeds, fan, 7, 0)
    blocks2, inputs2 = sampling.sample_blocks(part, seeds, fan, 7, 0)
    assert inputs.tolist() == inputs2.tolist()
    dst_nodes = seeds
    for layer in (2, 1, 0):
        b = blocks[layer]
        assert b["esrc"].tolist() == blocks2[layer]["esrc"].tolist()
        assert b["n_dst"] == dst_nodes.size
        src_nodes = b["src_nodes"]
        assert src_nodes[:b["n_dst"]].tolist() == dst_nodes.tolist()
        assert len(set(src_nodes.tolist())) == src_nodes.size
        new = src_nodes[b["n_dst"]:]
        assert (np.diff(new) > 0).all()
        deg = np.bincount(b["edst"], minlength=b["n_dst"])
        dl = part["d_local_in"][dst_nodes]
        assert deg.tolist() == np.minimum(dl, fan[layer]).tolist()
        for e in range(b["esrc"].size):                       # every sampled edge is a local edge
            v = dst_nodes[b["edst"][e]]
            u = src_nodes[b["esrc"][e]]
            row = part["col"][part["rowptr"][v]:part["rowptr"][v + 1]]
            assert u in row
        dst_nodes = src_nodes
    assert inputs.tolist() == dst_nodes.tolist()
    other, _ = sampling.sample_blocks(part, seeds, fan, 7, 1)
    assert any(other[l]["esrc"].tolist() != blocks[l]["esrc"].tolist() for l in range(3))


def test_selection_is_close_to_uniform():
    # one hub row with 40 distinct in-edges, fanout 10: each edge kept ~ 1/4 of the batches
    src = np.arange(1, 41)
    dst = np.zeros(40, dtype=np.int64)
    part = graph.local_graph_from_edges(src, dst, 41)
    counts = np.zeros(41)
    B = 2000
    for b in range(B):
        _, esrc = sampling.sample_layer(part, np.array([0]), 10, 3, b, 0)
        assert esrc.size == 10 and len(set(esrc.tolist())) == 10
        counts[esrc] += 1
    freq = counts[1:] / B
    sigma = (0.25 * 0.75 / B) ** 0.5
    assert np.abs(freq - 0.25).max() < 5 * sigma


def test_full_fanout_minibatch_equals_full_graph_loss_on_seeds():
    part = _part(N=120, E=700, K=2)
    n = part["n"]
    dims = [5, 6, 6, 3]
    x = synth.normal_matrix(n, 5, 3).double().numpy()
    y = synth.labels(n, 3, 3).numpy()
    theta = synth.model_weights("sage", dims, 3).double().numpy()
    seeds = np.array([4, 1, 30, 31, 17])
    big = int(part["d_local_in"].max()) + 1
    mb = dict(seeds=seeds, fanouts=(big, big, big), sampler_seed=1, batch_id=0)
    mask = np.zeros(n, dtype=np.uint8)
    mask[seeds] = 1
    for est in (cov.NONE, cov.NODE_LEVEL):
        g_mb, st_mb = step.train_step(part, "sage", dims, theta, x, y, estimator=est, minibatch=mb)
        g_fg, st_fg = step.train_step(part, "sage", dims, theta, x, y, train_mask=mask, estimator=est)
        np.testing.assert_allclose(g_mb, g_fg, rtol=1e-10, atol=1e-14)
        assert abs(st_mb["loss"] - st_fg["loss"]) < 1e-12
        assert st_mb["S"] == st_fg["S"] == 5
        assert abs(st_mb["sum_ratio"] - st_fg["sum_ratio"]) < 1e-12
        assert abs(st_mb["R"] - st_fg["R"]) < 1e-9            # |S_v| = d_local when nothing is cut


def test_minibatch_shrinkage_uses_sampled_counts():
    part = _part(scale=8, E=6000)
    seeds = np.arange(20)
    dims = [3, 4, 2]
    n = part["n"]
    x = synth.normal_matrix(n, 3, 1).double().numpy()
    y = synth.labels(n, 2, 1).numpy()
    theta = synth.model_weights("sage", dims, 1).double().numpy()
    mb = dict(seeds=seeds, fanouts=(5, 3), sampler_seed=2, batch_id=5)
    _, st = step.train_step(part, "sage", dims, theta, x, y, minibatch=mb)
    dl = part["d_local_in"][seeds].astype(float)
    dg = part["d_global_in"][seeds].astype(float)
    lit = sum((dg[i] / dl[i] - 1.0) * min(3, dl[i]) for i in range(20) if dl[i] > 0)
    assert abs(st["R"] - lit) < 1e-9
    blocks, _ = sampling.sample_blocks(part, seeds, (5, 3), 2, 5)
    assert st["nnz_used"] == blocks[0]["esrc"].size + blocks[1]["esrc"].size
