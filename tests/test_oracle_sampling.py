"""Pins for oracle.sampling: the subset-growing scheme enumerated over every possible sequence of
draws (each subset equally often: exact uniformity), a hand-worked example, the draw scaling against
exact integer arithmetic, a per-row selection redone with Python integers, structural invariants of
the sampled blocks, reproducibility, selection frequencies of single edges and of pairs, and the
reduction to the full-graph step when the fanout covers every row."""
import itertools
import math

import numpy as np
import pytest

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


@pytest.mark.parametrize("d,f", [(5, 2), (6, 3), (7, 1), (4, 3), (6, 5), (8, 4)])
def test_subset_growing_is_exactly_uniform_by_enumeration(d, f):
    # all (d-f+1)(d-f+2)...d sequences of draws are equally likely; they must hit each of the
    # C(d, f) subsets equally often
    ranges = [range(d - f + t + 1) for t in range(f)]
    seen = {}
    for draws in itertools.product(*ranges):
        sub = tuple(sampling.grow_subset(d, draws))
        assert len(set(sub)) == f and all(0 <= j < d for j in sub) and list(sub) == sorted(sub)
        seen[sub] = seen.get(sub, 0) + 1
    assert len(seen) == math.comb(d, f)
    assert set(seen.values()) == {math.prod(len(r) for r in ranges) // math.comb(d, f)}


def test_subset_growing_worked_example():
    # d = 10, f = 3: tops 7, 8, 9.  Draw 2 -> {2}; draw 2 again -> taken, so 8; draw 9 -> 9.
    assert sampling.grow_subset(10, [2, 2, 9]) == [2, 8, 9]
    assert sampling.grow_subset(10, [7, 8, 9]) == [7, 8, 9]
    assert sampling.grow_subset(3, [0, 0]) == [0, 2]
    with pytest.raises(ValueError):
        sampling.grow_subset(10, [8, 0, 0])                   # first draw must lie in [0, 7]


def test_scale_draw_is_the_exact_integer_quotient():
    rng = np.random.default_rng(5)
    u = rng.integers(0, 2 ** 64, 4000, dtype=np.uint64)
    span = rng.integers(1, 2 ** 64, 4000, dtype=np.uint64)
    span[:2000] = rng.integers(1, 2 ** 31, 2000)
    u[:4] = [0, 2 ** 64 - 1, 2 ** 63, 1]
    got = sampling.scale_draw(u, span)
    for g, a, b in zip(got.tolist(), u.tolist(), span.tolist()):
        assert g == (a * b) >> 64 and 0 <= g < b


def _mix_int(x):
    z = (x + 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & (2 ** 64 - 1)
    return z ^ (z >> 31)


def test_layer_sample_matches_selection_redone_with_python_integers():
    part = _part(scale=8, E=5000)
    dst = np.array([5, 0, 17, 3, 40, 41])
    f = 4
    edst, esrc = sampling.sample_layer(part, dst, f, sampler_seed=7, batch_id=2, layer=1)
    got = [[] for _ in dst]
    for e, u in zip(edst.tolist(), esrc.tolist()):
        got[e].append(u)
    some_sampled = False
    for i, v in enumerate(dst.tolist()):
        b, e = int(part["rowptr"][v]), int(part["rowptr"][v + 1])
        row = part["col"][b:e].tolist()
        d = len(row)
        if d <= f:
            want = row
        else:
            some_sampled = True
            h = _mix_int(_mix_int(_mix_int(_mix_int(7) ^ 2) ^ 1) ^ int(part["l2g"][v]))
            chosen = set()
            for t in range(f):
                top = d - f + t
                r = (_mix_int(h ^ t) * (top + 1)) >> 64
                chosen.add(top if r in chosen else r)
            want = [row[j] for j in sorted(chosen)]
        assert got[i] == want
        assert len(got[i]) == min(f, d)
    assert some_sampled


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
    # one hub row with 40 distinct in-edges, fanout 10: each edge kept ~ 1/4 of the batches and each
    # pair of edges together ~ (10 * 9) / (40 * 39) of them
    src = np.arange(1, 41)
    dst = np.zeros(40, dtype=np.int64)
    part = graph.local_graph_from_edges(src, dst, 41)
    counts = np.zeros(41)
    pairs = np.zeros((41, 41))
    B = 4000
    for b in range(B):
        _, esrc = sampling.sample_layer(part, np.array([0]), 10, 3, b, 0)
        assert esrc.size == 10 and len(set(esrc.tolist())) == 10
        counts[esrc] += 1
        pairs[np.ix_(esrc, esrc)] += 1
    freq = counts[1:] / B
    sigma = (0.25 * 0.75 / B) ** 0.5
    assert np.abs(freq - 0.25).max() < 5 * sigma
    pp = 90.0 / 1560.0
    pf = pairs[1:, 1:][np.triu_indices(40, 1)] / B
    assert np.abs(pf - pp).max() < 5 * (pp * (1 - pp) / B) ** 0.5


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


def test_epoch_seed_order_is_a_fresh_permutation_of_the_training_nodes():
    part = _part(scale=9, E=9000)
    n = part["n"]
    mask = (np.arange(n) % 3 != 0).astype(np.uint8)
    a = sampling.epoch_seed_order(part, mask, 11, 0)
    assert sorted(a.tolist()) == np.flatnonzero(mask).tolist()          # each training node exactly once
    assert a.tolist() == sampling.epoch_seed_order(part, mask, 11, 0).tolist()
    b = sampling.epoch_seed_order(part, mask, 11, 1)
    assert sorted(b.tolist()) == sorted(a.tolist()) and a.tolist() != b.tolist()
    assert sampling.epoch_seed_order(part, mask, 12, 0).tolist() != a.tolist()
    full = sampling.epoch_seed_order(part, None, 11, 0)
    assert sorted(full.tolist()) == list(range(n))
    assert sampling.epoch_seed_order(part, np.zeros(n, dtype=np.uint8), 11, 0).size == 0
    # the key is a function of the global id: a node keeps its rank relative to another whatever else is masked
    both = [v for v in full.tolist() if mask[v]]
    assert both == a.tolist()
    # and the key itself, redone with Python integers
    h = _mix_int(_mix_int(11) ^ 0)
    keys = [_mix_int(h ^ int(part["l2g"][v])) for v in a.tolist()]
    assert keys == sorted(keys)


def test_epoch_positions_are_spread_evenly():
    # over many epochs every node's position in the order is uniform: mean (n-1)/2, no node favoured
    part = graph.local_graph_from_edges(np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64), 50)
    pos = np.zeros(50)
    E = 600
    for e in range(E):
        order = sampling.epoch_seed_order(part, None, 5, e)
        pos[order] += np.arange(50)
    mean = pos / E
    sigma = ((50 ** 2 - 1) / 12.0 / E) ** 0.5
    assert np.abs(mean - 24.5).max() < 5 * sigma
