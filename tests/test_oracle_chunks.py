"""Pins for oracle.chunks: brute-force construction on tiny graphs, reduction to the plain
hash partition (already pinned) when the swept chunk is the base chunk, the whole graph when
two chunks are combined out of two, the coverage guarantee (every cross-chunk edge co-resides
in some partition of the cycle), the in-degree accounting identity over a cycle, and the
controller's schedule."""
import numpy as np
import pytest

import synth
from oracle import chunks, graph

KEYS = ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in")


def _graph(N=300, E=3000, seed=5):
    s, d = synth.uniform_graph(N, E, seed=seed)
    return s.numpy(), d.numpy()


@pytest.mark.parametrize("c", [1, 2, 3, 5])
def test_swept_equal_base_is_the_plain_hash_partition(c):
    s, d = _graph()
    for b in range(c):
        a = chunks.partition_from_chunks(s, d, 300, c, 7, b, b)
        want = graph.partition(s, d, 300, c, 7, b)
        for k in KEYS:
            assert np.array_equal(a[k], want[k]), k
        assert a["base_mask"].all()


def test_two_of_two_chunks_is_the_whole_graph():
    s, d = _graph()
    a = chunks.partition_from_chunks(s, d, 300, 2, 3, 0, 1)
    whole = graph.partition(s, d, 300, 1, 0, 0)
    for k in KEYS:
        assert np.array_equal(a[k], whole[k]), k
    assert np.array_equal(a["d_local_in"], a["d_global_in"])
    assert np.array_equal(a["base_mask"], (chunks.chunk_of(300, 2, 3) == 0).astype(np.uint8))


def test_brute_force_tiny():
    rng = np.random.default_rng(1)
    N, E, c = 23, 90, 4
    s, d = rng.integers(0, N, E), rng.integers(0, N, E)
    ch = chunks.chunk_of(N, c, 11)
    for base, swept in ((0, 1), (2, 0), (3, 3)):
        p = chunks.partition_from_chunks(s, d, N, c, 11, base, swept)
        nodes = [v for v in range(N) if ch[v] in (base, swept)]
        assert list(p["l2g"]) == nodes
        loc = {v: i for i, v in enumerate(nodes)}
        rows = [[] for _ in nodes]
        for u, v in zip(s, d):
            if u in loc and v in loc:
                rows[loc[v]].append(loc[u])
        col = [x for r in rows for x in sorted(r)]
        assert list(p["col"]) == col
        assert list(np.diff(p["rowptr"])) == [len(r) for r in rows]
        assert list(p["d_global_in"]) == [int((d == v).sum()) for v in nodes]
        assert list(p["base_mask"]) == [1 if ch[v] == base else 0 for v in nodes]


@pytest.mark.parametrize("c", [2, 3, 4, 6])
def test_coverage_guarantee_and_degree_accounting(c):
    s, d = _graph(N=240, E=2600, seed=9)
    N = 240
    ch = chunks.chunk_of(N, c, 2)
    sched = chunks.sweep_schedule(c)
    assert len(sched) == c - 1
    seen = np.zeros(s.size, dtype=bool)
    base_only = {b: chunks.partition_from_chunks(s, d, N, c, 2, b, b) for b in range(c)}
    gained = {b: np.zeros(base_only[b]["n"], dtype=np.int64) for b in range(c)}
    for pairs in sched:
        assert sorted(b for b, _ in pairs) == list(range(c))
        assert sorted(w for _, w in pairs) == list(range(c))           # every chunk is swept exactly once
        assert all(b != w for b, w in pairs)
        for b, w in pairs:
            p = chunks.partition_from_chunks(s, d, N, c, 2, b, w)
            seen |= np.isin(ch[s], (b, w)) & np.isin(ch[d], (b, w))
            m = p["base_mask"].astype(bool)
            # in-neighbours of the base nodes that arrived with the swept chunk
            gained[b] += p["d_local_in"][m].astype(np.int64) - base_only[b]["d_local_in"]
    assert seen.all()                                                  # every edge co-resides somewhere
    for b in range(c):
        # over a cycle a base node meets each of its in-neighbours exactly once
        np.testing.assert_array_equal(base_only[b]["d_local_in"] + gained[b], base_only[b]["d_global_in"])


def test_controller_schedule():
    ctl = chunks.Controller(total_epochs=12, n_chunks=4)
    assert ctl.epochs_per_super_epoch == 4
    switches = [ctl.end_epoch() for _ in range(12)]
    assert switches == [False, False, False, True] * 3
    assert ctl.super_epoch == 3
    assert ctl.pairs() == chunks.sweep_schedule(4)[0]                  # the cycle repeats
    # early switch: the deficit stays above the threshold for `patience` steps
    ctl = chunks.Controller(total_epochs=100, n_chunks=3, threshold=0.4, patience=3)
    ctl.observe_step([0.5, 0.5]); ctl.observe_step([0.5]); assert not ctl.end_epoch()
    ctl.observe_step([0.7])                                            # deficit 0.3: streak broken
    ctl.observe_step([0.5]); ctl.observe_step([0.5]); assert not ctl.end_epoch()
    ctl.observe_step([0.2]); assert ctl.end_epoch()
    assert ctl.super_epoch == 1 and ctl.pairs() == chunks.sweep_schedule(3)[1]


@pytest.mark.parametrize("c", [2, 3, 4, 7, 12])
def test_every_pair_of_chunks_shares_a_partition_within_a_cycle(c):
    """The coverage guarantee, by brute force over the controller's own schedule: walking the controller through
    c - 1 super-epochs (one epoch each), every unordered pair of distinct chunks must have been base + swept of
    some worker, and no worker ever sweeps its own base chunk."""
    ctl = chunks.Controller(total_epochs=c - 1, n_chunks=c)
    assert ctl.epochs_per_super_epoch == 1
    seen = set()
    for t in range(c - 1):
        pairs = ctl.pairs()
        assert [b for b, _ in pairs] == list(range(c))
        assert all(b != s for b, s in pairs)
        seen |= {frozenset(p) for p in pairs}
        assert ctl.end_epoch() and ctl.super_epoch == t + 1
    assert seen == {frozenset((a, b)) for a in range(c) for b in range(a + 1, c)}


def test_controller_switch_points_worked_by_hand():
    """10 epochs over 4 chunks: ceil(10 / 3) = 4 epochs per super-epoch, so the switches fall after epochs 4 and 8
    (1-based); 7 epochs over 3 chunks: ceil(7 / 2) = 4: after epoch 4; a single chunk never divides by zero and
    switches every total_epochs epochs.  With patience 2 and threshold 0.25, deficits 0.3, 0.3 switch at the end
    of that epoch, 0.3, 0.2, 0.3 do not."""
    ctl = chunks.Controller(total_epochs=10, n_chunks=4)
    assert [e + 1 for e in range(10) if ctl.end_epoch()] == [4, 8]
    ctl = chunks.Controller(total_epochs=7, n_chunks=3)
    assert [e + 1 for e in range(7) if ctl.end_epoch()] == [4]
    ctl = chunks.Controller(total_epochs=5, n_chunks=1)
    assert ctl.epochs_per_super_epoch == 5 and ctl.pairs() == [(0, 0)]
    ctl = chunks.Controller(total_epochs=100, n_chunks=5, threshold=0.25, patience=2)
    ctl.observe_step([0.7]); ctl.observe_step([0.6, 0.8]); assert ctl.end_epoch()          # deficits 0.3, 0.3
    ctl.observe_step([0.7]); ctl.observe_step([0.8]); ctl.observe_step([0.7]); assert not ctl.end_epoch()   # 0.3, 0.2, 0.3


def test_assigned_chunks_generalise_the_random_split():
    """A caller-supplied assignment equal to the random split gives the same partitions; a contiguous
    range assignment (what a locality-preserving partitioner returns) is checked by brute force."""
    rng = np.random.default_rng(4)
    N, E, c = 90, 400, 3
    s, d = rng.integers(0, N, E), rng.integers(0, N, E)
    same = chunks.chunk_of(N, c, 11)
    for b in range(c):
        for w in range(c):
            a = chunks.partition_from_chunks(s, d, N, c, 11, b, w)
            z = chunks.partition_from_chunks(s, d, N, c, 0, b, w, assignment=same)
            for k in a:
                assert np.array_equal(a[k], z[k]), k
    ranges = (np.arange(N) * c // N).astype(np.int32)
    part = chunks.partition_from_chunks(s, d, N, c, 0, 2, 0, assignment=ranges)
    members = [v for v in range(N) if ranges[v] in (0, 2)]
    assert list(part["l2g"]) == members
    loc = {v: i for i, v in enumerate(members)}
    rows = [[] for _ in members]
    for u, v in zip(s.tolist(), d.tolist()):
        if u in loc and v in loc:
            rows[loc[v]].append(loc[u])
    assert list(part["col"]) == [x for r in rows for x in sorted(r)]
    assert list(part["base_mask"]) == [1 if ranges[v] == 2 else 0 for v in members]
    with pytest.raises(ValueError):
        chunks.partition_from_chunks(s, d, N, c, 0, 0, 1, assignment=np.full(N, 3))
