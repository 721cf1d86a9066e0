"""The library's host-side controller calls against the oracle's controller (written separately) and against the
schedule's defining properties."""
import numpy as np
import pytest

from oracle import chunks as ochunks


def _product():
    # the controller calls are host arithmetic: they need the built library but no GPU
    from paper_2602_01872_amd import controller
    return controller


@pytest.mark.parametrize("c", [1, 2, 3, 5, 8])
def test_sweep_pairs_match_the_oracle_schedule(c):
    ctl = _product()
    sched = ochunks.sweep_schedule(c)
    for t in range(3 * max(1, c - 1)):
        assert ctl.sweep_pairs(c, t) == sched[t % len(sched)]


@pytest.mark.parametrize("total,c,thr,pat", [(12, 4, 1.0, 1 << 30), (10, 3, 0.4, 3), (7, 5, 0.2, 2), (5, 2, 0.5, 1)])
def test_controller_decisions_match_the_oracle(total, c, thr, pat):
    mod = _product()
    a = mod.Controller(total, c, thr, pat)
    b = ochunks.Controller(total, c, thr, pat)
    assert a.epochs_per_super_epoch == b.epochs_per_super_epoch
    rng = np.random.default_rng(total * 100 + c)
    for epoch in range(3 * total):
        for _ in range(rng.integers(1, 4)):
            c_hats = rng.uniform(0.2, 1.0, size=rng.integers(1, 4)).tolist()
            a.observe_step(c_hats)
            b.observe_step(c_hats)
        assert a.end_epoch() == b.end_epoch()
        assert a.super_epoch == b.super_epoch
        assert a.pairs() == b.pairs()


def test_observe_stats_derives_the_factor_from_the_records():
    mod = _product()
    from paper_2602_01872_amd import binding
    a = mod.Controller(10, 3, 0.4, 2)
    b = ochunks.Controller(10, 3, 0.4, 2)
    rng = np.random.default_rng(5)
    for epoch in range(12):
        for _ in range(3):
            rec = np.zeros(2, dtype=binding.STATS_DTYPE)
            rec["S"] = rng.integers(0, 50, size=2)
            rec["sum_ratio"] = rng.uniform(0.0, 1.0, size=2) * rec["S"]
            a.observe_stats(rec)
            b.observe_step([float(r["sum_ratio"]) / int(r["S"]) if int(r["S"]) > 0 else 1.0 for r in rec])
        assert a.end_epoch() == b.end_epoch()
        assert a.super_epoch == b.super_epoch


def test_sweep_chunk_and_super_epoch_length_reject_bad_arguments():
    from paper_2602_01872_amd import binding
    lib = binding.load()
    assert lib.grp_sweep_chunk(0, 0, 0) == -1 and lib.grp_sweep_chunk(3, 0, 3) == -1 and lib.grp_sweep_chunk(0, -1, 3) == -1
    assert lib.grp_super_epoch_epochs(-1, 3) == -1 and lib.grp_super_epoch_epochs(5, 0) == -1
    assert lib.grp_super_epoch_epochs(10, 4) == 4 and lib.grp_super_epoch_epochs(0, 4) == 1 and lib.grp_super_epoch_epochs(7, 1) == 7
