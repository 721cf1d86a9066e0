"""Host logic of the product's training controller against the oracle's (written separately)
and against the schedule's defining properties."""
import numpy as np
import pytest

from oracle import chunks as ochunks


def _product():
    # the controller module has no dependency on the HIP library
    import importlib.util
    import os
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2602_01872_amd", "controller.py")
    spec = importlib.util.spec_from_file_location("grp_controller", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


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
