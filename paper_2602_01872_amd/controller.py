"""Training controller: a thin wrapper over the library's host-side controller calls (grp_sweep_chunk,
grp_controller_*); the schedule and the switching decision are computed there."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import binding as _b


def sweep_pairs(n_chunks: int, super_epoch: int):
    """(base, swept) for every worker in the given super-epoch."""
    lib = _b.load()
    return [(i, int(lib.grp_sweep_chunk(i, super_epoch, n_chunks))) for i in range(n_chunks)]


class Controller:
    def __init__(self, total_epochs: int, n_chunks: int, threshold: float = 1.0, patience: int = 1 << 30):
        self.n_chunks = n_chunks
        h = C.c_void_p()
        _b._check(_b.load().grp_controller_create(total_epochs, n_chunks, threshold, patience, C.byref(h)))
        self._h = h

    def _state(self):
        se, ep = C.c_int64(), C.c_int64()
        _b._check(_b.load().grp_controller_state(self._h, C.byref(se), C.byref(ep)))
        return int(se.value), int(ep.value)

    @property
    def super_epoch(self) -> int:
        return self._state()[0]

    @property
    def epochs_per_super_epoch(self) -> int:
        return self._state()[1]

    def observe_step(self, c_hats) -> None:
        a = np.ascontiguousarray(np.asarray(list(c_hats), dtype=np.float32))
        _b._check(_b.load().grp_controller_observe(self._h, a.ctypes.data, int(a.size)))

    def observe_stats(self, records: np.ndarray) -> None:
        """``records``: host array of grp_step_stats (binding.STATS_DTYPE), one per active partition of the step."""
        a = np.ascontiguousarray(records)
        _b._check(_b.load().grp_controller_observe_stats(self._h, a.ctypes.data, int(a.size)))

    def end_epoch(self) -> bool:
        sw = C.c_int32()
        _b._check(_b.load().grp_controller_end_epoch(self._h, C.byref(sw)))
        return bool(sw.value)

    def pairs(self):
        return sweep_pairs(self.n_chunks, self.super_epoch)

    def __del__(self):
        try:
            _b.load().grp_controller_destroy(self._h)
        except Exception:
            pass
