"""Training controller: the sweep schedule and the decision when to switch partitions
(host logic; the paper's "Training Controller and Partitions Switching" subsection and the
round-robin sweep of its "Repartitioning" paragraph).

With c chunks a cycle has c - 1 super-epochs; in super-epoch t worker i (base chunk i) sweeps
chunk (i + 1 + t) mod c.  A super-epoch lasts ceil(e / (c - 1)) epochs for e epochs in total; it
ends earlier once the coverage deficit 1 - c_hat (c_hat = the mean minimum-distance factor of a
step's active partitions) has stayed above `threshold` for `patience` consecutive steps.
"""
from __future__ import annotations


def sweep_pairs(n_chunks: int, super_epoch: int):
    """(base, swept) for every worker in the given super-epoch (the cycle repeats)."""
    if n_chunks <= 1:
        return [(0, 0)] * n_chunks
    t = super_epoch % (n_chunks - 1)
    return [(i, (i + 1 + t) % n_chunks) for i in range(n_chunks)]


class Controller:
    def __init__(self, total_epochs: int, n_chunks: int, threshold: float = 1.0, patience: int = 1 << 30):
        self.n_chunks = n_chunks
        cycle = max(1, n_chunks - 1)
        self.epochs_per_super_epoch = max(1, (total_epochs + cycle - 1) // cycle)
        self.threshold = threshold
        self.patience = patience
        self.super_epoch = 0
        self._epochs = 0
        self._streak = 0

    def observe_step(self, c_hats) -> None:
        c_hats = list(c_hats)
        deficit = 1.0 - sum(c_hats) / len(c_hats)
        self._streak = self._streak + 1 if deficit > self.threshold else 0

    def end_epoch(self) -> bool:
        self._epochs += 1
        if self._epochs >= self.epochs_per_super_epoch or self._streak >= self.patience:
            self.super_epoch += 1
            self._epochs = 0
            self._streak = 0
            return True
        return False

    def pairs(self):
        return sweep_pairs(self.n_chunks, self.super_epoch)
