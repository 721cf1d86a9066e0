"""MI355X-native hot path of gradient-only GNN training (Grappa): Python binding.

A thin ctypes layer over ``libgrappa_hip.so`` (C ABI in ``include/grappa.h``).  It only
marshals arguments: device memory comes from torch tensors (``data_ptr()``), streams from
``torch.cuda.current_stream()``; every step of the path runs in the library's HIP kernels.
There is no CPU fallback: importing ``binding`` without the built library raises.
"""
from .binding import *  # noqa: F401,F403
from .controller import Controller, sweep_pairs  # noqa: F401
from .loop import MiniBatchTrainer, PhaseParallelTrainer, SweepingTrainer  # noqa: F401
