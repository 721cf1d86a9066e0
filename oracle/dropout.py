"""Dropout masks of the hidden layers (oracle; test infrastructure).

The paper trains with dropout 0.5 (experimental setup, hyper-parameters) and fixes nothing
else about it.  Reading used here:
  * inverted dropout on the output of every layer but the last, after the ReLU (a residual
    layer drops the activation before the skip is added): a' = a * keep / (1 - rate);
  * the keep decision of element (node v, column f) of layer l is a pure function of
    (seed, batch_id, l, global id of v, f), so it does not depend on which partition holds
    v or on the order of evaluation:
        key_l  = mix(seed + (batch_id * 16 + l + 1) * GAMMA)
        bits   = mix(key_l + (gid(v) * F_l + f + 1) * GAMMA) >> 40          (24 bits)
        keep   = bits >= floor(rate * 2^24)
    in wrapping uint64 arithmetic; mix and GAMMA are SplitMix64's output function and
    increment (Steele, Lea, Flood 2014), written out again in this module;
  * rate is an fp32 number in [0, 1); 1 / (1 - rate) is taken in fp32 too (the scale every
    kept element is multiplied by is part of the model, not of the arithmetic).
"""
from __future__ import annotations

import numpy as np

GAMMA = np.uint64(0x9E3779B97F4A7C15)
MAX_LAYERS = 16


def _mix(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def layer_key(seed: int, batch_id: int, layer: int) -> np.uint64:
    with np.errstate(over="ignore"):
        c = np.uint64((int(batch_id) * MAX_LAYERS + int(layer) + 1) % (1 << 64)) * GAMMA
        return _mix(np.uint64(int(seed) % (1 << 64)) + c)


def threshold(rate) -> int:
    r = np.float32(rate)
    if not (0.0 <= r < 1.0):
        raise ValueError("dropout rate must lie in [0, 1)")
    return int(np.floor(np.float64(r) * 16777216.0))


def scale(rate) -> float:
    return float(np.float32(1.0) / (np.float32(1.0) - np.float32(rate)))


def keep_mask(seed: int, batch_id: int, layer: int, gids, width: int, rate) -> np.ndarray:
    """bool [len(gids), width]: which elements of layer ``layer``'s output survive."""
    gids = np.asarray(gids, dtype=np.uint64)
    key = layer_key(seed, batch_id, layer)
    with np.errstate(over="ignore"):
        counter = gids[:, None] * np.uint64(width) + np.arange(width, dtype=np.uint64)[None, :] + np.uint64(1)
        bits = _mix(key + counter * GAMMA) >> np.uint64(40)
    return bits >= np.uint64(threshold(rate))


def layer_factors(seed: int, batch_id: int, gids, dims, rate) -> list:
    """Per hidden layer l (0 .. k-2) the array keep * 1/(1-rate), fp64; [] when rate == 0."""
    if np.float32(rate) == 0.0:
        return []
    s = scale(rate)
    return [keep_mask(seed, batch_id, l, gids, dims[l + 1], rate).astype(np.float64) * s
            for l in range(len(dims) - 2)]
