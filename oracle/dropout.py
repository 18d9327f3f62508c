"""CPU checker (test infrastructure only): seeded dropout on the FC worker's hidden activations.

The CNNs of the paper's evaluation (Sec. 6.1 "Setup": AlexNet, VGG) drop hidden FC units during
training; the paper does not describe the operation, so it is taken as published (inverted
dropout): every unit is kept with probability 1 - p, kept units are scaled by 1/(1 - p), and
the gradient passes through the same mask and scale.

Random numbers come from a counter-based generator so that both sides of a comparison draw the
same mask without exchanging it: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel
random numbers: as easy as 1, 2, 3", SC 2011).  Element i of a tensor takes word i mod 4 of the
block whose 128-bit counter is (i div 4 as 64 bits, stream as 64 bits) under the 64-bit key `seed`;
`stream` tells layers and iterations apart.  A unit is kept iff its 32-bit word is >= floor(p * 2^32).
"""
from __future__ import annotations

import numpy as np

_M0, _M1 = 0xD2511F53, 0xCD9E8D57          # round multipliers
_W0, _W1 = 0x9E3779B9, 0xBB67AE85          # key schedule increments (golden ratio, sqrt(3) - 1)
_MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """One block: counter (c0, c1, c2, c3) and key (k0, k1) as Python ints -> four 32-bit words."""
    c0, c1, c2, c3 = [int(v) & _MASK for v in counter]
    k0, k1 = [int(v) & _MASK for v in key]
    for rnd in range(10):
        if rnd:
            k0, k1 = (k0 + _W0) & _MASK, (k1 + _W1) & _MASK
        p0, p1 = _M0 * c0, _M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & _MASK, p1 & _MASK, ((p0 >> 32) ^ c3 ^ k1) & _MASK, p0 & _MASK
    return c0, c1, c2, c3


def random_words(numel: int, seed: int, stream: int) -> np.ndarray:
    """uint32 [numel]: the word every element draws (vectorised form of philox4x32_10 over the blocks)."""
    nblk = (numel + 3) // 4
    idx = np.arange(nblk, dtype=np.uint64)
    c = [idx & np.uint64(_MASK), idx >> np.uint64(32),
         np.full(nblk, stream & _MASK, np.uint64), np.full(nblk, (stream >> 32) & _MASK, np.uint64)]
    k0, k1 = seed & _MASK, (seed >> 32) & _MASK
    m = np.uint64(_MASK)
    for rnd in range(10):
        if rnd:
            k0, k1 = (k0 + _W0) & _MASK, (k1 + _W1) & _MASK
        p0, p1 = np.uint64(_M0) * c[0], np.uint64(_M1) * c[2]
        c = [((p1 >> np.uint64(32)) ^ c[1] ^ np.uint64(k0)) & m, p1 & m, ((p0 >> np.uint64(32)) ^ c[3] ^ np.uint64(k1)) & m, p0 & m]
    return np.stack(c, axis=1).reshape(-1)[:numel].astype(np.uint32)


def keep_threshold(p: float) -> int:
    """Words below this value drop their unit; p is taken at float32 precision (the type it is passed in)."""
    p = float(np.float32(p))
    assert 0.0 <= p < 1.0
    return int(np.floor(p * 4294967296.0))


def keep_mask(numel: int, p: float, seed: int, stream: int) -> np.ndarray:
    return random_words(numel, seed, stream) >= np.uint32(keep_threshold(p))


def dropout_fwd(x: np.ndarray, p: float, seed: int, stream: int) -> np.ndarray:
    keep = keep_mask(x.size, p, seed, stream).reshape(x.shape)
    scale = 1.0 / (1.0 - float(np.float32(p)))
    return np.where(keep, x.astype(np.float64) * scale, 0.0).astype(x.dtype)


def dropout_bwd(dy: np.ndarray, p: float, seed: int, stream: int) -> np.ndarray:
    """The operation is linear with a diagonal matrix, so its transpose is itself."""
    return dropout_fwd(dy, p, seed, stream)


def fc_stream(step: int, layer: int) -> int:
    """Stream number of the mask over the output of FC layer `layer` (0-based) in iteration `step`."""
    assert 0 <= layer < 256 and step >= 0
    return (int(step) << 8) | int(layer)
