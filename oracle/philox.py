"""Minibatch row sampling zeta_i^t for the oracle (test infrastructure).

The paper only asks that each worker observe unbiased, independent stochastic
gradients (Section 1, below eq. 1).  The reading taken here: at iteration t
worker i draws B rows of its own n-row shard iid uniformly *with replacement*.
So that no sampler state has to be stored or exchanged, the draw is a pure
function of (seed, worker, iteration, slot) through the counter-based generator
Philox4x32-10 as published by Salmon, Moraes, Dror and Shaw, "Parallel random
numbers: as easy as 1, 2, 3" (SC'11):

    counter = (slot // 4, t mod 2^32, t >> 32, worker)     four 32-bit words
    key     = (seed mod 2^32, seed >> 32)                  two  32-bit words
    word    = Philox4x32-10(counter, key)[slot % 4]
    row     = word >> (32 - log2 n)                        n a power of two

Taking the top log2(n) bits of a uniform 32-bit word is exactly uniform on
[0, n) -- no modulo bias and no rejection loop.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)   # multiplier applied to counter word 0
_M1 = np.uint64(0xCD9E8D57)   # multiplier applied to counter word 2
_W0 = 0x9E3779B9              # key word 0 increment per round (golden ratio)
_W1 = 0xBB67AE85              # key word 1 increment per round (sqrt(3) - 1)
_MASK = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds.

    counter: integer array [..., 4]; key: integer array [..., 2] (broadcastable).
    Returns uint32 array [..., 4].
    """
    c = np.asarray(counter).astype(np.uint64) & _MASK
    k = np.asarray(key).astype(np.uint64) & _MASK
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = k[..., 0], k[..., 1]
    for r in range(10):
        if r > 0:                                   # key schedule between rounds
            k0 = (k0 + np.uint64(_W0)) & _MASK
            k1 = (k1 + np.uint64(_W1)) & _MASK
        p0 = _M0 * c0                               # 64-bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK
        hi1, lo1 = p1 >> _SH32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0
    out = np.stack(np.broadcast_arrays(c0, c1, c2, c3), axis=-1)
    return out.astype(np.uint32)


def sample_rows(seed: int, worker: int, t: int, batch: int, rows_per_worker: int) -> np.ndarray:
    """The B row indices worker `worker` uses at iteration `t` (t counts from 1)."""
    n = int(rows_per_worker)
    if n <= 0 or (n & (n - 1)) != 0:
        raise ValueError("rows_per_worker must be a power of two")
    log2n = n.bit_length() - 1
    n_blocks = (batch + 3) // 4
    ctr = np.zeros((n_blocks, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(n_blocks, dtype=np.uint64)
    ctr[:, 1] = int(t) & 0xFFFFFFFF
    ctr[:, 2] = (int(t) >> 32) & 0xFFFFFFFF
    ctr[:, 3] = int(worker)
    key = np.array([int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF], dtype=np.uint64)
    words = philox4x32_10(ctr, key).reshape(-1)[:batch].astype(np.uint64)
    if log2n == 0:
        return np.zeros(batch, dtype=np.int64)
    return (words >> np.uint64(32 - log2n)).astype(np.int64)
