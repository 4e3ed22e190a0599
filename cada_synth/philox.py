"""Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
as 1, 2, 3", SC'11) in numpy, and the counter-based row recipe built on it.

The high-dimensional logistic workload (M=100, p=65536, 4096 samples per
worker) is 107 GB of features: it never exists on the host.  Every element is
instead a pure function of (seed, worker m, sample n, column j), so any row can
be regenerated anywhere.  This file is the host-side definition; the device
generator and the C generator implement the same published function and are
compared with it bit for bit in the tests.

Element recipe ("counter_gauss"):
  words (w0,w1,w2,w3) = philox4x32_10(counter=(j//2, n, m, 0), key=(seed, KEY1))
  column j even uses (w0,w1), odd uses (w2,w3)
  ih  = sum of the four 16-bit halves of the two words - 131070  (Irwin-Hall,
        exact integer, mean 0, standard deviation IH_STD)
  x   = fl32( fl32(float(ih) * scale) + shift[m, j] ),  scale = fl32(1/(IH_STD*sqrt(p)))
  t_j = (philox(counter=(j,0,0,1))[0] mod 255) - 127      planted integer direction
  y   = +1 if sum_j ih*t_j >= 0 else -1                   (exact int64 arithmetic)
"""
from __future__ import annotations

import numpy as np

M0 = np.uint64(0xD2511F53)
M1 = np.uint64(0xCD9E8D57)
W0 = 0x9E3779B9
W1 = 0xBB67AE85
KEY1 = 0x43414441
MASK32 = np.uint64(0xFFFFFFFF)
# standard deviation of the sum of four independent uniform integers on [0, 65535]
IH_STD = float(np.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0))


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32.  Counters are array-likes of uint32 (broadcast
    against each other), keys are Python ints.  Returns four uint32 arrays."""
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3)))
    c0, c1, c2, c3 = (c.copy() for c in (c0, c1, c2, c3))
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for r in range(10):
        if r > 0:
            k0 = (k0 + W0) & 0xFFFFFFFF
            k1 = (k1 + W1) & 0xFFFFFFFF
        p0 = M0 * c0            # 32x32 -> 64 bit products, exact in uint64
        p1 = M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & MASK32
        n0 = hi1 ^ c1 ^ np.uint64(k0)
        n2 = hi0 ^ c3 ^ np.uint64(k1)
        c0, c1, c2, c3 = n0, lo1, n2, lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def scale_for(p: int) -> np.float32:
    return np.float32(1.0 / (IH_STD * np.sqrt(float(p))))


def teacher_direction(seed: int, p: int) -> np.ndarray:
    """Integer planted direction t_j in [-127, 127], shape [p], int64."""
    j = np.arange(p, dtype=np.uint64)
    w0, _, _, _ = philox4x32_10(j, 0, 0, 1, seed, KEY1)
    return (w0.astype(np.int64) % 255) - 127


def irwin_hall_rows(seed: int, m: int, rows: np.ndarray, p: int) -> np.ndarray:
    """Integer Irwin-Hall values ih[r, j] (int32) for samples ``rows`` of worker m."""
    assert p % 2 == 0
    rows = np.asarray(rows, dtype=np.uint64).reshape(-1, 1)
    jp = np.arange(p // 2, dtype=np.uint64).reshape(1, -1)
    w0, w1, w2, w3 = philox4x32_10(jp, rows, m, 0, seed, KEY1)

    def halves(w):
        w = w.astype(np.int64)
        return (w & 0xFFFF) + (w >> 16)

    ih = np.empty((rows.shape[0], p), dtype=np.int32)
    ih[:, 0::2] = halves(w0) + halves(w1) - 131070
    ih[:, 1::2] = halves(w2) + halves(w3) - 131070
    return ih


def counter_rows(seed: int, m: int, rows: np.ndarray, p: int, shift_m: np.ndarray):
    """Features (float32 [R, p]) and labels (float32 [R], +-1) for samples
    ``rows`` of worker ``m``.  ``shift_m`` is the worker's float32 mean shift."""
    ih = irwin_hall_rows(seed, m, rows, p)
    x = ih.astype(np.float32) * scale_for(p)          # one rounding
    x = x + shift_m.astype(np.float32)[None, :]       # second rounding
    t = teacher_direction(seed, p)
    score = ih.astype(np.int64) @ t
    y = np.where(score >= 0, 1.0, -1.0).astype(np.float32)
    return x.astype(np.float32), y
