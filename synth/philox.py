"""Philox4x32-10 counter-based random numbers (Salmon, Moraes, Dror, Shaw, SC'11).

Input generation only: this module holds no arithmetic of the verification
method.  The uniforms it produces are handed, as plain arrays, to both the
CPU oracle and the HIP path, so neither side draws random numbers itself.

Vectorised numpy; one call produces four 32-bit words per counter.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9  # key schedule increments (golden ratio, sqrt(3)-1)
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SHIFT = np.uint64(32)


def philox4x32_10(counter: np.ndarray, key: tuple[int, int]) -> np.ndarray:
    """counter: uint32 array [..., 4]; key: two 32-bit ints.  Returns uint32 [..., 4]."""
    c = np.asarray(counter, dtype=np.uint32)
    if c.shape[-1] != 4:
        raise ValueError("counter must have a trailing dimension of 4")
    c0 = c[..., 0].astype(np.uint64)
    c1 = c[..., 1].astype(np.uint64)
    c2 = c[..., 2].astype(np.uint64)
    c3 = c[..., 3].astype(np.uint64)
    k0 = int(key[0]) & 0xFFFFFFFF
    k1 = int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0  # 64-bit products of 32-bit operands: no overflow in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SHIFT, p0 & _MASK
        hi1, lo1 = p1 >> _SHIFT, p1 & _MASK
        n0 = hi1 ^ c1 ^ np.uint64(k0)
        n2 = hi0 ^ c3 ^ np.uint64(k1)
        c0, c1, c2, c3 = n0, lo1, n2, lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    out = np.stack([c0, c1, c2, c3], axis=-1)
    return out.astype(np.uint32)


def uniforms(seed: int, n_rows: int, stream: int = 0, step: int = 0) -> np.ndarray:
    """float32 [n_rows, 2] in [0, 1): word >> 8 scaled by 2**-24, so every value is
    an exact multiple of 2**-24 and strictly below one.

    Counter = (row, step, stream, 0); key = (seed low word, seed high word).
    Column 0 is the acceptance draw, column 1 the resampling draw.
    """
    ctr = np.zeros((n_rows, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(n_rows, dtype=np.uint32)
    ctr[:, 1] = np.uint32(step & 0xFFFFFFFF)
    ctr[:, 2] = np.uint32(stream & 0xFFFFFFFF)
    words = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    u = (words[:, :2] >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)
    return np.ascontiguousarray(u)


def uniform_block(seed: int, count: int, stream: int = 0) -> np.ndarray:
    """float64 [count] in [0,1) with 24-bit resolution, for Monte-Carlo tests."""
    n_ctr = (count + 3) // 4
    ctr = np.zeros((n_ctr, 4), dtype=np.uint32)
    idx = np.arange(n_ctr, dtype=np.uint64)
    ctr[:, 0] = (idx & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    ctr[:, 1] = (idx >> np.uint64(32)).astype(np.uint32)
    ctr[:, 2] = np.uint32(stream & 0xFFFFFFFF)
    ctr[:, 3] = np.uint32(1)
    words = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)).reshape(-1)
    return (words[:count] >> np.uint32(8)).astype(np.float64) * 2.0 ** -24
