"""CPU oracle for the symmetry-aware packing of the statistics -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Sec. 5.2 ("Symmetry-aware communication"): a symmetric N x N statistic is communicated as its upper
triangle, N (N + 1) / 2 elements.  Plain numpy / Python written from that statement; only the tests
may import this module and it imports nothing from the GPU package.

Readings where the paper is silent (the same ones the library takes):
  * order inside the buffer: the rows of the upper triangle one after the other, row r contributing
    X[r][r], X[r][r+1], ..., X[r][N-1];
  * several statistics are packed back to back in the order given;
  * optional 16-bit storage is bfloat16, rounded to nearest, ties to even (NaN stays NaN);
  * unpacking writes both triangles (element (r, c) and (c, r) from the packed (r, c), r <= c), so
    the result is exactly symmetric; packing never looks at the strictly lower triangle.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def packed_elems(dims: Sequence[int]) -> int:
    return int(sum(int(d) * (int(d) + 1) // 2 for d in dims))


def pack_upper(mats: Sequence[np.ndarray]) -> np.ndarray:
    """float32 buffer holding the upper triangles of the matrices back to back."""
    out: List[np.ndarray] = []
    for X in mats:
        X = np.asarray(X, dtype=np.float32)
        n = X.shape[0]
        assert X.shape == (n, n)
        for r in range(n):
            out.append(X[r, r:])
    return np.concatenate(out) if out else np.zeros(0, dtype=np.float32)


def unpack_upper(buf: np.ndarray, dims: Sequence[int]) -> List[np.ndarray]:
    buf = np.asarray(buf, dtype=np.float32)
    res = []
    k = 0
    for n in dims:
        X = np.zeros((n, n), dtype=np.float32)
        for r in range(n):
            seg = buf[k:k + n - r]
            X[r, r:] = seg
            X[r:, r] = seg
            k += n - r
        res.append(X)
    assert k == buf.size
    return res


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even; NaN -> a quiet NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lower = u & 0xFFFF                   # the 16 bits that are dropped
    upper = u >> 16
    round_up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    r = upper + round_up.astype(np.uint64)
    nan = np.isnan(x)
    r = np.where(nan, (upper | 0x40), r)   # keep the sign and exponent, set the quiet bit
    return (r & 0xFFFF).astype(np.uint16).reshape(x.shape)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).reshape(np.shape(b))
