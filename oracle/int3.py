"""Dense 3-bit storage of INT3 codes -- CPU oracle (test infrastructure only; see formats.py).

Eq. 1-2 with b = 3 give integer codes z in {-3, ..., 3}.  The paper prints no storage layout for
them (its kernel appendix covers NVFP4 only), so the layout is a reading, and parity with the
authors' files is unpinned; what the tests pin is the layout stated here:

  * a row of K codes is a stream of 3 K bits, K a multiple of 8, so a row takes 3 K / 8 bytes
    and rows follow each other without padding;
  * code k occupies bits 3 k, 3 k + 1, 3 k + 2 of that stream, least significant bit first, as the
    3-bit two's complement of z (z mod 8; -4 is representable and never produced);
  * bit b of the stream is bit b mod 8 of byte b div 8 (little-endian bit order).

Eight codes therefore fill exactly three bytes.
"""
from __future__ import annotations

import numpy as np


def pack_dense(z) -> np.ndarray:
    """[rows, K] integer codes in -4..3 -> [rows, 3 K / 8] bytes."""
    z = np.asarray(z, dtype=np.int64)
    if z.ndim != 2 or z.shape[1] % 8:
        raise ValueError("codes must be [rows, K] with K a multiple of 8")
    if z.size and (z.min() < -4 or z.max() > 3):
        raise ValueError("a code does not fit three bits")
    rows, K = z.shape
    field = z % 8
    stream = np.zeros((rows, 3 * K), dtype=np.uint8)
    for i in range(3):
        stream[:, i::3] = (field >> i) & 1
    return np.packbits(stream, axis=1, bitorder="little")


def unpack_dense(packed, K: int) -> np.ndarray:
    """[rows, 3 K / 8] bytes -> [rows, K] integer codes in -4..3."""
    p = np.asarray(packed, dtype=np.uint8)
    if K % 8 or p.ndim != 2 or p.shape[1] != 3 * K // 8:
        raise ValueError("packed must be [rows, 3 K / 8] with K a multiple of 8")
    stream = np.unpackbits(p, axis=1, bitorder="little").astype(np.int64)
    field = stream[:, 0::3] + 2 * stream[:, 1::3] + 4 * stream[:, 2::3]
    return np.where(field >= 4, field - 8, field)
