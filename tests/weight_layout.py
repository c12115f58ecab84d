"""Checker for the library's streaming ("tiled") order of a quantized weight matrix.

The tile order is the HIP kernels' own design (the order in which a wavefront consumes the codes as an
MFMA operand), not something Section 5 of the paper defines, so it is not part of the oracle: this
module is test infrastructure that restates the documented permutation of include/fg.h in numpy, is
itself checked element by element in plain Python (tests/test_oracle_quant.py), and is what
fg_pack_weights is compared against.  It holds no arithmetic: bytes in, the same bytes out."""
import numpy as np

GROUP = 64


def tile_weights(codes: np.ndarray, meta: np.ndarray):
    """Canonical [n, k/2] codes and [n, k/64, 2] pairs -> the same bytes in tile order: tiles of 32
    rows x 64 columns, row blocks outermost, then the tiles of a row block along the columns; inside a
    tile the 16-byte piece of (row r, half h of the 64-column group) sits at byte 16*(32*h + r); the
    pairs: 32 per tile, in the same tile order."""
    n, kh = codes.shape
    k = kh * 2
    assert n % 32 == 0 and k % GROUP == 0
    ks = k // GROUP
    c = codes.reshape(n // 32, 32, ks, 2, 16)          # [row block, r, k tile, h, 16 bytes]
    c = c.transpose(0, 2, 3, 1, 4)                     # [row block, k tile, h, r, 16]
    m = meta.reshape(n // 32, 32, ks, 2).transpose(0, 2, 1, 3)   # [row block, k tile, r, {min,scale}]
    return np.ascontiguousarray(c).reshape(n, kh), np.ascontiguousarray(m).reshape(n, ks, 2)
