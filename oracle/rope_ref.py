"""Rotary position embedding of a matvec result, plain fp64 (test infrastructure, not product code).

Section 3 of the paper runs R = rope(O, T) after O = M @ N as its example of fusing two operators; it
does not print the formula or the layout of T.  The reading taken by this build: the rows of O are
taken in adjacent pairs (2i, 2i + 1), T has the shape of O and holds for pair i of vector b the cosine
at T[b][2i] and the sine at T[b][2i + 1] of that pair's angle (so no trigonometry runs on the device), and

    R[b][2i]     = O[b][2i] * cos - O[b][2i + 1] * sin
    R[b][2i + 1] = O[b][2i] * sin + O[b][2i + 1] * cos

i.e. every pair is turned by its angle.  Written out with Python loops over numpy scalars in fp64.
"""
import numpy as np


def rope(O, T):
    """O, T: [B][rows] (rows even).  Returns (R, Rabs): the rotated values in fp64 and the sums of the
    magnitudes of the two products that form each value (the scale of its rounding error)."""
    O = np.asarray(O, dtype=np.float64)
    T = np.asarray(T, dtype=np.float64)
    B, rows = O.shape
    assert T.shape == O.shape and rows % 2 == 0
    R = np.zeros_like(O)
    Rabs = np.zeros_like(O)
    for b in range(B):
        for i in range(rows // 2):
            x, y = O[b, 2 * i], O[b, 2 * i + 1]
            c, s = T[b, 2 * i], T[b, 2 * i + 1]
            R[b, 2 * i] = x * c - y * s
            R[b, 2 * i + 1] = x * s + y * c
            Rabs[b, 2 * i] = abs(x * c) + abs(y * s)
            Rabs[b, 2 * i + 1] = abs(x * s) + abs(y * c)
    return R, Rabs


def table(angles):
    """T for angles[b][i] (radians), cos and sin interleaved, float32."""
    a = np.asarray(angles, dtype=np.float64)
    T = np.empty((a.shape[0], a.shape[1] * 2), dtype=np.float32)
    T[:, 0::2] = np.cos(a)
    T[:, 1::2] = np.sin(a)
    return T
