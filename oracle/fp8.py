"""OCP e4m3fn decode written from the format definition (oracle side, test infrastructure).

e4m3fn byte = s eeee mmm : value = (-1)^s * 2^(e-7) * (1 + m/8) for e in 1..15,
(-1)^s * 2^-6 * (m/8) for e = 0, except e = 15, m = 7 which is NaN (there are no
infinities; the largest finite magnitude is 448).
"""
import numpy as np


def decode_code(code: int) -> float:
    s = (code >> 7) & 1
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 15 and m == 7:
        return float("nan")
    mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return -mag if s else mag


TABLE = np.array([decode_code(c) for c in range(256)], dtype=np.float64)


def decode(codes: np.ndarray) -> np.ndarray:
    """uint8 codes -> float64 values (exact)."""
    return TABLE[np.asarray(codes, dtype=np.uint8)]


# The 127 non-negative finite values in code order (codes 0x00..0x7E are increasing in value) and the
# 126 midpoints between neighbours, both exact in float64.
_POS = TABLE[:127]
_MID = (_POS[:-1] + _POS[1:]) / 2.0


def encode(y: np.ndarray) -> np.ndarray:
    """float32 values -> e4m3fn codes: the nearest finite value, ties to the even code, magnitudes beyond
    the largest finite value (448) saturate to it; the sign bit is copied (so -0.0 and negative values that
    round to zero give 0x80).  NaN input is not defined here.

    Written as a nearest-neighbour search over the decode table, not as bit manipulation: for |y| the
    number of midpoints strictly below it is the index of the nearest value, and a value exactly on a
    midpoint between codes i and i+1 goes to whichever of the two is even.
    """
    y = np.asarray(y, dtype=np.float32)
    mag = np.abs(y).astype(np.float64)
    idx = np.searchsorted(_MID, mag, side="left")            # midpoints strictly below |y|
    idx = np.minimum(idx, 126)
    on_mid = (idx < 126) & (mag == _MID[np.minimum(idx, 125)])
    idx = np.where(on_mid & (idx % 2 == 1), idx + 1, idx)    # tie between idx and idx+1: take the even one
    sign = np.signbit(y).astype(np.uint8) << np.uint8(7)
    return (idx.astype(np.uint8) | sign).astype(np.uint8)
