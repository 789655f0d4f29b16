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
