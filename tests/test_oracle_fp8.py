"""Pins for the oracle's e4m3fn decode: format definition, a library decoder, and the encoder round trip."""
import numpy as np
import torch

import workloads as wl
from oracle import fp8


def test_known_values_from_the_format_definition():
    # s eeee mmm, bias 7, subnormals in units of 2^-9, max finite 448, 0x7F / 0xFF NaN
    known = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125,
             0x40: 2.0, 0x7E: 448.0, 0x77: 240.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9)}
    for code, val in known.items():
        assert fp8.TABLE[code] == val, hex(code)
    assert np.isnan(fp8.TABLE[0x7F]) and np.isnan(fp8.TABLE[0xFF])
    assert np.isfinite(fp8.TABLE).sum() == 254


def test_all_codes_match_library_decoder():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.nan_to_num(fp8.TABLE, nan=12345.0), np.nan_to_num(ref, nan=12345.0))


def test_table_is_monotone_per_sign():
    pos = fp8.TABLE[:0x7F]
    assert np.all(np.diff(pos) > 0)
    assert np.array_equal(fp8.TABLE[0x80:0xFF], -pos)


def test_encode_decode_round_trip_and_ties():
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    vals = fp8.decode(finite).astype(np.float32)
    back = wl.e4m3_encode(vals)
    # -0.0 and +0.0 keep their sign bit
    assert np.array_equal(back, finite)
    # midpoints between neighbours go to the even code
    pos = fp8.TABLE[:0x7F]
    mid = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)
    enc = wl.e4m3_encode(mid)
    expect = np.array([c if c % 2 == 0 else c + 1 for c in range(0x7E)], dtype=np.uint8)
    assert np.array_equal(enc, expect)
