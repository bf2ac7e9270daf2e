"""Pins of oracle/lowbit.py (the oracle's decoding of 8- and 4-bit weights, Sec. 4.3's bit-width sweep): the
values the format documents print, torch's own FP8 widening for all 256 bytes, and a hand computation of the
packed layouts on a few entries."""
import math
import os

import numpy as np
import torch

from oracle import lowbit

GOLD = os.path.join(os.path.dirname(__file__), "golden", "ocp_lowbit_formats.txt")


def _rows():
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            kind, bits, val = line.split()
            yield kind, int(bits.replace(".", ""), 2), float(val)


def test_printed_values_of_the_formats():
    n = 0
    for kind, code, want in _rows():
        dec = {"fp8_e4m3": lowbit.decode_fp8_e4m3, "fp4_e2m1": lowbit.decode_fp4_e2m1, "e8m0": lowbit.decode_e8m0}[kind]
        got = float(dec(np.array([code]))[0])
        if math.isnan(want):
            assert math.isnan(got), (kind, code)
        else:
            assert got == want and math.copysign(1.0, got) == math.copysign(1.0, want), (kind, code, got, want)
        n += 1
    assert n >= 30


def test_fp8_all_bytes_equal_the_library_widening():
    b = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(b).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = lowbit.decode_fp8_e4m3(b)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_fp4_codes_are_monotone_and_symmetric():
    v = lowbit.decode_fp4_e2m1(np.arange(16))
    assert np.all(np.diff(v[:8]) > 0) and np.array_equal(v[8:], -v[:8])


def test_mxfp4_packing_and_block_scales():
    """Low nibble = even input index; one scale per 32 inputs; checked entry by entry with scalar arithmetic."""
    rng = np.random.default_rng(0)
    n, K = 5, 96
    packed = rng.integers(0, 256, size=(n, K // 2), dtype=np.uint8)
    sc = rng.integers(100, 140, size=(n, K // 32), dtype=np.uint8)
    W = lowbit.dequant_mxfp4(packed, sc)
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for r in range(n):
        for k in range(K):
            code = (int(packed[r, k // 2]) >> (4 * (k & 1))) & 15
            want = (-1.0 if code & 8 else 1.0) * mags[code & 7] * 2.0 ** (int(sc[r, k // 32]) - 127)
            assert W[r, k] == want


def test_fp8_row_scales():
    rng = np.random.default_rng(1)
    q = rng.integers(0, 0x7F, size=(4, 16), dtype=np.uint8)   # no NaN pattern
    s = rng.uniform(1e-3, 2e-3, size=4)
    W = lowbit.dequant_fp8_rows(q, s)
    ref = torch.from_numpy(q).view(torch.float8_e4m3fn).to(torch.float64).numpy() * s[:, None]
    assert np.array_equal(W, ref)
