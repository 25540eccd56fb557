"""Pins for the oracle's number formats (Sec. II): the 8-bit sign-less floats and
the IEEE half path.  None of these tests call the HIP library.

What pins what:
  * worked values written out by hand in tests/golden/e5m3_pins.txt;
  * numpy's own binary16: for exponent fields 1..30 an e5m3 code b is the half
    with bit pattern b << 7 (same bias, 3 of the 10 mantissa bits), so numpy
    decodes 240 of the 256 codes independently of the oracle;
  * the paper's "two instructions" description: shift the bit string, adjust
    the exponent bias -- written here with integer numpy ops on the FP32 bit
    pattern and compared with the oracle's definition-based (float64, table
    search) implementation on all codes / a million floats;
  * format invariants: round trip, monotonicity, nearest-ness by brute force
    over all 256 values, the 1/17 relative error bound, clamp behaviour;
  * IEEE half: numpy.float16 conversion on 10^6 floats incl. subnormals.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e5m3_pins.txt")


def _golden_rows():
    rows = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            x, code, val = line.split()
            rows.append((np.float32(float(x)), int(code, 16), float(val)))
    return rows


def test_e5m3_golden_values():
    rows = _golden_rows()
    assert len(rows) >= 15
    for x, code, val in rows:
        got = int(oracle.e5m3_encode(x)[0])
        assert got == code, f"enc({x}) = {got:#x}, expected {code:#x}"
        assert float(oracle.e5m3_decode(np.uint8(code))[0]) == val


def test_e5m3_decode_matches_numpy_half_for_normal_exponents():
    b = np.arange(256, dtype=np.uint16)
    as_half = (b << 7).astype(np.uint16).view(np.float16).astype(np.float32)
    dec = oracle.e5m3_decode(b.astype(np.uint8))
    e = b >> 3
    mid = (e >= 1) & (e <= 30)
    assert mid.sum() == 240
    np.testing.assert_array_equal(dec[mid], as_half[mid])
    # the two ends are where the format departs from binary16: no subnormals, no Inf/NaN
    assert np.all(np.isfinite(dec)) and np.all(dec > 0)
    np.testing.assert_array_equal(dec[:8], (1 + np.arange(8) / 8.0) * 2.0 ** -15)
    np.testing.assert_array_equal(dec[248:], (1 + np.arange(8) / 8.0) * 2.0 ** 16)


def test_e5m3_covers_fp16_normal_range():
    dec = oracle.e5m3_decode(np.arange(256, dtype=np.uint8))
    assert dec.min() <= np.float32(2.0 ** -14)       # smallest normal half
    assert dec.max() >= np.float32(65504.0)          # largest finite half


def test_e5m3_decode_is_shift_plus_bias():
    b = np.arange(256, dtype=np.uint32)
    bits = (b << 20) + np.uint32(0x38000000)
    np.testing.assert_array_equal(bits.view(np.float32), oracle.e5m3_decode(b.astype(np.uint8)))


def _encode_bits(x: np.ndarray, truncate: bool) -> np.ndarray:
    """FP32 -> e5m3 as integer ops on the bit pattern: signed clamp, bias subtract, shift."""
    i = x.astype(np.float32).view(np.int32).astype(np.int64)
    i = np.clip(i, 0x38000000, 0x47F00000)
    sub = 0x38000000 if truncate else 0x37F80000      # nearest: half an 8-bit ulp folded into the bias
    return ((i - sub) >> 20).astype(np.uint8)


def _random_floats(n, seed):
    rng = np.random.default_rng(seed)
    a = np.exp(rng.uniform(np.log(1e-7), np.log(1e6), size=n)).astype(np.float32)
    b = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32).view(np.float32)  # any bit pattern
    edge = np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, np.nan, 2.0 ** -15, 122880.0, 122880.5,
                     np.nextafter(np.float32(2.0 ** -15), np.float32(0)), 65504.0, 1e-45], dtype=np.float32)
    neg_nan = np.array([0xFFC00000], dtype=np.uint32).view(np.float32)
    return np.concatenate([a, b, edge, neg_nan])


@pytest.mark.parametrize("truncate", [False, True])
def test_e5m3_encode_is_clamp_subtract_shift(truncate):
    x = _random_floats(500_000, 1)
    np.testing.assert_array_equal(oracle.e5m3_encode(x, truncate), _encode_bits(x, truncate))


def test_e5m3_round_trip_and_monotone():
    b = np.arange(256, dtype=np.uint8)
    dec = oracle.e5m3_decode(b)
    np.testing.assert_array_equal(oracle.e5m3_encode(dec), b)
    np.testing.assert_array_equal(oracle.e5m3_encode(dec, truncate=True), b)
    assert np.all(np.diff(dec.astype(np.float64)) > 0)
    x = np.sort(np.abs(_random_floats(200_000, 2)[:400_000]))
    x = x[np.isfinite(x)]
    enc = oracle.e5m3_encode(x).astype(np.int32)
    assert np.all(np.diff(enc) >= 0)


def test_e5m3_encode_is_nearest_with_ties_up():
    rng = np.random.default_rng(3)
    x = np.exp(rng.uniform(np.log(2.0 ** -15), np.log(122880.0), size=100_000)).astype(np.float32)
    table = oracle.e5m3_decode(np.arange(256, dtype=np.uint8)).astype(np.float64)
    # exact midpoints between neighbours are representable in fp32: include them all
    mids = ((table[:-1] + table[1:]) / 2).astype(np.float32)
    assert np.all(mids.astype(np.float64) == (table[:-1] + table[1:]) / 2)
    x = np.concatenate([x, mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(np.inf))])
    enc = oracle.e5m3_encode(x)
    err = np.abs(table[None, :] - x.astype(np.float64)[:, None])           # brute force over all 256 values
    best = err.min(axis=1)
    got = np.abs(table[enc] - x.astype(np.float64))
    np.testing.assert_array_equal(got, best)
    tie = (err == best[:, None]).sum(axis=1) == 2
    assert tie.sum() >= 255
    larger = np.array([np.flatnonzero(e == b).max() for e, b in zip(err[tie], best[tie])])
    np.testing.assert_array_equal(enc[tie], larger)
    rel = got / x.astype(np.float64)
    assert rel.max() <= 1.0 / 17.0 + 1e-12
    # truncation never rounds up and stays within one step
    enc_t = oracle.e5m3_encode(x, truncate=True)
    assert np.all(table[enc_t] <= x.astype(np.float64))
    assert np.all(table[np.minimum(enc_t.astype(int) + 1, 255)] > x.astype(np.float64) - 1e-30)


def test_e4m4_general_format_round_trip():
    # the 4+4 split of Sec. II; its bias is not recoverable from the text, any bias must round-trip
    for bias in (7, 8, 11):
        b = np.arange(256, dtype=np.uint8)
        dec = oracle.fp8_decode(b, 4, bias)
        assert np.all(np.diff(dec.astype(np.float64)) > 0)
        np.testing.assert_array_equal(oracle.fp8_encode(dec, 4, bias), b)
        bits = (b.astype(np.uint32) << 19) + np.uint32((127 - bias) << 23)
        np.testing.assert_array_equal(bits.view(np.float32), dec)


def test_e4m4_hand_values_and_bit_formula():
    # bias 7: 1.0 = 2^0 has exponent field 7; one mantissa step is 1/16
    enc = lambda x, bias=7: int(oracle.fp8_encode(np.float32(x), 4, bias)[0])
    dec = lambda b, bias=7: float(oracle.fp8_decode(np.uint8(b), 4, bias)[0])
    assert enc(1.0) == 0x70 and dec(0x70) == 1.0
    assert enc(1.0625) == 0x71 and enc(1.03125) == 0x71 and enc(1.03124) == 0x70      # tie goes up
    assert dec(0x00) == 2.0 ** -7 and enc(0.0) == 0x00 and enc(1e-9) == 0x00
    assert dec(0xFF) == 1.9375 * 2.0 ** 8 and enc(1000.0) == 0xFF and enc(np.inf) == 0xFF
    assert enc(3.0) == 0x88 and dec(0x88) == 3.0                                        # 1.5 * 2^1
    assert enc(100.0, bias=1) == enc(100.0 / 64.0, bias=7)                              # a bias shift is a power-of-two scale
    x = _random_floats(300_000, 6)
    for bias in (-3, 1, 7, 12):
        lo = (127 - bias) << 23
        i = np.clip(x.view(np.int32).astype(np.int64), lo, lo + (255 << 19))
        want = ((i - (lo - (1 << 18))) >> 19).astype(np.uint8)
        np.testing.assert_array_equal(oracle.fp8_encode(x, 4, bias), want)
        F = np.abs(x[:4096]).reshape(16, 256)
        st, back = oracle.lut_store(F, oracle.LUT_E4M4, e4m4_bias=bias)
        np.testing.assert_array_equal(st, oracle.fp8_encode(F.ravel(), 4, bias))
        np.testing.assert_array_equal(back.ravel(), oracle.fp8_decode(st, 4, bias))


def test_fp16_encode_matches_numpy():
    rng = np.random.default_rng(4)
    x = np.concatenate([
        np.exp(rng.uniform(np.log(1e-9), np.log(65504.0), size=1_000_000)),
        rng.uniform(0, 2.0 ** -14, size=50_000),                 # subnormal halves
        [0.0, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -14, 65504.0, 65519.9, 1.0, 1.0 + 2.0 ** -11,
         1.0 + 3 * 2.0 ** -11, 2047.5 * 2.0 ** -10],
    ]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = oracle.fp16_encode(x)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(oracle.fp16_decode(got), want.view(np.float16).astype(np.float32))


def test_fp16_saturates_instead_of_inf():
    x = np.array([65520.0, 70000.0, 1e9, np.inf], dtype=np.float32)
    np.testing.assert_array_equal(oracle.fp16_encode(x), np.full(4, 0x7BFF, dtype=np.uint16))
    np.testing.assert_array_equal(oracle.fp16_decode(np.array([0x7BFF], dtype=np.uint16)), [65504.0])


def test_fp16_decode_all_finite_patterns():
    h = np.arange(0x7C00, dtype=np.uint16)
    np.testing.assert_array_equal(oracle.fp16_decode(h), h.view(np.float16).astype(np.float32))


def test_lut_store_decoded_matches_formats():
    rng = np.random.default_rng(5)
    F = np.exp(rng.uniform(np.log(1e-6), np.log(2e5), size=(8, 256))).astype(np.float32)
    st, dec = oracle.lut_store(F, oracle.LUT_FP32)
    np.testing.assert_array_equal(st.view(np.float32).reshape(F.shape), F)
    np.testing.assert_array_equal(dec, F)
    st, dec = oracle.lut_store(F, oracle.LUT_FP16)
    with np.errstate(over="ignore"):
        want = np.minimum(F, np.float32(65504.0)).astype(np.float16)
    np.testing.assert_array_equal(st.view(np.uint16), want.view(np.uint16).ravel())
    np.testing.assert_array_equal(dec, want.astype(np.float32))
    st, dec = oracle.lut_store(F, oracle.LUT_E5M3)
    np.testing.assert_array_equal(st, _encode_bits(F.ravel(), False))
    np.testing.assert_array_equal(dec.ravel(), oracle.e5m3_decode(st))
