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


# ------------------------------------------------------------------ general bias, truncation, per-table bias

@pytest.mark.parametrize("mant_bits,default_bias", [(3, 15), (4, 7)])
def test_fp8_bias_shift_is_a_power_of_two_scale(mant_bits, default_bias):
    # moving the bias by s multiplies every representable value by 2^-s: encode(x, B) = encode(x * 2^(B-B0), B0)
    rng = np.random.default_rng(7)
    x = np.exp(rng.uniform(np.log(1e-3), np.log(1e3), size=50_000)).astype(np.float32)
    b = np.arange(256, dtype=np.uint8)
    for bias in (default_bias - 9, default_bias - 1, default_bias + 4, default_bias + 20):
        s = bias - default_bias
        scaled = (x.astype(np.float64) * 2.0 ** s).astype(np.float32)
        assert np.all(scaled.astype(np.float64) == x.astype(np.float64) * 2.0 ** s)       # exact in fp32
        for trunc in (False, True):
            np.testing.assert_array_equal(oracle.fp8_encode(x, mant_bits, bias, trunc),
                                          oracle.fp8_encode(scaled, mant_bits, default_bias, trunc))
        np.testing.assert_array_equal(oracle.fp8_decode(b, mant_bits, bias).astype(np.float64) * 2.0 ** s,
                                      oracle.fp8_decode(b, mant_bits, default_bias).astype(np.float64))


@pytest.mark.parametrize("trunc", [False, True])
def test_e5m3_general_bias_bit_formula(trunc):
    x = _random_floats(300_000, 8)
    for bias in (-96, 0, 15, 31, 110):
        lo = (127 - bias) << 23
        i = np.clip(x.view(np.int32).astype(np.int64), lo, lo + (255 << 20))
        want = ((i - (lo if trunc else lo - (1 << 19))) >> 20).astype(np.uint8)
        np.testing.assert_array_equal(oracle.fp8_encode(x, 3, bias, trunc), want)
        dec = ((np.arange(256, dtype=np.int64) << 20) + lo).astype(np.uint32).view(np.float32)
        np.testing.assert_array_equal(oracle.fp8_decode(np.arange(256, dtype=np.uint8), 3, bias), dec)
        assert np.all(np.isfinite(dec)) and np.all(dec >= np.float32(2.0 ** -126))          # finite, normal


def test_table_bias_hand_values():
    tb = lambda vals, dt: oracle.fp8_table_bias(np.array(vals, dtype=np.float32), dt)
    E5, E4 = oracle.LUT_E5M3, oracle.LUT_E4M4
    assert tb([0.25, 1.0, 0.5], E5) == 31 and tb([0.25, 1.0, 0.5], E4) == 15      # [1, 2) is the top binade
    assert tb([1.9999], E5) == 31 and tb([2.0], E5) == 30 and tb([2.0], E4) == 14
    assert tb([0.75, 0.1], E5) == 32 and tb([0.75], E4) == 16
    assert tb([100.0, 3.0], E5) == 25 and tb([100.0], E4) == 9                    # 2^6 <= 100 < 2^7
    assert tb([65536.0], E5) == 15                                                # the fixed format's own top binade
    assert tb([0.0, 0.0], E5) == 110 and tb([1e-45], E4) == 110                   # nothing above 2^-126: clamped
    assert tb([np.inf], E5) == -96 and tb([np.inf], E4) == -100
    assert tb([3e38], E5) == 31 - 127 and tb([3e38], E4) == -100


@pytest.mark.parametrize("dt,mant_bits,top_low", [(oracle.LUT_E5M3, 3, 0xF8), (oracle.LUT_E4M4, 4, 0xF0)])
def test_table_bias_brute_force_and_scale_invariance(dt, mant_bits, top_low):
    rng = np.random.default_rng(9)
    lo_b, hi_b = oracle.FP8_BIAS_RANGE[dt]
    for trial in range(40):
        scale = 2.0 ** rng.integers(-60, 60)
        F = (np.exp(rng.uniform(np.log(1e-4), np.log(1.0), size=(8, 256))) * scale).astype(np.float32)
        B = oracle.fp8_table_bias(F, dt)
        # the smallest bias (largest values) whose top binade still starts at or below the largest entry
        ok = [b for b in range(lo_b, hi_b + 1) if oracle.lib().orc_fp8_value(top_low, mant_bits, b) <= float(F.max())]
        assert B == min(ok)
        for trunc in (False, True):
            st, dec, used = oracle.lut_store(F, dt, truncate=trunc, per_table=True, return_bias=True)
            assert used == B
            st_fixed, dec_fixed = oracle.lut_store(F, dt, truncate=trunc, bias=B)
            np.testing.assert_array_equal(st, st_fixed)
            np.testing.assert_array_equal(dec, dec_fixed)
            assert st.max() >= top_low                                              # the largest entry sits in the top binade
            # scaling the table by a power of two changes the bias, not the stored bytes
            st2, dec2, used2 = oracle.lut_store((F.astype(np.float64) * 2.0 ** -7).astype(np.float32), dt,
                                                truncate=trunc, per_table=True, return_bias=True)
            assert used2 == B + 7
            np.testing.assert_array_equal(st2, st)
            np.testing.assert_array_equal(dec2.astype(np.float64) * 2.0 ** 7, dec.astype(np.float64))
        st, dec = oracle.lut_store(F, dt, per_table=True)
        rel = np.abs(dec.astype(np.float64) - F) / F
        in_range = F >= dec.min()
        assert rel[in_range].max() <= 1.0 / (2 ** (mant_bits + 1)) + 1e-12          # half a step; the clamp at the top included
