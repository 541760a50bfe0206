"""Pins for the oracle's number formats (FP8 E4M3 / E5M2 encode + decode, BF16 rounding, scale).

Nothing here compares the oracle with itself: the expected values come from the constants the
paper prints (tests/golden/paper_constants.txt), from an exact-rational nearest-value search
(tests/refmodel.py), from PyTorch's CPU float8 casts (a library routine) and from hand-worked
cases."""
import os

import numpy as np
import pytest
import torch

import refmodel as R

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    d = {}
    with open(os.path.join(HERE, "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                d[line[0]] = float(line[1])
    return d


def all_bf16_as_f32():
    return (np.arange(65536, dtype=np.uint32) << np.uint32(16)).view(np.float32)


def test_paper_format_ranges(oracle):
    g = golden()
    e4 = [oracle.e4m3_decode(c) for c in range(256)]
    e5 = [oracle.e5m2_decode(c) for c in range(256)]
    pos4 = [v for v in e4 if np.isfinite(v) and v > 0]
    pos5 = [v for v in e5 if np.isfinite(v) and v > 0]
    assert min(pos4) == g["e4m3_min_positive"] and max(pos4) == g["e4m3_max"]
    assert min(pos5) == g["e5m2_min_positive"] and max(pos5) == g["e5m2_max"]
    # smallest E5M2 normal (Section 3.2): first code with a non-zero exponent field
    assert oracle.e5m2_decode(0b0_00001_00) == g["e5m2_min_normal"]
    # field widths: 2^mbits codes per binade
    assert oracle.e4m3_decode(0b0_0111_000) == 1.0 and oracle.e4m3_decode(0b0_0111_001) == 1.0 + 2.0 ** -g["e4m3_mantissa_bits"]
    assert oracle.e5m2_decode(0b0_01111_00) == 1.0 and oracle.e5m2_decode(0b0_01111_01) == 1.0 + 2.0 ** -g["e5m2_mantissa_bits"]
    # E4M3 has NaN only at S.1111.111 and no infinity; E5M2 has both
    assert sum(np.isnan(e4)) == 2 and sum(np.isinf(e4)) == 0
    assert sum(np.isnan(e5)) == 6 and sum(np.isinf(e5)) == 2
    assert sum(np.isfinite(e4)) == 254 and sum(np.isfinite(e5)) == 248


def test_decode_matches_exact_rational_definition(oracle):
    for ebits, mbits, dec in ((4, 3, oracle.e4m3_decode), (5, 2, oracle.e5m2_decode)):
        vals = R.fp8_values(ebits, mbits)
        for code, v in vals.items():
            assert dec(code) == float(v)
            assert dec(code | 0x80) == -float(v)
        # strictly increasing with the code
        ordered = [float(vals[c]) for c in sorted(vals)]
        assert all(a < b for a, b in zip(ordered, ordered[1:]))


def test_decode_matches_torch_cast(oracle):
    codes = torch.arange(256, dtype=torch.uint8)
    for dt, dec in ((torch.float8_e4m3fn, oracle.e4m3_decode), (torch.float8_e5m2, oracle.e5m2_decode)):
        ref = codes.view(dt).to(torch.float32).numpy()
        got = np.array([dec(int(c)) for c in range(256)], dtype=np.float64)
        assert np.array_equal(np.isnan(ref), np.isnan(got))
        ok = ~np.isnan(ref)
        assert np.array_equal(ref[ok].astype(np.float64), got[ok])
        assert np.array_equal(np.signbit(ref[ok]), np.signbit(got[ok]))


SCALES = [1.0, 2.0 ** -7, 2.0 ** 9, 448.0 / 3.0, 448.0 / 0.0123, 1.7777778, 57344.0 / 5.5, 180.32704]


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_encoder_bruteforce_all_bf16_patterns(oracle, fmt):
    """Every BF16 bit pattern times a set of scales, against the exact-rational nearest-value
    search with even-code tie-break (covers saturation, ties, subnormals, -0, NaN, Inf)."""
    ebits, mbits = (4, 3) if fmt == "e4m3" else (5, 2)
    enc = oracle.e4m3_encode_array if fmt == "e4m3" else oracle.e5m2_encode_array
    x = all_bf16_as_f32()
    n_checked = 0
    for s in SCALES:
        with np.errstate(over="ignore", invalid="ignore", under="ignore"):
            y = (x * np.float32(s)).astype(np.float32)
        got = enc(y)
        # exact-rational search is slow: check each distinct y once
        uniq, idx = np.unique(y.view(np.uint32), return_index=True)
        step = 1 if s == 1.0 else 3
        for i in idx[::step]:
            want = R.fp8_encode(y[i], ebits, mbits)
            assert got[i] == want, (fmt, s, float(y[i]), int(got[i]), want)
            n_checked += 1
    assert n_checked > 65000


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_encoder_matches_torch_cast_in_range(oracle, fmt):
    """Library third opinion on all in-range values: PyTorch's CPU float8 cast rounds to nearest
    even; it differs from the method only beyond the largest finite value (it does not clip)."""
    dt, top, enc = ((torch.float8_e4m3fn, 448.0, oracle.e4m3_encode_array) if fmt == "e4m3"
                    else (torch.float8_e5m2, 57344.0, oracle.e5m2_encode_array))
    x = all_bf16_as_f32()
    for s in SCALES:
        with np.errstate(over="ignore", invalid="ignore", under="ignore"):
            y = (x * np.float32(s)).astype(np.float32)
        sel = np.isfinite(y) & (np.abs(y) <= top)
        ref = torch.from_numpy(y[sel]).to(dt).view(torch.uint8).numpy()
        assert np.array_equal(enc(y[sel]), ref)


def test_encoder_handworked_cases(oracle):
    e = oracle.e4m3_encode
    assert e(448.0) == 0x7E and e(-448.0) == 0xFE
    assert e(463.99) == 0x7E and e(464.0) == 0x7E and e(465.0) == 0x7E    # clip to 448
    assert e(1e30) == 0x7E and e(float("inf")) == 0x7E and e(float("-inf")) == 0xFE
    assert e(0.0) == 0x00 and e(-0.0) == 0x80
    assert e(2.0 ** -10) == 0x00            # tie between 0 and 2^-9 -> even code 0
    assert e(-(2.0 ** -10)) == 0x80
    assert e(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 0x01
    assert e(3 * 2.0 ** -10) == 0x02        # tie between 2^-9 (code 1) and 2^-8 (code 2) -> even
    assert e(5 * 2.0 ** -10) == 0x02        # tie between code 2 and code 3 -> even code 2
    assert e(1.0625) == 0x38                # tie 1.0 / 1.125 -> even mantissa 000
    assert e(1.1875) == 0x3A                # tie 1.125 / 1.25 -> even mantissa 010
    assert e(float("nan")) == 0x7F
    assert e(2.0 ** -6) == 0x08             # smallest normal
    assert e(1e-45) == 0x00                 # FP32 subnormal flushes
    e5 = oracle.e5m2_encode
    assert e5(57344.0) == 0x7B and e5(1e9) == 0x7B and e5(float("inf")) == 0x7B
    assert e5(2.0 ** -17) == 0x00 and e5(2.0 ** -16) == 0x01 and e5(2.0 ** -14) == 0x04
    assert e5(float("nan")) == 0x7F and e5(-0.0) == 0x80


def test_roundtrip_every_code_is_a_fixed_point(oracle):
    for c in range(256):
        v = oracle.e4m3_decode(c)
        if not np.isnan(v):
            assert oracle.e4m3_encode(v) == c
        v = oracle.e5m2_decode(c)
        if np.isfinite(v):
            assert oracle.e5m2_encode(v) == c


def test_bf16_rounding_matches_torch(oracle):
    rng = np.random.default_rng(7)
    u = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    # add exact ties and near-overflow cases
    u = np.concatenate([u, np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F7FFFFF,
                                     0x7F800000, 0xFF800000, 0x00000001, 0x80000000, 0x00008000],
                                    dtype=np.uint32)])
    f = u.view(np.float32)
    fin = ~np.isnan(f)
    ref = torch.from_numpy(f[fin].copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(v) for v in f[fin]], dtype=np.uint16)
    assert np.array_equal(ref, got)
    assert oracle.f32_to_bf16(float("nan")) & 0x7FFF == 0x7FC0


def test_scale_rule(oracle):
    # amax maps onto the largest E4M3 value (Algorithm 1: s = q_amax / amax)
    for amax in (1.0, 3.0, 0.0123, 252.0, 1e-20, 3e38):
        a = np.float32(amax)
        s = oracle.scale(a)
        assert s == float(np.float32(448.0) / a)
        assert oracle.e4m3_encode(np.float32(a * np.float32(s))) == 0x7E
    assert oracle.scale(1.75 * 2.0 ** -3) == 2.0 ** 11          # power-of-two closed form
    assert oracle.scale(0.0) == 1.0
    assert oracle.scale(1e-40) == float(np.finfo(np.float32).max)   # quotient overflows -> FLT_MAX
    assert oracle.scale(float("inf")) == 1.0 and oracle.scale(float("nan")) == 1.0
    assert oracle.scale(57344.0, 57344.0) == 1.0
