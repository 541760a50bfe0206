"""Pins for the parts of the oracle that used to be checked only against itself: the de-scale arithmetic of the
fake-quantization workflow (Section 4, Figure 4), the tensor-wide decision when the criterion is Eq. (3)
(Section 3.1 applied to the two totals of Eq. (3)), and the closed edge of the near-threshold band of the statistics.
CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import refmodel as R
from paper_2512_22804_amd import workloads as W

TH = 0.045


def bf16(v):
    b = W.f32_to_bf16_bits(np.asarray(v, dtype=np.float32))
    assert np.array_equal(W.bf16_bits_to_f32(b), np.asarray(v, dtype=np.float32)), "value is not a BF16 number"
    return b


def one_block(values, fill=0.0):
    v = np.full(128, fill, dtype=np.float32)
    v[:len(values)] = values
    return bf16(v).reshape(1, 128)


def eight_blocks():
    rng = np.random.default_rng(77)
    blocks = [W.activation(1, 128, 1)[0],
              W.gradient(1, 128, 2, tiny_half=True, tiny_frac=1.0)[0],
              W.weight(1, 128, 3, spike_frac=0.02)[0],
              rng.integers(0, 0x7F80, size=128).astype(np.uint16),
              (rng.integers(0, 0x7F80, size=128) | (rng.integers(0, 2, size=128) << 15)).astype(np.uint16),
              rng.integers(0x3F00, 0x4100, size=128).astype(np.uint16),
              rng.integers(0, 0x0100, size=128).astype(np.uint16),
              np.where(rng.random(128) < 0.5, 0, rng.integers(0x3000, 0x4800, size=128)).astype(np.uint16)]
    return np.stack(blocks)


# ---------------------------------------------------------------- de-scale, bit for bit

def _rounded_quotient_bits(codes, scale, ebits, mbits):
    """The OTHER plausible de-scale, value(code) / scale rounded once to binary32 and then to BF16: what the test below
    must be able to tell apart from the multiplication by fl32(1 / scale)."""
    s = Fraction(float(np.float32(scale)))
    out = []
    for c in codes:
        v = R.fl32(R.fp8_decode(int(c), ebits, mbits) / s)
        b = R.bf16_rne_bits(v)
        out.append(b | (0x8000 if v == 0 and int(c) & 0x80 else 0))
    return out


@pytest.mark.parametrize("scaling", ["fp32_amax", "gam"])
def test_dequantize_and_fake_quantize_bit_for_bit_against_exact_rationals(oracle, scaling):
    xb = eight_blocks()
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=1.0, scaling=scaling, want_fake=True)   # th = 1: every finite block stays E4M3
    assert np.all(a.mask == 0)
    back = oracle.dequantize(a.fp8, a.scale, a.mask, None, "sub1x128")
    for p in range(xb.shape[0]):
        s = float(a.scale[p])
        want = R.dequantize_block(a.fp8[p], s)
        assert list(back[p]) == want, f"de-quantize, block {p}"
        assert list(a.fake[p]) == want, f"fake quantization, block {p}"
    assert sum(1 for p in range(8) if R._mant_exp(Fraction(float(a.scale[p])))[0] != 1) >= 6      # not powers of two


# Scales (binary32 bit patterns) for which, on some codes, multiplying by fl32(1 / s) and dividing by s round to
# DIFFERENT BF16 values.  With scales that come from 448 / amax of a BF16 amax the two only differ when the result is
# a BF16 subnormal (q * amax / 448 never comes close to a rounding boundary of the 8-bit grid otherwise), so the
# de-quantize entry point is pinned with free scales, and the fused output with a block of tiny values below.
_E4M3_SCALES = [0x431A14DE, 0x3F7172CC, 0x443B9A61, 0x3DCA7FB6, 0x3FF967B9, 0x4070783D]
_E5M2_SCALE = 0x3F76A40E


def test_dequantize_is_a_multiplication_by_the_rounded_reciprocal(oracle):
    e4 = np.array(list(range(0x00, 0x7F)) + list(range(0x80, 0xFF)) + [0, 0], np.uint8)         # every finite E4M3 code
    e5 = np.array(list(range(0x00, 0x7C)) + list(range(0x80, 0xFC)) + [0] * 8, np.uint8)       # every finite E5M2 code
    n4 = len(_E4M3_SCALES)
    codes = np.stack([e4] * n4 + [e5])                                                          # (7, 256): two blocks per row
    scale = np.array(_E4M3_SCALES + [_E5M2_SCALE], np.uint32).view(np.float32)
    mask = np.array([0] * n4 + [2], np.uint8)
    back = oracle.dequantize(codes, np.repeat(scale, 2), np.repeat(mask, 2), None, "sub1x128")
    for p in range(n4 + 1):
        fmt = (5, 2) if mask[p] == 2 else (4, 3)
        want = R.dequantize_block(codes[p], float(scale[p]), *fmt)
        assert list(back[p]) == want, f"row {p}"
        other = _rounded_quotient_bits(codes[p], float(scale[p]), *fmt)
        assert sum(1 for u, v in zip(want, other) if u != v) >= 2, f"row {p} cannot tell the two arithmetics apart"


def test_fake_quantize_of_tiny_blocks_uses_the_rounded_reciprocal(oracle):
    """Blocks whose amax is a tiny BF16 normal: their de-quantized values are BF16 subnormals, where the product with
    fl32(1 / s) and the quotient by s round differently; the fused fake-quantized output must be the product."""
    apart = 0
    rows = []
    for amax_bits in (0x04B1, 0x03E2, 0x040B, 0x040D, 0x03E9, 0x03ED, 0x03EF):
        rows.append(np.array([amax_bits] + list(range(1, 128)), np.uint16))                  # amax and every smaller subnormal
    xb = np.stack(rows)
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=1.0, want_fake=True)
    assert np.all(a.mask == 0)
    for p in range(xb.shape[0]):
        ref = R.analyze_block(xb[p], threshold=1.0)
        assert ref["codes"] == list(a.fp8[p]) and ref["scale"] == float(a.scale[p])
        want = R.dequantize_block(a.fp8[p], float(a.scale[p]))
        assert list(a.fake[p]) == want, f"block {p}"
        apart += sum(1 for u, v in zip(want, _rounded_quotient_bits(a.fp8[p], float(a.scale[p]), 4, 3)) if u != v)
    assert apart >= 3


def test_dequantize_e5m2_block_bit_for_bit_against_exact_rationals(oracle):
    """Three-way recipe: a block whose small half flushes in E4M3 but is held by E5M2 is kept in E5M2 (Eq. 3-4) and
    de-quantized from its E5M2 codes with the E5M2 scale."""
    rng = np.random.default_rng(5)
    big = rng.uniform(1.0, 1.99, size=64).astype(np.float32)
    small = (rng.uniform(1.0, 1.99, size=64) * 2.0 ** -20).astype(np.float32)
    xb = W.f32_to_bf16_bits(np.concatenate([big, small]) * rng.choice([-1.0, 1.0], size=128).astype(np.float32)).reshape(1, 128)
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats="e4m3|e5m2|bf16", want_fake=True)
    assert a.mask[0] == 2
    s5 = float(a.scale[0])
    assert R._mant_exp(Fraction(s5))[0] != 1
    ref = R.analyze_block(xb[0], crit="e4m3_vs_e5m2", three_way=True)
    assert ref["choice"] == "e5m2" and ref["scale"] == s5 and ref["codes"] == list(a.fp8[0])
    want = R.dequantize_block(a.fp8[0], s5, 5, 2)
    back = oracle.dequantize(a.fp8, a.scale, a.mask, None, "sub1x128")
    assert list(back[0]) == want and list(a.fake[0]) == want


def test_descale_handworked_elements(oracle):
    """amax = 3 gives s = fl32(448/3) = 149.33332824707031 (0x43155555) and fl32(1/s) = 0.0066964286379516 (0x3BDB6DB7);
    the code of y = fl32(3 s) = 448 is 0x7E and de-scales to fl32(448 * 0.00669642863...) = 3.0 -> BF16 0x4040;
    x = 1 scales to 149.33333 -> nearest E4M3 value 144 (0x71) -> 144 * s_inv = 0.96428573 -> BF16 0x3F77 (0.96484375)."""
    xb = one_block([3.0, 1.0, -1.0])
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=1.0, want_fake=True)
    assert np.array([a.scale[0]], np.float32).view(np.uint32)[0] == 0x43155555
    assert list(a.fp8[0][:3]) == [0x7E, 0x71, 0xF1]
    assert list(a.fake[0][:4]) == [0x4040, 0x3F77, 0xBF77, 0x0000]
    back = oracle.dequantize(a.fp8, a.scale, a.mask, None, "sub1x128")
    assert np.array_equal(back, a.fake)


def test_dequantize_without_fallback_payload_leaves_bf16_blocks_untouched(oracle):
    """Interface rule (Section 4, Figure 4: the fallback operand is used as it is): with no BF16 payload passed,
    a block whose mask says BF16 is not written at all -- the caller's y may already hold it -- while E4M3 blocks are
    de-quantized as usual."""
    keep = one_block([3.0, 1.0, -1.0])
    fall = one_block([448.0] + [2.0 ** -12] * 100)                     # 100 of 101 non-zeros flush: BF16
    a = oracle.analyze_quantize(np.vstack([keep, fall]), "sub1x128", threshold=0.045)
    assert list(a.mask) == [0, 1]
    back = oracle.dequantize(a.fp8, a.scale, a.mask, None, "sub1x128", fill=0xABCD)
    assert list(back[0][:4]) == [0x4040, 0x3F77, 0xBF77, 0x0000]
    assert (back[1] == 0xABCD).all()
    with_payload = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, "sub1x128", fill=0xABCD)
    assert np.array_equal(with_payload[1], fall[0]) and np.array_equal(with_payload[0], back[0])


# ---------------------------------------------------------------- tensor-wide decision under Eq. (3)

def _eq3_pair(n_flushed):
    """Two 1x128 blocks with amax 448 (s = 1, s5 = 128, both exact).
    Block A: 448 and 127 values of 288.  288 = 256 + 32 is on E4M3's grid (step 32 in [256, 448]) but halfway between
    E5M2's 256 and 320 (step 64): the tie goes to the even code, 256, so each costs 32/288 = 1/9 in E5M2 and nothing
    in E4M3.  err4 = 0, err5 = 127/9 = 14.11: alone, E4M3.
    Block B: 448 and n_flushed values of 2^-12, zeros elsewhere.  2^-12 is below half of E4M3's smallest subnormal
    (flushed: 1 each) and 128 * 2^-12 = 2^-5 is an E5M2 normal (exact: 0).  err4 = n_flushed, err5 = 0: alone, BF16."""
    a = one_block([448.0] + [288.0] * 127)
    b = one_block([448.0] + [2.0 ** -12] * n_flushed)
    return np.vstack([a, b])


@pytest.mark.parametrize("n_flushed, tensor_mask", [(20, 1), (10, 0)])
def test_tensor_scope_eq3_totals_decide(oracle, n_flushed, tensor_mask):
    xb = _eq3_pair(n_flushed)
    part = oracle.analyze_quantize(xb, "sub1x128", scope="partition", crit="e4m3_vs_e5m2")
    assert list(part.err_sum) == [0.0, float(n_flushed)]
    assert part.err5_sum[0] == pytest.approx(127.0 / 9.0, rel=1e-15) and part.err5_sum[1] == 0.0
    assert list(part.mask) == [0, 1]
    # totals: sum err4 = n_flushed against sum err5 = 14.11 -> 20 is not below it (BF16, although block A alone is E4M3),
    # 10 is (E4M3, although block B alone is BF16)
    t = oracle.analyze_quantize(xb, "sub1x128", scope="tensor", crit="e4m3_vs_e5m2", bf16_fill=0xBEEF)
    assert list(t.mask) == [tensor_mask, tensor_mask]
    assert np.array_equal(t.fp8, part.fp8) and np.array_equal(t.err5_sum, part.err5_sum)
    assert np.array_equal(t.bf16, xb if tensor_mask else np.full_like(xb, 0xBEEF))


def test_tensor_scope_eq3_tie_is_bf16(oracle):
    """Totals that tie exactly (0 = 0: everything exactly representable in both formats) are not "strictly below"."""
    xb = np.vstack([one_block([448.0] * 128), one_block([448.0, 224.0, 112.0])])
    t = oracle.analyze_quantize(xb, "sub1x128", scope="tensor", crit="e4m3_vs_e5m2")
    assert t.err_sum.sum() == 0.0 and t.err5_sum.sum() == 0.0 and list(t.mask) == [1, 1]


# ---------------------------------------------------------------- near-threshold band of the statistics

def test_near_threshold_band_is_closed(oracle):
    """|metric - th| <= near_tol * th counts the edge itself: th = 1/4, near_tol = 1/2 -> band [1/8, 3/8], all exact
    in binary32.  Blocks with metric 1/8 and 3/8 (16 and 48 flushed of 128) are on the edge and count, as does 1/4;
    the next binary32 above 3/8 and the one below 1/8 do not."""
    nnz = np.full(5, 128, np.uint32)
    up = np.nextafter(np.float32(48.0), np.float32(100.0))
    dn = np.nextafter(np.float32(16.0), np.float32(0.0))
    err = np.array([16.0, 48.0, 32.0, up, dn], np.float32)
    mask = np.array([0, 1, 1, 1, 0], np.uint8)
    st = oracle.select_stats(err, nnz, mask, 5, 128, "sub1x128", threshold=0.25, near_tol=0.5)
    assert st["n_near_threshold"] == 3
    st = oracle.select_stats(err[:2], nnz[:2], mask[:2], 2, 128, "sub1x128", threshold=0.25, near_tol=0.5)
    assert st["n_near_threshold"] == 2
    st = oracle.select_stats(err[3:], nnz[3:], mask[3:], 2, 128, "sub1x128", threshold=0.25, near_tol=0.5)
    assert st["n_near_threshold"] == 0
