"""Pins for the oracle's GAM and E8M0-only scaling (Algorithm 1), none of which re-uses the oracle's
own arithmetic: hand-worked cases, the algorithm's stated guarantees (no saturation, at most one
binade lost, one mantissa for the whole tensor, the tensor amax kept at full precision), an
exact-rational re-implementation, and the special cases that reduce to FP32 amax scaling."""
from fractions import Fraction

import numpy as np
import pytest

import refmodel as R
from paper_2512_22804_amd import workloads as W

F32 = np.float32


def bf16(v):
    return int(W.f32_to_bf16_bits(np.array([v], np.float32))[0])


def block_tensor(amaxes, cols=128, seed=0):
    """One 1x128 block per entry, whose largest magnitude is exactly the given BF16 value."""
    rng = np.random.default_rng(seed)
    x = np.zeros((len(amaxes), cols), np.uint16)
    for i, a in enumerate(amaxes):
        v = (rng.uniform(-1, 1, cols) * float(a) * 0.999).astype(np.float32)
        b = W.f32_to_bf16_bits(v)
        b[(b & 0x7FFF) > bf16(a)] = bf16(a)
        b[rng.integers(cols)] = bf16(a) | (0x8000 if rng.random() < 0.5 else 0)
        x[i] = b
    return x


# ---- hand-worked cases (Algorithm 1 followed by hand; 448 = 1.75 * 2^8) -------------------------
#   g_amax = 1:    s_g = 448       = 1.75 * 2^8            -> m_g = 1.75
#     b_amax = 1:    s_b = 448       m_b = 1.75  >= m_g  -> e = 8,  applied 1.75 * 2^8 = 448
#     b_amax = 0.75: s_b = 597.33..  = 1.1666.. * 2^9, m_b < m_g -> e = 9 - 1 = 8, applied 448
#     b_amax = 0.5:  s_b = 896       = 1.75 * 2^9         -> e = 9,  applied 896
#     b_amax = 2^-10: s_b = 448 * 1024 = 1.75 * 2^18      -> e = 18
#   g_amax = 3:    s_g = fl32(149.33..) = 1.1666.. * 2^7   -> m_g = fl32(448/3) / 128
#     b_amax = 1:    s_b = 448, m_b = 1.75 >= m_g         -> e = 8,  applied 2 * fl32(448/3)
#     b_amax = 2:    s_b = 224 = 1.75 * 2^7               -> e = 7,  applied fl32(448/3)
#     b_amax = 3:    the block that holds the tensor amax -> e = 7,  applied s_g itself
S3 = float(F32(448.0) / F32(3.0))
WORKED = [
    (1.0, 1.0, 448.0, 8), (1.0, 0.75, 448.0, 8), (1.0, 0.5, 896.0, 9), (1.0, 2.0 ** -10, 448.0 * 1024, 18),
    (3.0, 1.0, 2 * S3, 8), (3.0, 2.0, S3, 7), (3.0, 3.0, S3, 7),
]


@pytest.mark.parametrize("g_amax,b_amax,want_scale,want_e", WORKED)
def test_gam_hand_worked(oracle, g_amax, b_amax, want_scale, want_e):
    m_g = oracle.group_mantissa(g_amax)
    s, e = oracle.gam_block_scale(b_amax, m_g)
    assert (s, e) == (want_scale, want_e)


def test_gam_hand_worked_through_the_pipeline(oracle):
    x = block_tensor([3.0, 1.0, 2.0, 0.75])
    a = oracle.analyze_quantize(x, "sub1x128", scaling="gam")
    # 0.75 = 3/4: s_b = 4 * s_g has the group's own mantissa, so m_g <= m_b holds with equality and e stays 9
    assert list(a.scale) == [F32(S3), F32(2 * S3), F32(S3), F32(4 * S3)]
    assert list(a.e8m0) == [127 + 7, 127 + 8, 127 + 7, 127 + 9]
    assert a.group_mantissa == int(np.array([S3], np.float32).view(np.uint32)[0] & 0x7FFFFF)
    # E8M0-only: the power of two at or below 448/amax:  149.3 -> 128, 448 -> 256, 224 -> 128, 597.3 -> 512
    b = oracle.analyze_quantize(x, "sub1x128", scaling="e8m0")
    assert list(b.scale) == [128.0, 256.0, 128.0, 512.0]
    assert list(b.e8m0) == [127 + 7, 127 + 8, 127 + 7, 127 + 9]
    assert b.group_mantissa == 0


# ---- the algorithm's guarantees, over many (group amax, block amax) pairs --------------------------
def amax_pairs():
    rng = np.random.default_rng(11)
    pats = np.unique(np.concatenate([rng.integers(1, 0x7F80, 400), [1, 2, 0x7F, 0x80, 0x3F80, 0x7F7F, 0x7F00, 0x0080]]))
    out = []
    for g in pats:
        for b in rng.choice(pats[pats <= g], size=min(6, int((pats <= g).sum())), replace=False):
            out.append((int(g), int(b)))
        out.append((int(g), int(g)))
    return out


def test_gam_guarantees(oracle):
    for g_bits, b_bits in amax_pairs():
        g_amax, b_amax = float(R.bf16_to_f32(g_bits)), float(R.bf16_to_f32(b_bits))
        s_b = Fraction(float(R.scale_of(b_amax, 448.0)))
        m_g = oracle.group_mantissa(g_amax)
        s, e = oracle.gam_block_scale(b_amax, m_g)
        sf = Fraction(s)
        assert s_b / 2 < sf <= s_b, (g_bits, b_bits)                  # never above the ideal scale, at most one binade below
        if s_b == Fraction(float(np.finfo(np.float32).max)):          # 448/amax overflowed (R2): nothing more to check
            continue
        assert Fraction(b_amax) * sf <= 448 * (1 + Fraction(1, 2 ** 23))   # no saturation of the block amax
        assert sf == Fraction(m_g) * Fraction(2) ** e                  # mantissa * 2^e, exactly
        bits = int(np.array([s], np.float32).view(np.uint32)[0])
        g_frac = int(np.array([float(R.scale_of(g_amax, 448.0))], np.float32).view(np.uint32)[0]) & 0x7FFFFF
        assert bits & 0x7FFFFF == g_frac                               # one mantissa for the whole tensor
        assert (bits >> 23) == e + 127
        if b_bits == g_bits:
            assert sf == s_b                                           # the tensor amax keeps its full-precision scale
        # the exact-rational re-implementation agrees
        rs, re_, _ = R.gam_scale(b_amax, g_amax, 448.0)
        assert (rs, re_) == (sf, e)
        # E8M0 only: a power of two, floor of the ideal scale
        s8, e8 = oracle.gam_block_scale(b_amax, 1.0)
        assert Fraction(s8) == Fraction(2) ** e8 and Fraction(s8) <= s_b < 2 * Fraction(s8)


def test_gam_e5m2_side_and_edge_amax(oracle):
    # the E5M2 yardstick of Eq. (3) gets its own group mantissa from 57344 / g_amax
    for g_bits, b_bits in amax_pairs()[::7]:
        g_amax, b_amax = float(R.bf16_to_f32(g_bits)), float(R.bf16_to_f32(b_bits))
        s, e = oracle.gam_block_scale(b_amax, oracle.group_mantissa(g_amax, 57344.0), 57344.0)
        rs, re_, _ = R.gam_scale(b_amax, g_amax, 57344.0)
        assert (Fraction(s), e) == (rs, re_)
    # zero and non-finite amax follow the scale rule first (s = 1), then the algorithm
    assert oracle.group_mantissa(0.0) == 1.0 and oracle.group_mantissa(float("inf")) == 1.0
    assert oracle.gam_block_scale(0.0, 1.75) == (0.875, -1)      # s_b = 1 = 1.0 * 2^0, m_g > m_b -> 1.75 * 2^-1
    assert oracle.gam_block_scale(0.0, 1.0) == (1.0, 0)
    assert oracle.group_mantissa(3.0, scaling="e8m0") == 1.0


def test_gam_when_only_the_e5m2_scale_overflows(oracle):
    # amax = 2^-118: 448/amax = 1.75 * 2^126 is finite, 57344/amax overflows to FLT_MAX (R2), so the two formats
    # have different group mantissas (1.75 and 2 - 2^-23)
    v = np.ldexp(np.random.default_rng(4).uniform(-1, 1, (2, 128)), -118).astype(np.float32)
    x = W.f32_to_bf16_bits(v)
    x[0, 0] = bf16(2.0 ** -118)
    x[1] = x[1] & 0x8000 | np.minimum(x[1] & 0x7FFF, bf16(2.0 ** -121))
    a = oracle.analyze_quantize(x, "sub1x128", "partition", "e4m3_vs_e5m2", scaling="gam")
    for p in range(2):
        r = R.analyze_block(x[p], "e4m3_vs_e5m2", scaling="gam", g_amax=2.0 ** -118)
        assert a.err_sum[p] == pytest.approx(float(r["err_sum"]), rel=1e-12)
        assert a.err5_sum[p] == pytest.approx(float(r["err5_sum"]), rel=1e-12)
    assert oracle.group_mantissa(2.0 ** -118, 57344.0) == 2.0 - 2.0 ** -23


# ---- whole pipeline against the exact-rational model ---------------------------------------------------
@pytest.mark.parametrize("scaling", ["gam", "e8m0"])
@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
def test_pipeline_matches_rational_model(oracle, scaling, crit):
    x = W.gradient(6, 256, 77, tiny_half=True)
    x[2, :128] = 0
    a = oracle.analyze_quantize(x, "sub1x128", "partition", crit, 0.045, scaling=scaling)
    g_amax = float(R.bf16_to_f32(int((x & 0x7FFF).max())))
    blocks = x.reshape(6, 2, 128).reshape(12, 128)
    for p in range(12):
        r = R.analyze_block(blocks[p], crit, 0.045, scaling=scaling, g_amax=g_amax)
        assert a.scale[p] == F32(r["scale"])
        assert list(a.fp8.reshape(6, 2, 128).reshape(12, 128)[p]) == r["codes"]
        assert a.err_sum[p] == pytest.approx(float(r["err_sum"]), rel=1e-12, abs=1e-300)
        if crit == "e4m3_vs_e5m2":
            assert a.err5_sum[p] == pytest.approx(float(r["err5_sum"]), rel=1e-12, abs=1e-300)
        assert a.mask[p] == (0 if r["fp8"] else 1)
        s_rebuilt = np.ldexp(F32(1.0) + F32(a.group_mantissa) / F32(2 ** 23), int(a.e8m0[p]) - 127)
        assert F32(s_rebuilt) == a.scale[p]                     # scale = stored mantissa and exponent, nothing else


# ---- special cases that reduce to FP32 amax scaling ---------------------------------------------------------
def test_gam_equals_fp32_scaling_when_one_block_or_equal_amaxes(oracle):
    x = W.gradient(64, 256, 5)
    for crit in ("mean_rel_err", "e4m3_vs_e5m2"):
        a = oracle.analyze_quantize(x, "tensor", "partition", crit, scaling="fp32_amax")
        b = oracle.analyze_quantize(x, "tensor", "partition", crit, scaling="gam")
        assert np.array_equal(a.fp8, b.fp8) and np.array_equal(a.scale, b.scale)
        assert np.array_equal(a.err_sum, b.err_sum) and np.array_equal(a.err5_sum, b.err5_sum)
        assert np.array_equal(a.mask, b.mask)
    y = block_tensor([1.5] * 8, seed=3)
    a = oracle.analyze_quantize(y, "sub1x128", scaling="fp32_amax")
    b = oracle.analyze_quantize(y, "sub1x128", scaling="gam")
    assert np.array_equal(a.fp8, b.fp8) and np.array_equal(a.scale, b.scale) and np.array_equal(a.err_sum, b.err_sum)


def test_power_of_two_data_is_exact_under_every_scaling(oracle):
    # values +-2^k within 8 binades of the block amax are E4M3 numbers under any scale of the form c * 2^e with
    # c <= 1.75 only if c is a power of two: exact under E8M0-only scaling (closed form: zero error)
    rng = np.random.default_rng(9)
    v = np.ldexp(1.0, rng.integers(-6, 1, (4, 128))).astype(np.float32) * rng.choice([-1, 1], (4, 128))
    x = W.f32_to_bf16_bits(v.astype(np.float32))
    a = oracle.analyze_quantize(x, "sub1x128", scaling="e8m0")
    assert np.all(a.err_sum == 0.0) and np.all(a.mask == 0)
    y = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, "sub1x128")
    assert np.array_equal(y, x)


def test_gam_never_loses_more_than_one_binade_of_range(oracle):
    # the metric under GAM is at least that of FP32 scaling minus rounding noise only through flushing: the number
    # of flushed (non-zero -> 0) elements under GAM is between FP32's and what FP32 would flush with half the scale
    x = W.gradient(32, 512, 21, tiny_half=True)
    f = oracle.analyze_quantize(x, "sub1x128", scaling="fp32_amax")
    g = oracle.analyze_quantize(x, "sub1x128", scaling="gam")
    nz = (x & 0x7FFF) != 0
    flushed_f = (((f.fp8 & 0x7F) == 0) & nz).reshape(32, 4, 128).sum(-1).reshape(-1)
    flushed_g = (((g.fp8 & 0x7F) == 0) & nz).reshape(32, 4, 128).sum(-1).reshape(-1)
    assert np.all(flushed_g >= flushed_f)
    xs = W.bf16_bits_to_f32(x).reshape(32, 4, 128).reshape(-1, 128)
    half = np.abs(xs * (f.scale[:, None] / 2)) <= 2.0 ** -10          # at or below half the smallest subnormal: flushed at s/2
    bound = (half & nz.reshape(-1, 128)).sum(-1)
    assert np.all(flushed_g <= np.maximum(bound, flushed_f))


# ---- several groups per tensor (the partition G of Algorithm 1 taken as bands of rows) ----------------------------
def test_gam_row_band_groups_hand_worked(oracle):
    """Four 1x128 blocks, groups of two rows.  Band 0 holds amax 3 and 1: m_g = mantissa(448/3) = 1.1666.., the block of
    amax 1 (s_b = 448 = 1.75 * 2^8, m_b >= m_g) gets 1.1666.. * 2^8.  Band 1 holds amax 5 and 7: s_g = 64, m_g = 1; the
    block of amax 5 (s_b = 89.6 = 1.4 * 2^6) gets 2^6.  As ONE group (amax 7, m_g = 1) the first two blocks would get 2^7 and
    2^8: the bands keep more of their blocks' range."""
    x = block_tensor([3.0, 1.0, 5.0, 7.0])
    a = oracle.analyze_quantize(x, "sub1x128", scaling="gam", gam_group_rows=2)
    assert list(a.scale) == [F32(S3), F32(2 * S3), F32(64.0), F32(64.0)]
    assert list(a.e8m0) == [127 + 7, 127 + 8, 127 + 6, 127 + 6]
    frac3 = int(np.array([S3], np.float32).view(np.uint32)[0]) & 0x7FFFFF
    assert a.group_mantissas.tolist() == [[frac3, frac3], [0, 0]]          # 57344 / amax has the mantissa of 448 / amax
    one = oracle.analyze_quantize(x, "sub1x128", scaling="gam")
    assert list(one.scale) == [F32(128.0), F32(256.0), F32(64.0), F32(64.0)]
    assert one.group_mantissas.tolist() == [[0, 0]]
    # a band that covers the tensor is the single group; E8M0-only scaling has no groups to speak of
    whole = oracle.analyze_quantize(x, "sub1x128", scaling="gam", gam_group_rows=4)
    assert np.array_equal(whole.scale, one.scale) and np.array_equal(whole.fp8, one.fp8)
    e8 = oracle.analyze_quantize(x, "sub1x128", scaling="e8m0", gam_group_rows=2)
    assert np.array_equal(e8.scale, oracle.analyze_quantize(x, "sub1x128", scaling="e8m0").scale)


@pytest.mark.parametrize("gran,shape,band,crit", [("sub1x128", (10, 256), 4, "mean_rel_err"), ("sub1x128", (6, 128), 2, "e4m3_vs_e5m2"),
                                                  ("channel_row", (9, 384), 2, "mean_rel_err"), ("block128", (384, 256), 128, "mean_rel_err"),
                                                  ("block64", (192, 128), 128, "e4m3_vs_e5m2"), ("sub128x1", (256, 8), 128, "mean_rel_err")])
def test_gam_row_band_groups_match_rational_model(oracle, gran, shape, band, crit):
    """Every block against the exact-rational Algorithm 1 with the amax of ITS band as group amax (the last band may be
    shorter), and the stored form (band mantissa + E8M0 byte) rebuilds the applied scale."""
    rows, cols = shape
    rng = np.random.default_rng(rows * 7 + cols)
    x = (np.exp2(rng.uniform(-6.0, 6.0, size=(rows, cols))) * rng.choice([-1.0, 1.0], size=(rows, cols))).astype(np.float32)
    x *= np.exp2(rng.integers(-8, 8, size=(rows, 1))).astype(np.float32)            # row magnitudes differ: the bands' amaxes too
    xb = W.f32_to_bf16_bits(x)
    a = oracle.analyze_quantize(xb, gran, "partition", crit, 0.045, scaling="gam", gam_group_rows=band)
    pr, pc = {"sub1x128": (1, 128), "channel_row": (1, cols), "block128": (128, 128), "block64": (64, 64), "sub128x1": (128, 1)}[gran]
    gc = cols // pc
    n_groups = -(-rows // band)
    assert a.group_mantissas.shape == (n_groups, 2)
    mags = xb & 0x7FFF
    for p in range(a.mask.size):
        r0, c0 = (p // gc) * pr, (p % gc) * pc
        g = r0 // band
        g_amax = float(R.bf16_to_f32(int(mags[g * band:(g + 1) * band].max())))
        blk = xb[r0:r0 + pr, c0:c0 + pc].reshape(-1)
        if blk.size > 2048 and (p > 0 or blk.size > 8192):
            # large blocks: only the scale of Algorithm 1 (what the grouping changes); everything after the scale is pinned elsewhere
            b_amax = float(R.bf16_to_f32(int((blk & 0x7FFF).max())))
            assert Fraction(float(a.scale[p])) == R.gam_scale(b_amax, g_amax, 448.0)[0], (p, g)
        else:
            r = R.analyze_block(blk, crit, 0.045, scaling="gam", g_amax=g_amax)
            assert a.scale[p] == F32(r["scale"]), (p, g)
            assert list(a.fp8[r0:r0 + pr, c0:c0 + pc].reshape(-1)) == r["codes"]
            assert a.err_sum[p] == pytest.approx(float(r["err_sum"]), rel=1e-12, abs=1e-300)
            assert a.mask[p] == (0 if r["fp8"] else 1)
        rebuilt = np.ldexp(F32(1.0) + F32(int(a.group_mantissas[g, 0])) / F32(2 ** 23), int(a.e8m0[p]) - 127)
        assert F32(rebuilt) == a.scale[p]


def test_gam_row_band_groups_guarantees(oracle):
    """Per band: no saturation, at most one binade lost against the block's own FP32 scale, and the block that holds the
    band's amax is scaled by s_g itself (the band's amax is kept at full precision)."""
    rng = np.random.default_rng(3)
    rows, cols, band = 64, 128, 8
    x = (rng.standard_normal((rows, cols)) * np.exp2(rng.integers(-20, 20, size=(rows, 1)))).astype(np.float32)
    xb = W.f32_to_bf16_bits(x)
    a = oracle.analyze_quantize(xb, "sub1x128", scaling="gam", gam_group_rows=band)
    own = oracle.analyze_quantize(xb, "sub1x128", scaling="fp32_amax")
    assert np.all(a.scale <= own.scale) and np.all(a.scale > own.scale / 2)
    y = W.bf16_bits_to_f32(xb) * a.scale[:, None]
    assert np.all(np.abs(y) <= 448.0 * (1 + 2.0 ** -22))
    for g in range(rows // band):
        top = g * band + int(np.argmax(a.amax[g * band:(g + 1) * band]))
        assert a.scale[top] == own.scale[top]
    # more groups never scale a block down further than one group does
    one = oracle.analyze_quantize(xb, "sub1x128", scaling="gam")
    assert np.all(a.scale >= one.scale / 2) and (a.scale != one.scale).any()


def test_gam_row_band_groups_must_hold_whole_blocks(oracle):
    xb = W.activation(256, 256, 9)
    with pytest.raises(ValueError):
        oracle.analyze_quantize(xb, "block128", scaling="gam", gam_group_rows=64)
    with pytest.raises(ValueError):
        oracle.analyze_quantize(xb, "channel_col", scaling="gam", gam_group_rows=128)      # a column block spans every band
    with pytest.raises(ValueError):
        oracle.analyze_quantize(xb, "tensor", scaling="gam", gam_group_rows=128)
