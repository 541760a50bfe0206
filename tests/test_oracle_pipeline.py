"""Pins for the oracle's analyse-select-quantize pipeline: closed forms, hand-worked blocks,
invariants, the paper's flushed-fraction remark, and an exact-rational brute force on small
inputs (tests/refmodel.py).  No expected value here comes from the oracle itself."""
import math
from fractions import Fraction

import numpy as np
import pytest

import refmodel as R
from paper_2512_22804_amd import workloads as W

TH = 0.045


def bf16(v):
    """BF16 bits of values that are exactly representable (asserted)."""
    a = np.asarray(v, dtype=np.float32)
    b = W.f32_to_bf16_bits(a)
    assert np.array_equal(W.bf16_bits_to_f32(b), a), "test value is not a BF16 number"
    return b


def e4m3_grid():
    """All positive finite E4M3 values."""
    vals = R.fp8_values(4, 3)
    return np.array(sorted(float(v) for v in vals.values() if v > 0), dtype=np.float32)


# ---------------------------------------------------------------- closed forms (power-of-two scale)

@pytest.mark.parametrize("gran,shape", [("sub1x128", (4, 256)), ("block128", (128, 256)), ("tensor", (8, 128))])
@pytest.mark.parametrize("j", [-20, -3, 0, 5, 40])
def test_power_of_two_scale_closed_form(oracle, gran, shape, j):
    """Values drawn from the E4M3 grid times 2^(j-8), every block containing 448*2^(j-8) = 1.75*2^j:
    then s = 2^(8-j) exactly, every y is an E4M3 value, codes are known by construction, the
    error is exactly 0, E4M3 is selected and de-quantizing returns the input bits."""
    rng = np.random.default_rng(100 + j)
    grid = e4m3_grid()
    # only normal E4M3 values and the largest subnormals keep 8 significant bits -> all BF16-exact
    k = rng.integers(0, len(grid), size=shape)
    sign = rng.integers(0, 2, size=shape) * 2 - 1
    y = grid[k] * sign.astype(np.float32)
    y[:, ::128] = 448.0                              # every 1x128 / 128x128 / tensor block holds the amax
    x = (y * np.float32(2.0 ** (j - 8))).astype(np.float32)
    xb = bf16(x)
    a = oracle.analyze_quantize(xb, gran, threshold=TH)
    assert np.all(a.amax == np.float32(1.75 * 2.0 ** j))
    assert np.all(a.scale == np.float32(2.0 ** (8 - j)))
    want_codes = np.array([[R.fp8_encode(v, 4, 3) for v in row] for row in y], dtype=np.uint8)
    assert np.array_equal(a.fp8, want_codes)
    assert np.all(a.err_sum == 0.0) and np.all(a.err_sum_unscaled == 0.0)
    assert np.all(a.nnz == (128 if gran == "sub1x128" else 128 * 128 if gran == "block128" else x.size))
    assert np.all(a.mask == 0)
    back = oracle.dequantize(a.fp8, a.scale, a.mask, None, gran)
    assert np.array_equal(back, xb)


# ---------------------------------------------------------------- hand-worked blocks

def one_block(values):
    x = np.zeros((1, 128), dtype=np.float32)
    x[0, :len(values)] = values
    return bf16(x)


def test_all_zero_block(oracle):
    xb = np.zeros((2, 128), dtype=np.uint16)
    xb[1, 5] = 0x8000                                   # a negative zero is still a zero
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH)
    assert np.all(a.amax == 0) and np.all(a.scale == 1.0) and np.all(a.nnz == 0)
    assert np.all(a.err_sum == 0) and np.all(a.mask == 0)          # Eq. (2): metric 0 < th -> E4M3
    assert a.fp8[1, 5] == 0x80 and a.fp8.sum() == 0x80
    b = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2")
    assert np.all(b.mask == 1)                                      # Eq. (3) strict: 0 < 0 is false


def test_flushed_block_falls_back(oracle):
    """One element 448 and 127 elements 2^-11: s = 1, y = 2^-11 < 2^-10 flushes, each contributes
    exactly 1 -> err_sum = 127, metric = 127/128 -> BF16, and the fallback payload is the input."""
    xb = one_block([448.0] + [2.0 ** -11] * 127)
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH, bf16_fill=0xDEAD)
    assert a.scale[0] == 1.0 and a.amax[0] == 448.0 and a.nnz[0] == 128
    assert a.err_sum[0] == 127.0 and a.err_sum_unscaled[0] == 127.0
    assert a.mask[0] == 1
    assert a.fp8[0, 0] == 0x7E and np.all(a.fp8[0, 1:] == 0)
    assert np.array_equal(a.bf16, xb)
    back = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, "sub1x128")
    assert np.array_equal(back, xb)


def test_individual_error_terms(oracle):
    """s = 1 (amax 448).  2^-10 -> 0 (term 1); 3*2^-10 -> 2^-8 (term 1/3); 1.0625 -> 1.0
    (term 1/17); -1.1875 -> -1.25 (term 1/19); 2^-9 exact (term 0); zeros do not count."""
    xb = one_block([448.0, 2.0 ** -10, 3 * 2.0 ** -10, 1.0625, -1.1875, 2.0 ** -9, 0.0, -0.0])
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH)
    assert a.nnz[0] == 6
    want = 1 + Fraction(1, 3) + Fraction(1, 17) + Fraction(1, 19)
    assert a.err_sum[0] == pytest.approx(float(want), rel=1e-15)
    assert list(a.fp8[0, :8]) == [0x7E, 0x00, 0x02, 0x38, 0xBA, 0x01, 0x00, 0x80]
    assert a.mask[0] == 1                                # metric = 0.238 > 4.5 %


def test_saturation_term(oracle):
    """amax = 3 -> s = fl32(448/3); y = fl32(3*s) is within one ulp of 448 and encodes to 448; the
    term is |y-448|/y, at most 2^-23."""
    xb = one_block([3.0, -3.0, 1.5])
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH)
    s = np.float32(448.0) / np.float32(3.0)
    assert a.scale[0] == s
    assert list(a.fp8[0, :3]) == [0x7E, 0xFE, 0x76]
    y = float(np.float32(3.0) * s)
    y15 = float(np.float32(1.5) * s)
    assert a.err_sum[0] == pytest.approx(2 * abs(y - 448.0) / y + abs(y15 - 224.0) / y15, rel=1e-12, abs=1e-300)
    assert a.err_sum[0] < 3 * 2.0 ** -23 and a.mask[0] == 0


def test_subnormal_amax_clamps_scale(oracle):
    """amax below 448/FLT_MAX: the quotient overflows, s = FLT_MAX; y = x*FLT_MAX stays finite."""
    tiny = np.array([[0x0001, 0x0002, 0x8003] + [0] * 125], dtype=np.uint16)   # BF16 subnormals
    a = oracle.analyze_quantize(tiny, "sub1x128", threshold=TH)
    flt_max = float(np.finfo(np.float32).max)
    assert a.scale[0] == flt_max and a.nnz[0] == 3
    r = R.analyze_block(tiny[0])
    assert list(a.fp8[0]) == r["codes"]
    assert a.err_sum[0] == pytest.approx(float(r["err_sum"]), rel=1e-14)


def test_dynamic_range_beyond_e4m3_falls_back(oracle):
    """Half the block at 1.0, half at 2^-19: after scaling by 448 the small half sits at
    448*2^-19 < 2^-10 and flushes -> metric 0.5 -> BF16.  The same small half alone (its own
    amax) is exactly representable -> E4M3."""
    xb = one_block([1.0] * 64 + [2.0 ** -19] * 64)
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH)
    assert a.err_sum[0] == 64.0 and a.mask[0] == 1
    xs = one_block([2.0 ** -19] * 128)
    b = oracle.analyze_quantize(xs, "sub1x128", threshold=TH)
    assert b.err_sum[0] <= 128 * 2.0 ** -23 and b.mask[0] == 0


def test_nonfinite_block_policy(oracle):
    xb = one_block([1.0, 2.0, 3.0])
    xb = np.vstack([xb, xb, xb])
    xb[1, 7] = 0x7F80          # +Inf
    xb[2, 9] = 0xFFC1          # a NaN
    for crit in ("mean_rel_err", "e4m3_vs_e5m2"):
        a = oracle.analyze_quantize(xb, "sub1x128", crit=crit, threshold=TH)
        assert list(a.mask) == [0 if crit == "mean_rel_err" else a.mask[0], 1, 1]
        assert a.scale[1] == 1.0 and a.scale[2] == 1.0
        assert np.isinf(a.amax[1]) and np.isnan(a.amax[2])
        assert np.isinf(a.err_sum[1]) and np.isinf(a.err_sum[2])
        assert a.fp8[1, 7] == 0x7E and a.fp8[2, 9] == 0xFF and a.fp8[1, 0] == 0x38
    t = oracle.analyze_quantize(xb, "sub1x128", scope="tensor", threshold=TH)
    assert np.all(t.mask == 1)


# ---------------------------------------------------------------- invariants on random data

def random_operand(seed, rows=128, cols=256):
    return W.gradient(rows, cols, seed, tiny_half=True)


@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor"])
def test_elementwise_invariants(oracle, gran):
    xb = np.concatenate([W.activation(128, 256, 11), random_operand(12)], axis=0)
    a = oracle.analyze_quantize(xb, gran, threshold=TH)
    pr, pc = {"sub1x128": (1, 128), "block128": (128, 128), "tensor": xb.shape}[gran]
    x = W.bf16_bits_to_f32(xb)
    gc = xb.shape[1] // pc
    for p in range(len(a.mask)):
        br, bc = divmod(p, gc)
        blk = x[br * pr:(br + 1) * pr, bc * pc:(bc + 1) * pc]
        codes = a.fp8[br * pr:(br + 1) * pr, bc * pc:(bc + 1) * pc]
        assert a.amax[p] == np.abs(blk).max()
        assert a.nnz[p] == np.count_nonzero(blk)
        s = a.scale[p]
        y = (blk * s).astype(np.float32).astype(np.float64)
        q = np.vectorize(oracle.e4m3_decode)(codes)
        assert np.all(np.abs(q) <= 448.0)
        # amax lands on +-448
        assert np.all(np.abs(q[np.abs(blk) == a.amax[p]]) == 448.0)
        nz = blk != 0
        with np.errstate(divide="ignore", invalid="ignore"):
            t = np.where(q == 0, 1.0, np.abs(y - q) / np.abs(y))
        t = t[nz]
        assert np.all((t >= 0) & (t <= 1))
        yn = np.abs(y[nz]); qn = np.abs(q[nz])
        normal = (yn >= 2.0 ** -6) & (yn <= 448.0)
        assert np.all(t[normal] <= 2.0 ** -4)                     # half an ulp of a 3-bit mantissa
        assert np.all(np.abs(yn - qn)[yn < 2.0 ** -6] <= 2.0 ** -10)   # half a subnormal step
        assert a.err_sum[p] == pytest.approx(t.sum(), rel=1e-12)
        # the reading "evaluate Eq. (2) in the scaled domain" is faithful to the unscaled form
        assert abs(a.err_sum[p] - a.err_sum_unscaled[p]) <= 1e-5 * a.err_sum[p] + 1e-7 * max(1, a.nnz[p])


def test_mask_monotone_in_threshold(oracle):
    xb = random_operand(21, rows=256, cols=512)
    prev = None
    seen = set()
    for th in (0.0, 0.01, 0.02, 0.03, 0.045, 0.05, 0.2, 0.6, 1.01):
        m = oracle.analyze_quantize(xb, "sub1x128", threshold=th).mask
        if prev is not None:
            assert np.all(m <= prev)          # FP8 set only grows with the threshold
        prev = m
        seen.add(int(m.sum()))
    assert prev.sum() == 0 and len(seen) > 3  # th > 1 accepts everything; the mask really varied
    assert np.all(oracle.analyze_quantize(xb, "sub1x128", threshold=0.0).mask[
        oracle.analyze_quantize(xb, "sub1x128", threshold=0.0).err_sum > 0] == 1)


def test_metric_invariant_under_power_of_two_and_permutation(oracle):
    xb = W.activation(4, 256, 31)
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH)
    x = W.bf16_bits_to_f32(xb)
    b = oracle.analyze_quantize(bf16(x * np.float32(2.0 ** 20)), "sub1x128", threshold=TH)
    assert np.array_equal(a.fp8, b.fp8) and np.array_equal(a.err_sum, b.err_sum)
    assert np.array_equal(b.scale, a.scale * np.float32(2.0 ** -20))
    rng = np.random.default_rng(5)
    perm = rng.permutation(128)
    xp = xb.reshape(-1, 128)[:, perm].reshape(xb.shape)
    c = oracle.analyze_quantize(xp, "sub1x128", threshold=TH)
    assert np.array_equal(c.fp8.reshape(-1, 128), a.fp8.reshape(-1, 128)[:, perm])
    assert np.allclose(c.err_sum, a.err_sum, rtol=1e-13, atol=0)
    assert np.array_equal(c.amax, a.amax) and np.array_equal(c.nnz, a.nnz)


@pytest.mark.parametrize("gran", ["sub1x128", "block128"])
def test_tensor_scope_is_nnz_weighted_mean(oracle, gran):
    xb = random_operand(41, rows=256, cols=256)
    part = oracle.analyze_quantize(xb, gran, scope="partition", threshold=TH)
    m = part.err_sum.sum() / part.nnz.sum()
    for th, want in ((m * 1.001, 0), (m * 0.999, 1)):
        t = oracle.analyze_quantize(xb, gran, scope="tensor", threshold=th, bf16_fill=0xBEEF)
        assert np.all(t.mask == want)
        assert np.array_equal(t.fp8, part.fp8) and np.array_equal(t.err_sum, part.err_sum)
        assert np.array_equal(t.bf16, xb if want else np.full_like(xb, 0xBEEF))
    # not a mean of block means
    assert abs(part.metric().mean() - m) > 1e-6


def test_fallback_payload_only_where_masked(oracle):
    xb = random_operand(51, rows=128, cols=512)
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=TH, bf16_fill=0xABCD)
    assert 0 < a.mask.sum() < a.mask.size
    m = np.repeat(a.mask.reshape(128, 4), 128, axis=1).astype(bool)
    assert np.array_equal(a.bf16[m], xb[m]) and np.all(a.bf16[~m] == 0xABCD)
    back = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, "sub1x128")
    assert np.array_equal(back[m], xb[m])
    # de-quantized E4M3 values: within 2^-4 relative (normal range) plus BF16 re-rounding
    x = W.bf16_bits_to_f32(xb)[~m].astype(np.float64)
    y = W.bf16_bits_to_f32(back)[~m].astype(np.float64)
    big = np.abs(x) > 0
    amax_e = np.repeat(a.amax.reshape(128, 4), 128, axis=1)[~m]
    tol = np.maximum(np.abs(x) * (2.0 ** -4 + 2.0 ** -8), amax_e / 448.0 * 2.0 ** -10 * 1.01)
    assert np.all(np.abs(x - y)[big] <= tol[big])


def test_leading_dimension(oracle):
    xb = W.activation(128, 384, 61)
    dense = oracle.analyze_quantize(np.ascontiguousarray(xb[:, :256]), "block128", threshold=TH)
    padded = oracle.analyze_quantize(xb, "block128", threshold=TH, ld=384, cols=256)
    for f in ("fp8", "scale", "amax", "err_sum", "nnz", "mask"):
        assert np.array_equal(getattr(dense, f), getattr(padded, f))


# ---------------------------------------------------------------- the paper's flushed-fraction remark

def test_flushed_fraction_remark(oracle):
    """Section 4.1.3: about 2.4 % flushed values are enough to push the tensor error above 4.5 %.
    With log-uniform magnitudes the surviving values have mean relative error 2^-5/(2 ln 2) =
    2.254 % (closed form for round-to-nearest with 3 mantissa bits), so 2.4 % flushed gives
    0.024 + 0.976*0.02254 = 4.60 % (> 4.5 %, BF16) and 2.2 % flushed gives 4.40 % (E4M3)."""
    rng = np.random.default_rng(2024)
    n = 1 << 20
    mag = np.exp2(rng.uniform(-5.0, 8.0, size=n)).astype(np.float32)       # well inside E4M3 normals after scaling
    sign = rng.integers(0, 2, size=n).astype(np.float32) * 2 - 1
    base = mag * sign
    closed_form = 2.0 ** -5 / (2 * math.log(2))
    for frac, want_mask in ((0.024, 1), (0.022, 0)):
        x = base.copy()
        k = int(frac * n)
        x[:k] = 2.0 ** -30                                                 # flushes under a per-tensor scale
        x[-1] = 256.0                                                       # pins amax -> s = 1.75
        xb = W.f32_to_bf16_bits(x.reshape(1024, 1024))
        a = oracle.analyze_quantize(xb, "tensor", threshold=TH)
        metric = a.err_sum[0] / a.nnz[0]
        survivors = (a.err_sum[0] - k) / (a.nnz[0] - k)
        assert abs(survivors - closed_form) < 5e-4
        assert abs(metric - (frac + (1 - frac) * closed_form)) < 5e-4
        assert a.mask[0] == want_mask


# ---------------------------------------------------------------- exact-rational brute force

@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
def test_against_exact_rational_reference(oracle, crit):
    rng = np.random.default_rng(77)
    blocks = []
    blocks.append(W.activation(1, 128, 1)[0])
    blocks.append(W.gradient(1, 128, 2, tiny_half=True, tiny_frac=1.0)[0])
    blocks.append(W.weight(1, 128, 3, spike_frac=0.02)[0])
    blocks.append(rng.integers(0, 0x7F80, size=128).astype(np.uint16))               # any finite magnitude
    blocks.append((rng.integers(0, 0x7F80, size=128) | (rng.integers(0, 2, size=128) << 15)).astype(np.uint16))
    blocks.append(rng.integers(0x3F00, 0x4100, size=128).astype(np.uint16))          # narrow range
    blocks.append(rng.integers(0, 0x0100, size=128).astype(np.uint16))               # subnormals + tiny normals
    blocks.append(np.where(rng.random(128) < 0.5, 0, rng.integers(0x3000, 0x4800, size=128)).astype(np.uint16))
    xb = np.stack(blocks)
    a = oracle.analyze_quantize(xb, "sub1x128", crit=crit, threshold=TH)
    for p, blk in enumerate(blocks):
        r = R.analyze_block(blk, crit=crit, threshold=TH)
        assert a.amax[p] == r["amax"] and a.scale[p] == r["scale"] and a.nnz[p] == r["nnz"]
        assert list(a.fp8[p]) == r["codes"]
        assert a.err_sum[p] == pytest.approx(float(r["err_sum"]), rel=1e-13)
        if crit == "e4m3_vs_e5m2":
            assert a.err5_sum[p] == pytest.approx(float(r["err5_sum"]), rel=1e-13)
        assert a.mask[p] == (0 if r["fp8"] else 1)
    # the same blocks as one 8x128 tensor-granularity operand and as a padded 128x128 block
    t = oracle.analyze_quantize(xb, "tensor", crit=crit, threshold=TH)
    r = R.analyze_block(xb.reshape(-1), crit=crit, threshold=TH)
    assert t.amax[0] == r["amax"] and t.scale[0] == r["scale"] and t.nnz[0] == r["nnz"]
    assert list(t.fp8.reshape(-1)) == r["codes"]
    assert t.err_sum[0] == pytest.approx(float(r["err_sum"]), rel=1e-13)
    assert t.mask[0] == (0 if r["fp8"] else 1)


def test_block128_against_exact_rational_reference(oracle):
    xb = np.concatenate([W.activation(128, 128, 91), W.gradient(128, 128, 92, tiny_half=True)], axis=1)
    a = oracle.analyze_quantize(xb, "block128", threshold=TH)
    for p in range(2):
        blk = xb[:, p * 128:(p + 1) * 128]
        r = R.analyze_block(blk.reshape(-1), threshold=TH)
        assert a.amax[p] == r["amax"] and a.scale[p] == r["scale"] and a.nnz[p] == r["nnz"]
        assert list(a.fp8[:, p * 128:(p + 1) * 128].reshape(-1)) == r["codes"]
        assert a.err_sum[p] == pytest.approx(float(r["err_sum"]), rel=1e-13)
        assert a.mask[p] == (0 if r["fp8"] else 1)


def test_eq3_two_way_selection_handworked(oracle):
    """E5M2 has one mantissa bit less but 2^7 more range.  A narrow-range block (E4M3 more
    accurate) -> E4M3; a block whose small half flushes in E4M3 but survives in E5M2 -> BF16."""
    narrow = one_block(list(np.linspace(1.0, 1.9921875, 128, dtype=np.float32)))
    wide = one_block([1.0] * 64 + [2.0 ** -20] * 64)      # 448*2^-20 flushes in E4M3; 57344*2^-20 = 0.0547 is an E5M2 normal
    xb = np.vstack([narrow, wide])
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2")
    assert a.err_sum[0] < a.err5_sum[0] and a.mask[0] == 0
    assert a.err_sum[1] == 64.0 and a.err5_sum[1] == 0.0 and a.mask[1] == 1


# ---------------------------------------------------------------- statistics

def test_select_stats_handworked(oracle):
    err = np.array([0.0, 0.63, 0.64, 5.75, 5.76, 7.04, 7.05, 100.0, 0.0, np.inf], dtype=np.float32)
    nnz = np.array([128, 128, 128, 128, 128, 128, 128, 128, 0, 128], dtype=np.uint32)
    mask = np.array([0, 0, 0, 0, 1, 1, 1, 1, 0, 1], dtype=np.uint8)
    st = oracle.select_stats(err, nnz, mask, 10, 128, "sub1x128", threshold=TH, near_tol=1e-3)
    assert st["n_part"] == 10 and st["n_fp8_part"] == 5 and st["n_bf16_part"] == 5
    assert st["n_elem_fp8"] == 5 * 128 and st["n_elem_bf16"] == 5 * 128
    assert st["nnz_total"] == 9 * 128
    # metrics: 0, .00492, .005, .04492, .045, .055, .05508, .78, 0, inf
    assert st["hist"] == [3, 1, 0, 0, 0, 0, 0, 0, 1, 1, 0, 4]
    assert st["n_near_threshold"] == 1
    assert math.isinf(st["err_sum_total"]) and math.isinf(st["mean_err"])
    st2 = oracle.select_stats(err[:8], nnz[:8], mask[:8], 8, 128, "sub1x128", threshold=TH, near_tol=1e-3)
    assert st2["err_sum_total"] == pytest.approx(float(err[:8].astype(np.float64).sum()), rel=1e-15)
    assert st2["mean_err"] == pytest.approx(st2["err_sum_total"] / (8 * 128), rel=1e-15)
    assert sum(st2["hist"]) == 8


def test_workloads_are_deterministic_and_shaped():
    a = W.activation(256, 256, W.seed_for(2))
    b = W.activation(256, 256, W.seed_for(2))
    assert a.dtype == np.uint16 and a.shape == (256, 256) and np.array_equal(a, b)
    g = W.gradient(256, 256, W.seed_for(4))
    zf = np.mean((g & 0x7FFF) == 0)
    assert 0.03 < zf < 0.07
    sweep = W.cfg5(row_div=32)
    assert [s[0] for s in sweep] == [r[0] for r in W.LAYER_SWEEP] and len(sweep) == 12


def test_threshold_compare_is_strict(oracle):
    """Eq. (2) uses "<": three exact values and one flushed one give a metric of exactly 1/4;
    a threshold of exactly 1/4 must reject E4M3, the next float above must accept it."""
    xb = one_block([448.0, 224.0, 1.0, 2.0 ** -12])
    a = oracle.analyze_quantize(xb, "sub1x128", threshold=0.25)
    assert a.err_sum[0] == 1.0 and a.nnz[0] == 4 and a.mask[0] == 1
    up = float(np.nextafter(np.float32(0.25), np.float32(1)))
    assert oracle.analyze_quantize(xb, "sub1x128", threshold=up).mask[0] == 0
    assert oracle.analyze_quantize(xb, "tensor", threshold=0.25).mask[0] == 1
    assert oracle.analyze_quantize(xb, "sub1x128", scope="tensor", threshold=up).mask[0] == 0


@pytest.mark.parametrize("scaling", ["fp32_amax", "gam", "e8m0"])
@pytest.mark.parametrize("gran", ["tensor", "sub1x128", "channel_col"])
def test_values_below_two_to_minus_20_of_amax_flush_and_force_bf16(oracle, gran, scaling):
    """The bound the kernels' early BF16 proof rests on: a non-zero element below 2^-20 of (any lower bound of) its
    block's amax scales to less than half the smallest E4M3 subnormal under every scaling algorithm, so its code is
    zero and it adds exactly 1 to Eq. 2's sum; more than th * N such elements therefore force BF16."""
    rng = np.random.default_rng(11)
    rows, cols = 128, 256
    x = np.exp2(rng.uniform(-2.0, 2.0, size=(rows, cols))).astype(np.float32) * rng.choice([-1.0, 1.0], size=(rows, cols)).astype(np.float32)
    xb = W.f32_to_bf16_bits(x)
    tiny = rng.random((rows, cols)) < 0.06                         # 6 % > 1.01 * 4.5 %
    mag = xb & 0x7FFF
    # just below 2^-20 of the SMALLEST amax any block can have here (2^-2): every such element is below the bound of its block
    below = ((mag.astype(np.int32) & 0x7F) | ((125 - 20 - 1) << 7)).astype(np.uint16)      # exponent 2^-23 .. < 2^-22
    xb = np.where(tiny, (xb & 0x8000) | below, xb).astype(np.uint16)
    a = oracle.analyze_quantize(xb, gran, "partition", "mean_rel_err", 0.045, scaling=scaling)
    codes = a.fp8[tiny]
    assert np.all((codes & 0x7F) == 0), "an element below 2^-20 of the amax did not flush"
    # a block whose count of such elements exceeds th * (block size) is BF16 whatever its other elements are
    counts, size = {"tensor": (np.array([tiny.sum()]), rows * cols),
                    "sub1x128": (tiny.reshape(rows, cols // 128, 128).sum(-1).ravel(), 128),
                    "channel_col": (tiny.sum(0), rows)}[gran]
    assert a.err_sum.sum() >= int(tiny.sum())
    forced = counts > 0.045 * size
    assert forced.any() and np.all(a.mask[forced] == 1)
