"""Pins for the three-way recipe [E4M3, E5M2, BF16] of Section 3.2 in the oracle: the paper's range
constants, hand-worked blocks on both sides of each decision, the relation to the two-way recipe,
PyTorch's float8_e5m2 cast for the emitted payload, and an exact-rational brute force
(tests/refmodel.py).  No expected value comes from the oracle itself."""
import os

import numpy as np
import pytest
import torch

import refmodel as R
from paper_2512_22804_amd import workloads as W

THREE = "e4m3|e5m2|bf16"


def bf16(v):
    a = np.asarray(v, dtype=np.float32)
    b = W.f32_to_bf16_bits(a)
    assert np.array_equal(W.bf16_bits_to_f32(b), a), "test value is not a BF16 number"
    return b


def block(values):
    x = np.zeros((1, 128), dtype=np.float32)
    x[0, :len(values)] = values
    return bf16(x)


def golden():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                out[line[0]] = float(line[1])
    return out


def test_e4m3_flushes_e5m2_holds_selects_e5m2(oracle):
    """amax 1 and 127 elements 2^-20: 448 * 2^-20 < 2^-10 flushes in E4M3 (error sum 127), while
    57344 * 2^-20 = 1.75 * 2^-5 is an E5M2 value (error sum 0).  Eq. (3) rejects E4M3; the range
    2^20 is below 57344 / 2^-14, so Eq. (4) accepts E5M2.  Codes: 57344 -> 0x7B, 1.75 * 2^-5 ->
    exponent field 10, fraction 11b -> 0x2B."""
    xb = block([1.0] + [2.0 ** -20] * 127)
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    assert a.err_sum[0] == 127.0 and a.err5_sum[0] == 0.0
    assert a.mask[0] == 2 and a.scale[0] == 57344.0 and a.amin[0] == np.float32(2.0 ** -20)
    assert a.fp8[0, 0] == 0x7B and np.all(a.fp8[0, 1:] == 0x2B)
    # the two-way recipe with the same metric leaves this block in BF16
    b = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2")
    assert b.mask[0] == 1 and b.scale[0] == 448.0 and b.fp8[0, 0] == 0x7E
    # de-quantizing the E5M2 payload gives the input back exactly
    back = oracle.dequantize(a.fp8, a.scale, a.mask, None, "sub1x128")
    assert np.array_equal(back, xb)


def test_range_beyond_e5m2_normal_range_falls_back_to_bf16(oracle):
    """amax 1 and 2^-30: in E5M2 57344 * 2^-30 = 3.5 * 2^-16 sits midway between the subnormals
    3 * 2^-16 and 2^-14 and rounds to the even code (2^-14): relative error 1/7 each, still far
    better than E4M3's 127 flushed values -- but the range 2^30 is not below 57344 * 2^14."""
    xb = block([1.0] + [2.0 ** -30] * 127)
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    assert a.err_sum[0] == 127.0 and a.err5_sum[0] == pytest.approx(127.0 / 7.0, rel=1e-12)
    assert a.mask[0] == 1 and a.scale[0] == 448.0
    assert np.array_equal(a.bf16[0], xb[0])


def test_range_bound_is_strict_and_uses_the_papers_constants(oracle):
    g = golden()
    bound = g["e5m2_max"] / g["e5m2_min_normal"]
    assert bound == 57344.0 * 2.0 ** 14 == 1.75 * 2.0 ** 29
    rows = [
        [1.75] + [2.0 ** -29] * 100,                       # ratio == bound: not below -> BF16
        [1.75] + [2.0 ** -29 * (1 + 2.0 ** -7)] * 100,     # one BF16 step inside -> E5M2
        [1.75, 2.0 ** -29 * (1 + 2.0 ** -7)] + [2.0 ** -25] * 100 + [2.0 ** -29],   # the minimum decides
    ]
    xb = np.concatenate([block(r) for r in rows])
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    assert a.mask.tolist() == [1, 2, 1]
    ratio = a.amax.astype(np.float64) / a.amin.astype(np.float64)
    assert (ratio[0] == bound) and (ratio[1] < bound) and (ratio[2] == bound)


def test_zeros_do_not_enter_the_minimum_and_empty_blocks_pass(oracle):
    xb = np.concatenate([block([1.0] + [2.0 ** -20] * 50),      # 77 zeros in the block
                         block([]),                              # no non-zero element at all
                         np.array([[0x8000] * 128], dtype=np.uint16)])
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    assert a.mask.tolist() == [2, 2, 2]           # Eq. (3) ties at 0 < 0 for empty blocks, Eq. (4) has no range to cover
    assert a.amin[0] == np.float32(2.0 ** -20) and a.amin[1] == 0 and a.nnz.tolist() == [51, 0, 0]
    assert a.scale[1] == 1.0 and not a.fp8[1].any() and np.all(a.fp8[2] == 0x80)


def test_nonfinite_blocks_stay_bf16(oracle):
    x = np.zeros((3, 128), dtype=np.uint16)
    x[0, :] = 0x3F80; x[0, 3] = 0x7F80          # +Inf
    x[1, :] = 0x3F80; x[1, 9] = 0xFFC0          # NaN
    x[2, :] = 0x7F80                            # all Inf: the ratio Inf/Inf is no number
    a = oracle.analyze_quantize(x, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    assert a.mask.tolist() == [1, 1, 1]


def test_eq2_as_first_metric(oracle):
    """The framework lets M_1 be the mean-relative-error test: flushed block -> E5M2 if the range fits."""
    xb = np.concatenate([block([1.0] + [2.0 ** -20] * 127), block([1.0] + [2.0 ** -30] * 127), block([1.0, 0.5, 0.25])])
    a = oracle.analyze_quantize(xb, "sub1x128", crit="mean_rel_err", threshold=0.045, formats=THREE)
    assert a.mask.tolist() == [2, 1, 0]
    assert a.scale.tolist() == [57344.0, 448.0, 448.0]


def mixed_operand(seed, rows=64, cols=256):
    """Blocks of three kinds: well-behaved, wide (E4M3 flushes, E5M2 holds), very wide (nothing holds)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    kind = rng.integers(0, 3, size=(rows, cols // 128))
    for r in range(rows):
        for b in range(cols // 128):
            sl = x[r, b * 128:(b + 1) * 128]
            if kind[r, b] == 1:
                sl[16:] *= np.float32(2.0 ** -22)
            elif kind[r, b] == 2:
                sl[16:] *= np.exp2(rng.integers(-40, -20, size=112)).astype(np.float32)
            sl[rng.random(128) < 0.05] = 0.0
    return W.f32_to_bf16_bits(x), kind


@pytest.mark.parametrize("gran", ["sub1x128", "block128"])
@pytest.mark.parametrize("crit", ["e4m3_vs_e5m2", "mean_rel_err"])
def test_relation_to_two_way(oracle, gran, crit):
    """Same M_1: the E4M3 set is identical; BF16 blocks of the three-way recipe are BF16 in the two-way one;
    every quantity that does not depend on the choice is unchanged; E4M3 payloads are identical."""
    xb, _ = mixed_operand(3, rows=128, cols=512)
    a3 = oracle.analyze_quantize(xb, gran, crit=crit, formats=THREE)
    a2 = oracle.analyze_quantize(xb, gran, crit=crit)
    assert np.array_equal(a3.mask == 0, a2.mask == 0)
    assert np.all(a2.mask[a3.mask == 1] == 1)
    if gran == "sub1x128":
        assert {0, 1, 2} <= set(a3.mask.tolist())
    for f in ("amax", "err_sum", "err5_sum", "nnz"):
        assert np.array_equal(getattr(a3, f), getattr(a2, f))
    keep = a3.mask != 2
    assert np.array_equal(a3.scale[keep], a2.scale[keep])
    pr, pc = (1, 128) if gran == "sub1x128" else (128, 128)
    m = np.repeat(np.repeat(a3.mask.reshape(128 // pr, 512 // pc), pr, 0), pc, 1)
    assert np.array_equal(a3.fp8[m != 2], a2.fp8[m != 2])
    # Eq. (4) on the selected blocks, from numpy: amax < bound * amin
    sel = a3.mask == 2
    nz = a3.nnz[sel] > 0
    assert np.all(a3.amax[sel][nz].astype(np.float64) < 57344.0 * 16384.0 * a3.amin[sel][nz].astype(np.float64))
    rej = (a3.mask == 1) & (a3.nnz > 0) & np.isfinite(a3.amax)
    assert np.all(a3.amax[rej].astype(np.float64) >= 57344.0 * 16384.0 * a3.amin[rej].astype(np.float64))


def test_e5m2_payload_matches_torch_cast(oracle):
    """The payload of an E5M2 block is the library's float8_e5m2 cast of fl32(x * scale)."""
    xb, _ = mixed_operand(5)
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    sel = np.flatnonzero(a.mask == 2)
    assert len(sel) > 10
    x = W.bf16_bits_to_f32(xb).reshape(-1, 128)
    y = (x[sel] * a.scale[sel, None]).astype(np.float32)
    want = torch.from_numpy(y).to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(a.fp8.reshape(-1, 128)[sel], want)
    # ... and the scale is the E5M2 scale of the block
    assert np.array_equal(a.scale[sel], (np.float32(57344.0) / a.amax[sel]).astype(np.float32))


@pytest.mark.parametrize("crit", ["e4m3_vs_e5m2", "mean_rel_err"])
@pytest.mark.parametrize("scaling", ["fp32_amax", "gam", "e8m0"])
def test_against_exact_rational_reference(oracle, crit, scaling):
    xb, _ = mixed_operand(11, rows=24, cols=256)
    xb[3, :128] = 0                                        # an empty block
    xb[5, 7] = 0x7F80                                      # a non-finite block
    a = oracle.analyze_quantize(xb, "sub1x128", crit=crit, formats=THREE, scaling=scaling)
    g_amax = float(W.bf16_bits_to_f32(np.array([(xb & 0x7FFF).max()], dtype=np.uint16))[0])
    names = {"e4m3": 0, "bf16": 1, "e5m2": 2}
    blocks = xb.reshape(-1, 128)
    for p in range(blocks.shape[0]):
        if (blocks[p] & 0x7FFF).max() >= 0x7F80:
            assert a.mask[p] == 1
            continue
        ref = R.analyze_block(blocks[p], crit=crit, scaling=scaling, g_amax=g_amax, three_way=True)
        assert names[ref["choice"]] == a.mask[p], p
        assert ref["scale"] == float(a.scale[p]), p
        assert ref["codes"] == a.fp8.reshape(-1, 128)[p].tolist(), p
        if scaling != "fp32_amax":
            assert a.e8m0[p] == (np.float32(ref["scale"]).view(np.uint32) >> 23), p
    if scaling == "gam":
        s4 = R.scale_of(g_amax, 448.0); s5 = R.scale_of(g_amax, 57344.0)
        assert a.group_mantissa == int(s4.view(np.uint32) & 0x7FFFFF) and a.group_mantissa5 == int(s5.view(np.uint32) & 0x7FFFFF)


def test_three_way_needs_block_scope(oracle):
    xb, _ = mixed_operand(1)
    with pytest.raises(ValueError):
        oracle.analyze_quantize(xb, "sub1x128", scope="tensor", crit="e4m3_vs_e5m2", formats=THREE)


def test_stats_count_e5m2_blocks(oracle):
    xb, _ = mixed_operand(9)
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats=THREE)
    st = oracle.select_stats(a.err_sum.astype(np.float32), a.nnz, a.mask, 64, 256, "sub1x128")
    counts = np.bincount(a.mask, minlength=3)
    assert (st["n_fp8_part"], st["n_bf16_part"], st["n_e5m2_part"]) == tuple(int(c) for c in counts)
    assert st["n_elem_e5m2"] == 128 * counts[2] and st["n_elem_fp8"] + st["n_elem_bf16"] + st["n_elem_e5m2"] == xb.size
