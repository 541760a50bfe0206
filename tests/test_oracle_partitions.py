"""Pins for the oracle's further partitions (per-channel rows / columns, 128 x 1 column sub-channels,
64 x 64 blocks), ragged edges, the fake-quantization output and the running histogram.  The new
partitions are tied to the already pinned 1 x 128 / 128 x 128 / per-tensor ones through
transposition, block extraction with numpy reshapes, zero padding and planted maxima; no expected
value comes from the code under test."""
import numpy as np
import pytest

import refmodel as R
from paper_2512_22804_amd import workloads as W

TH = 0.045


def operand(seed, rows, cols):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols)).astype(np.float32) * np.exp2(rng.integers(-6, 6, size=(rows, 1))).astype(np.float32)
    x *= np.exp2(rng.integers(-3, 3, size=(1, cols))).astype(np.float32)
    x[rng.random((rows, cols)) < 0.04] = 0.0
    wide = rng.random((rows, cols)) < 0.03
    x[wide] *= np.float32(2.0 ** -24)
    return W.f32_to_bf16_bits(x)


SHAPES = {"channel_row": lambda r, c: (1, c), "channel_col": lambda r, c: (r, 1), "sub128x1": lambda r, c: (128, 1),
          "block64": lambda r, c: (64, 64), "sub1x128": lambda r, c: (1, 128), "block128": lambda r, c: (128, 128),
          "tensor": lambda r, c: (r, c)}


def test_block_counts(oracle):
    assert oracle.num_partitions("channel_row", 8192, 4096) == 8192
    assert oracle.num_partitions("channel_col", 8192, 4096) == 4096
    assert oracle.num_partitions("sub128x1", 8192, 4096) == 64 * 4096
    assert oracle.num_partitions("block64", 8192, 4096) == 128 * 64
    assert oracle.num_partitions("block64", 100, 64) == -1 and oracle.num_partitions("sub128x1", 100, 64) == -1
    assert oracle.num_partitions("block64", 100, 70, ragged=True) == 2 * 2
    assert oracle.num_partitions("sub1x128", 3, 130, ragged=True) == 3 * 2
    assert oracle.num_partitions("block128", 129, 128, ragged=True) == 2
    assert oracle.num_partitions("sub128x1", 130, 5, ragged=True) == 2 * 5


@pytest.mark.parametrize("gran", ["channel_row", "channel_col", "sub128x1", "block64"])
def test_planted_maxima_land_in_their_blocks(oracle, gran):
    """One distinct power of two per intended block, planted at a random position inside it over a
    background of small values: amax[p] must be exactly that power, in row-major block order."""
    rows, cols = 256, 192
    pr, pc = SHAPES[gran](rows, cols)
    rng = np.random.default_rng(4)
    x = (rng.random((rows, cols)).astype(np.float32) + 1) * np.float32(2.0 ** -20)
    want = []
    p = 0
    for br in range(rows // pr):
        for bc in range(cols // pc):
            v = np.float32(2.0 ** (p % 40 - 10))
            x[br * pr + rng.integers(pr), bc * pc + rng.integers(pc)] = -v if p % 3 == 0 else v
            want.append(v)
            p += 1
    a = oracle.analyze_quantize(W.f32_to_bf16_bits(x), gran, threshold=TH)
    assert np.array_equal(a.amax, np.array(want, dtype=np.float32))
    assert np.all(a.nnz == pr * pc)


@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
@pytest.mark.parametrize("scaling", ["fp32_amax", "gam"])
def test_columns_are_rows_of_the_transpose(oracle, crit, scaling):
    """Per-channel columns of X are per-channel rows of X^T; 128 x 1 sub-channels of X are the 1 x 128
    sub-channels of X^T (the already pinned partition).  Payloads transpose, block lists re-index."""
    xb = operand(1, 256, 384)
    xt = np.ascontiguousarray(xb.T)
    col = oracle.analyze_quantize(xb, "channel_col", crit=crit, scaling=scaling, threshold=TH, bf16_fill=7)
    row = oracle.analyze_quantize(xt, "channel_row", crit=crit, scaling=scaling, threshold=TH, bf16_fill=7)
    for f in ("scale", "amax", "err_sum", "err5_sum", "nnz", "mask"):
        assert np.array_equal(getattr(col, f), getattr(row, f)), f
    assert np.array_equal(col.fp8, row.fp8.T) and np.array_equal(col.bf16, row.bf16.T)
    sub_c = oracle.analyze_quantize(xb, "sub128x1", crit=crit, scaling=scaling, threshold=TH, bf16_fill=7)
    sub_r = oracle.analyze_quantize(xt, "sub1x128", crit=crit, scaling=scaling, threshold=TH, bf16_fill=7)
    # block (i, c) of X, i = r // 128, is block (c, i) of X^T
    for f in ("scale", "amax", "err_sum", "err5_sum", "nnz", "mask"):
        assert np.array_equal(getattr(sub_c, f).reshape(2, 384), getattr(sub_r, f).reshape(384, 2).T), f
    assert np.array_equal(sub_c.fp8, sub_r.fp8.T) and np.array_equal(sub_c.bf16, sub_r.bf16.T)
    if scaling == "gam":
        assert sub_c.group_mantissa == sub_r.group_mantissa
        assert np.array_equal(sub_c.e8m0.reshape(2, 384), sub_r.e8m0.reshape(384, 2).T)


def test_channel_row_is_one_sub_channel_when_cols_is_128(oracle):
    xb = operand(2, 64, 128)
    a = oracle.analyze_quantize(xb, "channel_row", threshold=TH)
    b = oracle.analyze_quantize(xb, "sub1x128", threshold=TH)
    for f in ("scale", "amax", "err_sum", "nnz", "mask", "fp8"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f


@pytest.mark.parametrize("gran,pr,pc", [("block64", 64, 64), ("channel_row", 1, 256), ("sub128x1", 128, 1)])
def test_blocks_against_exact_rational_reference(oracle, gran, pr, pc):
    """Blocks cut out with numpy reshapes, each analysed by the exact-rational model."""
    rows, cols = 128, 256
    xb = operand(3, rows, cols)
    a = oracle.analyze_quantize(xb, gran, crit="e4m3_vs_e5m2")
    blocks = xb.reshape(rows // pr, pr, cols // pc, pc).transpose(0, 2, 1, 3).reshape(-1, pr * pc)
    codes = a.fp8.reshape(rows // pr, pr, cols // pc, pc).transpose(0, 2, 1, 3).reshape(-1, pr * pc)
    pick = np.random.default_rng(0).choice(len(blocks), size=min(max(1, 2048 // (pr * pc)), len(blocks)), replace=False)
    for p in pick:
        ref = R.analyze_block(blocks[p], crit="e4m3_vs_e5m2")
        assert ref["amax"] == float(a.amax[p]) and ref["nnz"] == int(a.nnz[p]) and ref["scale"] == float(a.scale[p])
        assert ref["codes"] == codes[p].tolist()
        assert float(ref["err_sum"]) == pytest.approx(a.err_sum[p], rel=1e-12)
        assert float(ref["err5_sum"]) == pytest.approx(a.err5_sum[p], rel=1e-12)
        assert (0 if ref["fp8"] else 1) == a.mask[p]


@pytest.mark.parametrize("gran", ["sub1x128", "block128", "block64", "sub128x1"])
@pytest.mark.parametrize("rows,cols", [(130, 200), (64, 136), (257, 128), (5, 8)])
def test_ragged_edges_equal_zero_padding(oracle, gran, rows, cols):
    """Zeros enter neither amax, nor the non-zero count, nor the error sums, so a tensor with ragged
    edges must give, block by block, what the zero-padded tensor (whole blocks only) gives."""
    pr, pc = SHAPES[gran](rows, cols)
    R_, C_ = -(-rows // pr) * pr, -(-cols // pc) * pc
    xb = operand(rows * 1000 + cols, rows, cols)
    pad = np.zeros((R_, C_), dtype=np.uint16)
    pad[:rows, :cols] = xb
    for crit in ("mean_rel_err", "e4m3_vs_e5m2"):
        a = oracle.analyze_quantize(xb, gran, crit=crit, threshold=TH, ragged=True, bf16_fill=9, want_fake=True)
        b = oracle.analyze_quantize(pad, gran, crit=crit, threshold=TH, bf16_fill=9, want_fake=True)
        for f in ("scale", "amax", "err_sum", "err5_sum", "nnz", "mask", "amin"):
            assert np.array_equal(getattr(a, f), getattr(b, f)), f
        assert np.array_equal(a.fp8, b.fp8[:rows, :cols]) and np.array_equal(a.bf16, b.bf16[:rows, :cols])
        assert np.array_equal(a.fake, b.fake[:rows, :cols])
    with pytest.raises(ValueError):
        if rows % pr or cols % pc:
            oracle.analyze_quantize(xb, gran, threshold=TH)          # whole blocks are required unless asked
        else:
            raise ValueError


def test_ragged_statistics_count_real_elements(oracle):
    xb = operand(8, 130, 200)
    a = oracle.analyze_quantize(xb, "block64", threshold=0.02, ragged=True)
    st = oracle.select_stats(a.err_sum.astype(np.float32), a.nnz, a.mask, 130, 200, "block64", threshold=0.02, ragged=True)
    assert st["n_part"] == 3 * 4 and st["n_elem_fp8"] + st["n_elem_bf16"] == 130 * 200
    sizes = np.array([[min(64, 130 - r) * min(64, 200 - c) for c in range(0, 200, 64)] for r in range(0, 130, 64)]).reshape(-1)
    assert st["n_elem_bf16"] == int(sizes[a.mask == 1].sum())


# ---------------------------------------------------------------- fake quantization (Figure 4)

@pytest.mark.parametrize("gran", ["tensor", "sub1x128", "block128", "channel_row", "channel_col", "sub128x1", "block64"])
def test_fake_quantize_is_dequantize_of_quantize(oracle, gran):
    xb = operand(12, 128, 256)
    a = oracle.analyze_quantize(xb, gran, threshold=0.03, want_fake=True, bf16_fill=3)
    want = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, gran)
    assert np.array_equal(a.fake, want)
    pr, pc = SHAPES[gran](128, 256)
    m = np.repeat(np.repeat(a.mask.reshape(128 // pr, 256 // pc), pr, 0), pc, 1)
    assert np.array_equal(a.fake[m == 1], xb[m == 1])                 # BF16 blocks pass through
    # information loss of a 3-bit mantissa: |fake - x| <= (2^-4 + 2^-9) |x| for values in E4M3's normal range
    x = W.bf16_bits_to_f32(xb).astype(np.float64); f = W.bf16_bits_to_f32(a.fake).astype(np.float64)
    s = np.repeat(np.repeat(a.scale.reshape(128 // pr, 256 // pc), pr, 0), pc, 1).astype(np.float64)
    normal = (m == 0) & (np.abs(x) * s >= 2.0 ** -6)
    assert np.all(np.abs(f - x)[normal] <= (2.0 ** -4 + 2.0 ** -9) * np.abs(x)[normal])
    if normal.any():                                                  # (coarse blocks of this operand all fall back at 3 %)
        assert (np.abs(f - x)[normal] > 0).mean() > 0.5               # and it really is lossy


def test_fake_quantize_of_grid_values_is_the_identity(oracle):
    grid = np.array(sorted(float(v) for v in R.fp8_values(4, 3).values() if v >= 2.0 ** -6), dtype=np.float32)
    rng = np.random.default_rng(5)
    y = grid[rng.integers(0, len(grid), size=(64, 256))] * (rng.integers(0, 2, size=(64, 256)) * 2 - 1).astype(np.float32)
    y[:, ::64] = 448.0                      # every row, 64 x 64 block ...
    y[0, :] = 448.0                         # ... and every column holds the amax
    xb = W.f32_to_bf16_bits(y * np.float32(2.0 ** -5))
    for gran in ("tensor", "sub1x128", "channel_row", "channel_col", "block64"):
        a = oracle.analyze_quantize(xb, gran, want_fake=True)
        assert np.array_equal(a.fake, xb) and np.all(a.mask == 0) and np.all(a.err_sum == 0)


def test_fake_quantize_three_way_decodes_e5m2_blocks(oracle):
    x = np.zeros((2, 128), dtype=np.float32)
    x[0, 0] = 1.0; x[0, 1:] = 2.0 ** -20          # E5M2 block, exactly representable there
    x[1, :] = 1.0                                 # both formats exact: Eq. (3) ties, Eq. (4) holds -> E5M2 as well
    xb = W.f32_to_bf16_bits(x)
    a = oracle.analyze_quantize(xb, "sub1x128", crit="e4m3_vs_e5m2", formats="e4m3|e5m2|bf16", want_fake=True)
    assert a.mask.tolist() == [2, 2] and np.array_equal(a.fake, xb)


# ---------------------------------------------------------------- running histogram (Section 4.1.3)

def test_histogram_counts_one_per_step_and_resets(oracle):
    h = np.full(12, 99, dtype=np.uint32)
    metrics = [0.0, 0.0049, 0.005, 0.0225, 0.0449, 0.045, 0.0549, 0.055, 0.3, float("inf")]
    for step, m in enumerate(metrics):
        oracle.histogram_update(h, m, step, 6000)                      # step 0 clears the stale contents
    assert h.tolist() == [2, 1, 0, 0, 1, 0, 0, 0, 1, 1, 1, 3] and h.sum() == len(metrics)
    for step in range(10, 14):
        oracle.histogram_update(h, 0.012, step, 12)                    # step 12 is a reset step
    assert h.tolist() == [0, 0, 2, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    oracle.histogram_update(h, 0.012, 5, 0)                            # interval 0: never reset
    assert h[2] == 3
