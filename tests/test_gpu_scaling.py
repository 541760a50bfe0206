"""GPU parity of GAM and E8M0-only scaling (Algorithm 1) against the CPU oracle, through the C ABI:
scales, E8M0 bytes, group mantissa, FP8 codes, nnz and BF16 payload bit-exact; error sums to 1e-5."""
import numpy as np
import pytest
import torch

from paper_2512_22804_amd import binding as B
from paper_2512_22804_amd import workloads as W
import parity

pytestmark = pytest.mark.gpu

SCALINGS = ["gam", "e8m0"]


def spread(xb, seed):
    """Give every row its own magnitude (2^-12 .. 2^4) so that block exponents differ within one operand."""
    rng = np.random.default_rng(seed)
    f = W.bf16_bits_to_f32(xb) * np.ldexp(1.0, rng.integers(-12, 5, (xb.shape[0], 1))).astype(np.float32)
    br, bc = (xb.shape[0] + 127) // 128, (xb.shape[1] + 127) // 128          # and every 128x128 block on top of that
    blk = np.ldexp(1.0, rng.integers(-6, 7, (br, bc))).astype(np.float32)
    f = f * np.repeat(np.repeat(blk, 128, 0), 128, 1)[:xb.shape[0], :xb.shape[1]]
    return W.f32_to_bf16_bits(f.astype(np.float32))


@pytest.mark.parametrize("scaling", SCALINGS)
@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
@pytest.mark.parametrize("gran,shape", [("sub1x128", (321, 1024)), ("sub1x128", (64, 4096)), ("block128", (384, 640)),
                                        ("tensor", (300, 520)), ("sub1x128", (3, 128))])
def test_scaling_parity_partition_scope(scaling, crit, gran, shape):
    cols_gen = (shape[1] + 127) // 128 * 128
    xb = np.ascontiguousarray(spread(W.gradient(shape[0], cols_gen, 31, tiny_half=True), 5)[:, :shape[1]])
    r = parity.compare(xb, gran, "partition", crit, 0.045, label="scaling", scaling=scaling)
    if gran == "sub1x128" and scaling == "gam" and shape[0] > 3:
        e = r["gpu"].scale_e8m0.cpu().numpy()
        assert len(np.unique(e)) > 3                      # the operand really has blocks in several binades


@pytest.mark.parametrize("scaling", SCALINGS)
@pytest.mark.parametrize("gran", ["sub1x128", "block128"])
def test_scaling_parity_tensor_scope(scaling, gran):
    # the tensor-level recipe of Section 3.1: global mantissa, per-block E8M0 exponents, one decision
    for idx, xb in enumerate([W.activation(256, 1024, 3), spread(W.gradient(256, 1024, 4), 9)]):
        parity.compare(xb, gran, "tensor", "mean_rel_err", 0.045, label=f"tensor-scope-{idx}", scaling=scaling)


@pytest.mark.parametrize("scaling", SCALINGS)
@pytest.mark.parametrize("gran,ld", [("sub1x128", 640), ("block128", 640), ("tensor", 520)])
def test_scaling_parity_padded_leading_dimension(scaling, gran, ld):
    cols = 512
    xb = spread(W.weight(256, ld, 8), 2)
    parity.compare(xb, gran, "partition", "mean_rel_err", 0.045, cols=cols, label="padded", scaling=scaling)


@pytest.mark.parametrize("scaling", SCALINGS)
def test_scaling_every_finite_amax(scaling):
    # one 1x128 block per finite BF16 magnitude (fast path, careful path, subnormal amax, scale overflow),
    # under a group amax at the top of the range
    mags = np.arange(0, 0x7F80, dtype=np.uint16)
    rng = np.random.default_rng(17)
    xb = np.zeros((mags.size, 128), np.uint16)
    for k in range(0, 128, 8):
        frac = rng.uniform(0, 1, mags.size)
        v = (W.bf16_bits_to_f32(mags) * frac).astype(np.float32)
        xb[:, k] = W.f32_to_bf16_bits(v) | (rng.integers(0, 2, mags.size).astype(np.uint16) << 15)
    xb[:, 5] = mags
    xb[:, 9] = 1          # smallest subnormal: the element that can round to a binary32 zero under a halved scale
    parity.compare(xb, "sub1x128", "partition", "mean_rel_err", 0.045, label="all-amax", scaling=scaling)
    parity.compare(xb[:0x4000], "sub1x128", "partition", "e4m3_vs_e5m2", 0.045, label="all-amax-low", scaling=scaling)


def test_scaling_nonfinite_and_zero_blocks():
    xb = spread(W.gradient(64, 512, 12), 3)
    xb[3, 130] = 0x7F80; xb[7, 5] = 0xFFC0; xb[9, :128] = 0; xb[11, 128:256] = 0x8000
    for scaling in SCALINGS:
        for gran in ("sub1x128", "tensor"):
            parity.compare(xb, gran, "partition", "mean_rel_err", 0.045, label="nonfinite", scaling=scaling)
    z = np.zeros((4, 256), np.uint16)
    for scaling in SCALINGS:
        parity.compare(z, "sub1x128", "partition", "mean_rel_err", 0.045, label="zeros", scaling=scaling)


def test_scaling_batch_mixes_modes():
    # one batch call with all three scaling algorithms and granularities == single calls
    dev = torch.device("cuda")
    cases = []
    for i, (gran, scaling) in enumerate([("sub1x128", "gam"), ("block128", "gam"), ("tensor", "gam"), ("sub1x128", "e8m0"),
                                         ("block128", "fp32_amax"), ("tensor", "e8m0"), ("sub1x128", "fp32_amax")]):
        xb = spread(W.gradient(256, 512, 40 + i, tiny_half=True), i)
        params = B.make_params(256, 512, gran, "partition", "mean_rel_err", 0.045, scaling=scaling)
        x = parity.to_dev(xb)
        cases.append((xb, gran, scaling, params, x, B.alloc_outputs(params, dev, bf16_fill=parity.FILL),
                      B.alloc_outputs(params, dev, bf16_fill=parity.FILL)))
    items = B.make_batch([(c[3], c[4], c[5], None) for c in cases])
    ws = torch.empty(max(B.mor_batch_workspace_bytes(items), 16), dtype=torch.uint8, device=dev)
    B.mor_analyze_quantize_batch(items, 1e-5, ws, None)
    for c in cases:
        B.mor_analyze_quantize(c[3], c[4], c[6])
    torch.cuda.synchronize()
    for xb, gran, scaling, params, x, ob, os_ in cases:
        for name in ("fp8", "bf16", "scale", "amax", "err_sum", "nnz", "mask", "scale_e8m0", "group_mantissa"):
            tb, ts = getattr(ob, name), getattr(os_, name)
            if tb is None:
                assert ts is None
                continue
            assert torch.equal(tb, ts), (gran, scaling, name)


@pytest.mark.parametrize("scaling", SCALINGS)
@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor"])
def test_dequantize_from_stored_scale_form(oracle, scaling, gran):
    xb = spread(W.gradient(256, 512, 61, tiny_half=True), 4)
    params, g = parity.run_gpu(xb, gran, scaling=scaling)
    a = oracle.analyze_quantize(xb, gran, scaling=scaling, bf16_fill=parity.FILL)
    want = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, gran)
    y = torch.full((256, 512), 0x1111, dtype=torch.int16, device="cuda")
    B.mor_dequantize_e8m0(params, g.fp8, g.scale_e8m0, g.group_mantissa, g.mask, g.bf16, y)
    y2 = torch.full((256, 512), 0x1111, dtype=torch.int16, device="cuda")
    B.mor_dequantize(params, g.fp8, g.scale, g.mask, g.bf16, y2)
    torch.cuda.synchronize()
    assert np.array_equal(parity.u16(y), want) and np.array_equal(parity.u16(y2), want)
    with pytest.raises(B.MorError):
        B.mor_dequantize_e8m0(params, g.fp8, None, g.group_mantissa, g.mask, g.bf16, y)
