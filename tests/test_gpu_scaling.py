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
@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor", "channel_row", "channel_col", "sub128x1", "block64"])
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


def _with_tiny(rows, cols, frac, seed, tiny_exp=-40):
    rng = np.random.default_rng(seed)
    x = np.exp2(rng.uniform(-3.0, 3.0, size=(rows, cols))).astype(np.float32) * (rng.integers(0, 2, size=(rows, cols)) * 2 - 1)
    x[rng.random((rows, cols)) < frac] = np.float32(2.0 ** tiny_exp)
    return x


@pytest.mark.parametrize("frac", [0.0, 0.04, 0.2])
@pytest.mark.parametrize("pad", [0, 64])
@pytest.mark.parametrize("gran,shape", [("block128", (640, 1152)), ("block64", (640, 1152)), ("block64", (192, 320)),
                                        ("channel_row", (70, 1152)), ("channel_row", (9, 9000)), ("channel_row", (5, 20000)),
                                        ("sub1x128", (640, 1152)), ("sub1x128", (128, 128)), ("sub1x128", (200, 384)),
                                        ("sub128x1", (640, 1152)), ("sub128x1", (256, 384))])
def test_gam_tensor_level_decision_proven_by_the_pre_pass(frac, pad, gran, shape):
    """Tensor-level decision over GAM-scaled 128x128 blocks or per-channel rows (the recipe of Section 3.1): with enough
    certain flushes the amax pre-pass proves the BF16 decision and the block kernel writes the fallback itself; with 4 %
    flushed values the decision is BF16 without a proof (separate copy), with none it is E4M3.  Every output equals the
    oracle's either way, and the fallback buffer is untouched when the decision is E4M3."""
    rows, cols = shape
    x = _with_tiny(rows, cols, frac, 11 + int(frac * 100))
    xb = np.zeros((rows, cols + pad), np.uint16)
    xb[:, :cols] = W.f32_to_bf16_bits(x)
    r = parity.compare(xb, gran, "tensor", "mean_rel_err", 0.045, cols=cols, label=f"gam proof frac={frac}", scaling="gam")
    assert r["n_bf16"] == (r["P"] if frac > 0 else 0)
    # fake quantization of the same operand: a proven BF16 tensor passes through without its de-quantized values being stored
    f = parity.compare_fake(xb, gran, "tensor", "mean_rel_err", 0.045, cols=cols, label=f"gam proof fake frac={frac}", scaling="gam")
    assert f["n_bf16"] == r["n_bf16"] and f["n_mismatch"] == 0


def test_gam_tensor_level_proof_uses_each_rows_own_amax():
    """Per-channel rows: rows of small values only do not flush, whatever the other rows hold."""
    x = _with_tiny(64, 4096, 0.0, 15)
    x[1:, :] *= np.float32(2.0 ** -30)
    x[0, np.random.default_rng(16).random(4096) < 0.5] = np.float32(2.0 ** -30)     # half of one row flushes
    r = parity.compare(W.f32_to_bf16_bits(x), "channel_row", "tensor", "mean_rel_err", 0.045, label="gam proof per row", scaling="gam")
    assert r["n_bf16"] == 0


@pytest.mark.parametrize("gran", ["sub1x128", "sub128x1"])
def test_gam_tensor_level_proof_uses_each_sub_channels_own_amax(gran):
    """Sub-channels of small values only do not flush; the few sub-channels with large values hold 3 % of flushes: no proof,
    and the decision (E4M3) comes from the error sums.  With 30 % of certain flushes in every sub-channel the pre-pass
    proves BF16."""
    rows, cols = 256, 384
    x = _with_tiny(rows, cols, 0.0, 45)
    big = np.zeros((rows, cols), bool)
    if gran == "sub1x128":
        big[::8, :128] = True                              # one sub-row in eight of the first column strip keeps its large values
    else:
        big[:128, ::8] = True                              # one sub-column in eight of the first row strip
    x[~big] *= np.float32(2.0 ** -30)
    x[big & (np.random.default_rng(46).random((rows, cols)) < 0.03)] = np.float32(2.0 ** -30)
    xb = W.f32_to_bf16_bits(x)
    r = parity.compare(xb, gran, "tensor", "mean_rel_err", 0.045, label="gam proof per sub-channel", scaling="gam")
    assert r["n_bf16"] == 0
    assert parity.compare_fake(xb, gran, "tensor", "mean_rel_err", 0.045, label="gam proof per sub-channel, fake", scaling="gam")["n_bf16"] == 0
    x2 = _with_tiny(rows, cols, 0.3, 47, tiny_exp=-30)
    x2[128:, :] *= np.float32(2.0 ** -20)                  # flushes relative to their own sub-channel's amax all the same
    r = parity.compare(W.f32_to_bf16_bits(x2), gran, "tensor", "mean_rel_err", 0.045, label="gam proof per sub-channel, mixed", scaling="gam")
    assert r["n_bf16"] == r["P"]


def test_gam_tensor_level_proof_uses_each_blocks_own_amax():
    """Values that flush next to the large amax of one block do not flush in blocks that hold nothing larger: a bound taken
    from the operand's amax would 'prove' a BF16 decision that the error sums do not support."""
    rows, cols = 256, 256
    x = _with_tiny(rows, cols, 0.0, 5)
    x[128:, :] *= np.float32(2.0 ** -30)                  # two blocks of small values only
    x[:128, 128:] *= np.float32(2.0 ** -30)               # and a third
    top = np.random.default_rng(6).random((128, 128)) < 0.03
    x[:128, :128][top] = np.float32(2.0 ** -30)            # 3 % of the remaining block flushes
    xb = W.f32_to_bf16_bits(x)
    r = parity.compare(xb, "block128", "tensor", "mean_rel_err", 0.045, label="gam proof per block", scaling="gam")
    assert r["n_bf16"] == 0
    assert parity.compare_fake(xb, "block128", "tensor", "mean_rel_err", 0.045, label="gam proof per block, fake", scaling="gam")["n_bf16"] == 0
    # 64 x 64 blocks: the same picture one size down (the block at the origin holds the large values and its 3 % of flushes)
    x = _with_tiny(128, 256, 0.0, 25)
    x[64:, :] *= np.float32(2.0 ** -30)
    x[:64, 64:] *= np.float32(2.0 ** -30)
    x[:64, :64][np.random.default_rng(26).random((64, 64)) < 0.03] = np.float32(2.0 ** -30)
    r = parity.compare(W.f32_to_bf16_bits(x), "block64", "tensor", "mean_rel_err", 0.045, label="gam proof per 64x64 block", scaling="gam")
    assert r["n_bf16"] == 0
    # the same operand once its flushes are frequent enough in every block
    x2 = _with_tiny(rows, cols, 0.3, 9, tiny_exp=-30)
    x2[128:, :] *= np.float32(2.0 ** -20)
    r = parity.compare(W.f32_to_bf16_bits(x2), "block128", "tensor", "mean_rel_err", 0.045, label="gam proof mixed", scaling="gam")
    assert r["n_bf16"] == r["P"]


def test_gam_tensor_level_proof_in_a_batch_with_statistics():
    """Several provable and unprovable operands in one batch call (one pre-pass launch for all of them)."""
    from oracle import mor_oracle as O
    dev = torch.device("cuda")
    specs = [(512, 1024, 0.2, "block128"), (256, 384, 0.0, "block128"), (384, 512, 0.04, "block128"), (128, 128, 0.5, "block128"),
             (640, 256, 0.1, "block128"), (256, 640, 0.2, "block64"), (128, 128, 0.0, "block64"), (33, 4096, 0.2, "channel_row"), (7, 17000, 0.3, "channel_row"), (50, 512, 0.0, "channel_row"),
             (384, 512, 0.2, "sub1x128"), (128, 256, 0.0, "sub1x128"), (256, 256, 0.04, "sub1x128"), (384, 256, 0.2, "sub128x1"), (128, 384, 0.0, "sub128x1")]
    ops, keep = [], []
    for k, (rows, cols, frac, gran) in enumerate(specs):
        xb = W.f32_to_bf16_bits(_with_tiny(rows, cols, frac, 40 + k))
        params = B.make_params(rows, cols, gran, "tensor", "mean_rel_err", 0.045, scaling="gam")
        xd = parity.to_dev(xb)
        out = B.alloc_outputs(params, dev, want_bf16=True, bf16_fill=parity.FILL)
        st = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)
        ops.append((params, xd, out, st)); keep.append(xb)
    items = B.make_batch(ops)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    for _ in range(2):                                     # twice on the same workspace
        B.mor_analyze_quantize_batch(items, 1e-5, ws)
    torch.cuda.synchronize()
    for (params, xd, out, st), xb, (rows, cols, frac, gran) in zip(ops, keep, specs):
        r = parity.compare(xb, gran, "tensor", "mean_rel_err", 0.045, label="gam proof batch", scaling="gam", gpu=(params, out))
        assert r["n_bf16"] == (r["P"] if frac > 0 else 0)
        s = B.read_stats(st)
        assert s["n_bf16_part"] == r["n_bf16"] and s["n_part"] == r["P"]


def test_gam_tensor_level_full_benchmark_sizes():
    """The full-size weight (cfg3, stays E4M3) and gradient (cfg4, BF16 proven by the pre-pass) operands with a tensor-level
    decision over GAM-scaled 128x128 blocks and per-channel rows, all in one batch call as the benchmark issues it."""
    dev = torch.device("cuda")
    (_, w, _), _ = W.cfg3()
    (_, g, _), _ = W.cfg4()
    ops, keep = [], []
    for xb in (w, g):
        xd = parity.to_dev(xb)
        for gran in ("block128", "block64", "channel_row", "sub1x128", "sub128x1"):
            params = B.make_params(xb.shape[0], xb.shape[1], gran, "tensor", "mean_rel_err", 0.045, scaling="gam")
            out = B.alloc_outputs(params, dev, want_bf16=True, bf16_fill=parity.FILL)
            ops.append((params, xd, out, None)); keep.append((xb, gran))
    items = B.make_batch(ops)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    B.mor_analyze_quantize_batch(items, 1e-5, ws)
    torch.cuda.synchronize()
    for (params, xd, out, _), (xb, gran) in zip(ops, keep):
        r = parity.compare(xb, gran, "tensor", "mean_rel_err", 0.045, label="gam tensor-level full size", scaling="gam", gpu=(params, out))
        if gran == "sub1x128":      # a uniformly shrunk sub-channel does not flush under its own scale: the gradient stays E4M3 too
            assert r["n_bf16"] == 0
        else:
            assert r["n_bf16"] == (r["P"] if xb is g else 0)


@pytest.mark.parametrize("th", [0.0, 0.01, 0.3, 0.95, 1.5])
@pytest.mark.parametrize("gran", ["block128", "block64", "channel_row", "sub1x128", "sub128x1"])
def test_gam_tensor_level_thresholds_outside_the_usual_range(th, gran):
    """20 % flushed values: BF16 for th <= 0.2 (proven or not), E4M3 above; thresholds for which no proof is attempted
    (0, >= 0.9) take the separate copy and give the same outputs."""
    xb = W.f32_to_bf16_bits(_with_tiny(256, 512, 0.2, 77))
    r = parity.compare(xb, gran, "tensor", "mean_rel_err", th, label=f"gam th={th}", scaling="gam")
    assert r["n_bf16"] == (r["P"] if th < 0.2 else 0)


def test_gam_tensor_level_proof_with_a_dirty_workspace_and_in_a_graph():
    """Nothing may depend on what the workspace held before (partials, the 'proven' word): the batch of provable and
    unprovable operands is run on a workspace filled with 0xFF, then captured in a HIP graph and replayed three times with
    the workspace and the outputs scrubbed in between; every run gives the outputs of the first, which equal the oracle's."""
    dev = torch.device("cuda")
    specs = [(512, 1024, 0.2, "block128"), (256, 384, 0.0, "block128"), (384, 512, 0.04, "block128"),
             (33, 4096, 0.2, "channel_row"), (50, 512, 0.0, "channel_row"), (256, 512, 0.2, "sub1x128"), (256, 384, 0.2, "sub128x1")]
    ops, keep = [], []
    for k, (rows, cols, frac, gran) in enumerate(specs):
        xb = W.f32_to_bf16_bits(_with_tiny(rows, cols, frac, 60 + k))
        params = B.make_params(rows, cols, gran, "tensor", "mean_rel_err", 0.045, scaling="gam")
        out = B.alloc_outputs(params, dev, want_bf16=True, bf16_fill=parity.FILL)
        ops.append((params, parity.to_dev(xb), out, None)); keep.append(xb)
    items = B.make_batch(ops)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    fields = ("fp8", "bf16", "scale", "amax", "nnz", "mask", "err_sum", "scale_e8m0", "group_mantissa")

    def snapshot():
        torch.cuda.synchronize()
        return [[getattr(o, f).clone() for f in fields] for _, _, o, _ in ops]

    def scrub():
        ws.fill_(0xFF)
        for _, _, o, _ in ops:
            o.fp8.zero_(); o.mask.fill_(9); o.err_sum.fill_(-1.0)
            o.bf16.fill_(parity.FILL if parity.FILL < 0x8000 else parity.FILL - 0x10000)

    scrub()
    B.mor_analyze_quantize_batch(items, 1e-5, ws)
    want = snapshot()
    for (params, xd, out, _), xb, (rows, cols, frac, gran) in zip(ops, keep, specs):
        r = parity.compare(xb, gran, "tensor", "mean_rel_err", 0.045, label="gam proof dirty workspace", scaling="gam", gpu=(params, out))
        assert r["n_bf16"] == (r["P"] if frac > 0 else 0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.mor_analyze_quantize_batch(items, 1e-5, ws)
    for _ in range(3):
        scrub()
        graph.replay()
        for a, b in zip(want, snapshot()):
            for ta, tb in zip(a, b):
                assert torch.equal(ta.view(torch.uint8), tb.view(torch.uint8))
        scrub()
        B.mor_analyze_quantize_batch(items, 1e-5, ws)       # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("scaling", ["fp32_amax", "gam", "e8m0"])
@pytest.mark.parametrize("frac", [0.0, 0.04, 0.2])
@pytest.mark.parametrize("shape,pad,ragged", [((1280, 384), 0, False), ((700, 264), 8, True), ((2304, 128), 0, False)])
def test_per_channel_columns_tensor_level_decision(scaling, frac, shape, pad, ragged):
    """Per-channel columns with a tensor-level decision (the second GEMM operand of the per-channel strategy, Section
    4.1.1): under GAM the group mantissa comes out of the column-amax pass (no pre-pass), and with enough certain
    flushes over all columns the quantize pass writes the BF16 fallback itself.  Every output equals the oracle's."""
    rows, cols = shape
    x = _with_tiny(rows, cols, frac, 90 + int(frac * 100))
    xb = np.zeros((rows, cols + pad), np.uint16)
    xb[:, :cols] = W.f32_to_bf16_bits(x)
    r = parity.compare(xb, "channel_col", "tensor", "mean_rel_err", 0.045, cols=cols, label=f"columns tensor-level frac={frac}",
                       scaling=scaling, ragged=ragged)
    assert r["n_bf16"] == (r["P"] if frac > 0 else 0)
    f = parity.compare_fake(xb, "channel_col", "tensor", "mean_rel_err", 0.045, cols=cols, label="columns tensor-level fake",
                            scaling=scaling, ragged=ragged)
    assert f["n_bf16"] == r["n_bf16"] and f["n_mismatch"] == 0


def test_per_channel_columns_tensor_level_proof_uses_each_columns_own_amax():
    """Columns of small values only do not flush; a bound taken from the operand's amax would prove a BF16 decision that
    the error sums do not support."""
    x = _with_tiny(512, 256, 0.0, 35)
    x[:, 1:] *= np.float32(2.0 ** -30)
    x[np.random.default_rng(36).random(512) < 0.5, 0] = np.float32(2.0 ** -30)      # half of one column flushes
    r = parity.compare(W.f32_to_bf16_bits(x), "channel_col", "tensor", "mean_rel_err", 0.045, label="columns own amax", scaling="gam")
    assert r["n_bf16"] == 0


# ---- GAM with several groups per tensor: the groups of Algorithm 1 as bands of rows ---------------------------------
def _banded(rows, cols, seed, tiny_frac=0.0):
    """Rows of very different magnitude, so that the bands' amaxes (and mantissas) differ."""
    rng = np.random.default_rng(seed)
    x = (np.exp2(rng.uniform(-4.0, 4.0, size=(rows, cols))) * rng.choice([-1.0, 1.0], size=(rows, cols))).astype(np.float32)
    x *= np.exp2(rng.integers(-12, 12, size=(rows, 1))).astype(np.float32)
    if tiny_frac:
        x[rng.random((rows, cols)) < tiny_frac] = np.float32(2.0 ** -60)
    return W.f32_to_bf16_bits(x)


@pytest.mark.parametrize("gran,shape,band", [("sub1x128", (64, 512), 8), ("sub1x128", (10, 256), 4), ("sub1x128", (96, 4096), 1),
                                             ("channel_row", (37, 640), 5), ("channel_row", (8, 9000), 2), ("block128", (640, 384), 128),
                                             ("block128", (512, 256), 384), ("block64", (320, 256), 64), ("block64", (256, 128), 128),
                                             ("sub128x1", (384, 256), 128), ("sub128x1", (512, 136), 256)])
@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
def test_gam_row_band_groups(gran, shape, band, crit):
    """Every output equals the oracle's: one mantissa pair per band in group_mantissa, per-block E8M0 exponents, scales,
    codes, error sums, decisions (per block and per tensor), fake quantization, and de-quantization from the stored form."""
    rows, cols = shape
    xb = _banded(rows, cols, rows + cols + band, tiny_frac=0.02)
    r = parity.compare(xb, gran, "partition", crit, 0.045, label="gam bands", scaling="gam", gam_group_rows=band)
    assert r["gpu"].group_mantissa.numel() == 2 * -(-rows // band)
    g, params = r["gpu"], r["params"]
    # stored form -> scale, band by band
    y = torch.full((rows, cols), 0x1111, dtype=torch.int16, device="cuda")
    y2 = torch.full_like(y, 0x2222)
    B.mor_dequantize_e8m0(params, g.fp8, g.scale_e8m0, g.group_mantissa, g.mask, g.bf16, y)
    B.mor_dequantize(params, g.fp8, g.scale, g.mask, g.bf16, y2)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    from oracle import mor_oracle as O
    want = O.dequantize(g.fp8.cpu().numpy(), g.scale.cpu().numpy(), g.mask.cpu().numpy(), parity.u16(g.bf16), gran)
    assert np.array_equal(parity.u16(y), want)
    if crit == "mean_rel_err":
        parity.compare(xb, gran, "tensor", crit, 0.045, label="gam bands, tensor-level", scaling="gam", gam_group_rows=band)
        f = parity.compare_fake(xb, gran, "partition", crit, 0.045, label="gam bands, fake", scaling="gam", gam_group_rows=band)
        assert f["n_mismatch"] == 0


def test_gam_row_band_groups_in_a_batch_and_degenerate_bands():
    """Operands with and without bands in one batch call (de-quantized in one batch call from the stored form); a band of
    at least `rows` rows is one group; the parameter is ignored without GAM scaling."""
    dev = torch.device("cuda")
    specs = [("sub1x128", (64, 512), 8), ("block128", (384, 256), 128), ("block128", (256, 256), 0), ("channel_row", (20, 1024), 4),
             ("sub128x1", (256, 128), 128), ("block64", (128, 192), 64)]
    ops, keep = [], []
    for k, (gran, (rows, cols), band) in enumerate(specs):
        xb = _banded(rows, cols, 300 + k)
        params = B.make_params(rows, cols, gran, scaling="gam", gam_group_rows=band)
        out = B.alloc_outputs(params, dev, want_bf16=True, bf16_fill=parity.FILL)
        out.workspace = None
        ops.append((params, parity.to_dev(xb), out, None)); keep.append((xb, gran, band))
    items = B.make_batch(ops)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    B.mor_analyze_quantize_batch(items, 1e-5, ws)
    torch.cuda.synchronize()
    ys = [torch.full_like(o.bf16, 0x1111) for _, _, o, _ in ops]
    B.mor_dequantize_batch(B.make_dequant_batch([(p, o, y, True) for (p, _, o, _), y in zip(ops, ys)]))
    torch.cuda.synchronize()
    from oracle import mor_oracle as O
    for (params, xd, out, _), (xb, gran, band), y in zip(ops, keep, ys):
        parity.compare(xb, gran, label="gam bands in a batch", scaling="gam", gam_group_rows=band, gpu=(params, out))
        want = O.dequantize(out.fp8.cpu().numpy(), out.scale.cpu().numpy(), out.mask.cpu().numpy(), parity.u16(out.bf16), gran)
        assert np.array_equal(parity.u16(y), want)
    xb = _banded(256, 256, 400)
    one = parity.compare(xb, "block128", label="one group", scaling="gam")
    whole = parity.compare(xb, "block128", label="band >= rows", scaling="gam", gam_group_rows=256)
    assert torch.equal(one["gpu"].scale, whole["gpu"].scale) and whole["gpu"].group_mantissa.numel() == 2
    parity.compare(xb, "block128", label="ignored for E8M0", scaling="e8m0", gam_group_rows=128)
    parity.compare(xb, "block128", label="ignored for FP32 amax", scaling="fp32_amax", gam_group_rows=128)
