"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Element-by-element at sizes that span several tiles and ragged tails, then at the
full benchmark sizes, plus edge cases.  All marked ``gpu``."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2512_22804_amd import workloads as W

pytestmark = pytest.mark.gpu

TH = 0.045


@pytest.fixture(scope="module")
def P():
    import parity
    from paper_2512_22804_amd import binding as B
    B.load()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return parity


def all_patterns():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


# ------------------------------------------------------------------ converter / edge-case sweeps

@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor"])
@pytest.mark.parametrize("order", ["natural", "shuffled", "finite_shuffled", "small_shuffled"])
def test_all_bf16_patterns(P, gran, order):
    """Every BF16 bit pattern (incl. NaN, Inf, -0, subnormals) in 512 blocks of 128: in natural order
    each block is a narrow range with its own scale; shuffled blocks have a huge dynamic range."""
    x = all_patterns()
    rng = np.random.default_rng(3)
    if order == "shuffled":
        x = rng.permutation(x)
    elif order == "finite_shuffled":
        x = rng.permutation(np.where((x & 0x7FFF) >= 0x7F80, x & 0x80FF, x))
    elif order == "small_shuffled":
        x = rng.permutation(np.where((x & 0x7FFF) >= 0x4B80, (x & 0x807F) | 0x3F00, x))   # amax < 2^25
    xb = x.reshape(512, 128) if gran == "sub1x128" else x.reshape(256, 256)
    for crit in ("mean_rel_err", "e4m3_vs_e5m2"):
        P.compare(xb, gran, crit=crit, threshold=TH, label=f"patterns-{order}")


def test_every_finite_scale_is_correctly_rounded(P):
    """One block per finite BF16 amax value (32 640 of them): the per-block IEEE division 448/amax,
    the FLT_MAX clamp for subnormal amax and the scale-1 rule for amax 0 must match bit for bit."""
    amax_bits = np.arange(0, 0x7F80, dtype=np.uint16)
    xb = np.zeros((len(amax_bits), 128), dtype=np.uint16)
    xb[:, 17] = amax_bits | 0x8000            # negative: sign must not matter
    xb[:, 90] = amax_bits >> 1                # something smaller
    P.compare(xb, "sub1x128", threshold=TH, label="all-amax")
    P.compare(xb, "sub1x128", crit="e4m3_vs_e5m2", label="all-amax-eq3")


def test_handworked_blocks(P):
    def blk(vals):
        v = np.zeros(128, dtype=np.float32); v[:len(vals)] = vals
        return W.f32_to_bf16_bits(v)
    rows = [
        blk([]),                                             # all zero
        blk([448.0] + [2.0 ** -11] * 127),                   # flushed -> err 127 -> BF16
        blk([448.0, 2.0 ** -10, 3 * 2.0 ** -10, 1.0625, -1.1875, 2.0 ** -9, 0.0, -0.0]),
        blk([3.0, -3.0, 1.5]),
        blk([1.0] * 64 + [2.0 ** -19] * 64),
        blk([448.0, 224.0, 1.0, 2.0 ** -12]),                # metric exactly 1/4
        np.array([1, 2, 0x8003] + [0] * 125, dtype=np.uint16),   # subnormal amax -> s = FLT_MAX
        blk([2.0 ** 100, 1.0, 2.0 ** -100]),                 # y underflows to exact zero in binary32
        blk([3e38, 1e-38, -2e-38]),
    ]
    xb = np.stack(rows * 15)[:128]                            # 128 rows so that block128 also runs
    r = P.compare(xb, "sub1x128", threshold=TH, label="handworked")
    g = r["gpu"]
    assert g.err_sum[1].item() == 127.0 and g.mask[1].item() == 1 and g.mask[0].item() == 0
    r = P.compare(xb, "sub1x128", threshold=0.25, label="handworked-th-quarter")
    assert r["gpu"].mask[5].item() == 1                       # strict "<"
    up = float(np.nextafter(np.float32(0.25), np.float32(1)))
    assert P.compare(xb, "sub1x128", threshold=up, label="handworked-th-above")["gpu"].mask[5].item() == 0
    P.compare(xb, "sub1x128", crit="e4m3_vs_e5m2", label="handworked-eq3")
    P.compare(xb, "block128", threshold=TH, label="handworked-block")
    P.compare(xb, "tensor", threshold=TH, label="handworked-tensor")


def test_power_of_two_closed_form_on_gpu(P):
    import refmodel as R
    grid = np.array(sorted(float(v) for v in R.fp8_values(4, 3).values() if v > 0), dtype=np.float32)
    rng = np.random.default_rng(8)
    y = grid[rng.integers(0, len(grid), size=(128, 256))] * (rng.integers(0, 2, size=(128, 256)) * 2 - 1).astype(np.float32)
    y[:, ::128] = 448.0
    xb = W.f32_to_bf16_bits(y * np.float32(2.0 ** -11))
    for gran in ("sub1x128", "block128", "tensor"):
        r = P.compare(xb, gran, threshold=TH, label="pow2")
        g = r["gpu"]
        assert torch.all(g.err_sum == 0) and torch.all(g.mask == 0) and torch.all(g.scale == 2.0 ** 11)
        from paper_2512_22804_amd import binding as B
        yb = torch.empty_like(g.bf16)
        B.mor_dequantize(r["params"], g.fp8, g.scale, g.mask, g.bf16, yb)
        torch.cuda.synchronize()
        assert np.array_equal(P.u16(yb), xb)


# ------------------------------------------------------------------ workloads, reduced size, all modes

def reduced_cases():
    return {
        "act": W.activation(384, 1024, W.seed_for(2)),
        "weight": W.weight(384, 512, W.seed_for(3)),
        "grad": W.gradient(256, 1792, W.seed_for(4)),
        "grad_half": W.gradient(384, 768, W.seed_for(4, 1), tiny_half=True),  # mixed mask at 1x128
        "outlier": W.outlier_normal(256, 256, W.seed_for(1)),
    }


@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor"])
@pytest.mark.parametrize("scope", ["partition", "tensor"])
@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
def test_reduced_workloads(P, gran, scope, crit):
    n_bf16 = 0
    for name, xb in reduced_cases().items():
        r = P.compare(xb, gran, scope, crit, TH, label=name)
        n_bf16 += r["n_bf16"]
    if gran != "sub1x128" and crit == "mean_rel_err":
        assert n_bf16 > 0                                     # the fallback path really ran


@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor"])
def test_leading_dimensions(P, gran):
    """Strided operand (ld > cols): the padding columns must be ignored."""
    xb = W.gradient(256, 640, 99, tiny_half=True)
    r = P.compare(xb, gran, threshold=TH, cols=512, label="strided")
    dense = P.compare(np.ascontiguousarray(xb[:, :512]), gran, threshold=TH, label="dense-of-strided")
    assert torch.equal(r["gpu"].fp8, dense["gpu"].fp8) and torch.equal(r["gpu"].mask, dense["gpu"].mask)
    r = P.compare(xb, gran, scope="tensor", crit="e4m3_vs_e5m2", cols=512, label="strided-tensor-scope")


@pytest.mark.parametrize("rows,cols", [(1, 128), (3, 128), (1, 256), (65, 384), (130, 128), (321, 1024)])
def test_small_and_ragged_shapes_sub(P, rows, cols):
    xb = W.activation(rows, cols, 5 + rows)
    P.compare(xb, "sub1x128", threshold=TH, label="small")
    P.compare(xb, "tensor", threshold=TH, label="small-tensor")


@pytest.mark.parametrize("rows,cols", [(1, 8), (7, 24), (33, 2056), (1000, 72)])
def test_ragged_shapes_tensor(P, rows, cols):
    xb = W.f32_to_bf16_bits(np.random.default_rng(rows).standard_normal((rows, cols)).astype(np.float32))
    P.compare(xb, "tensor", threshold=TH, label="ragged-tensor")
    P.compare(xb, "tensor", crit="e4m3_vs_e5m2", label="ragged-tensor-eq3")


def test_threshold_monotone_on_gpu(P):
    xb = W.gradient(256, 512, 21, tiny_half=True)
    prev = None
    for th in (0.0, 0.02, 0.045, 0.2, 0.6, 1.01):
        _, g = P.run_gpu(xb, "sub1x128", threshold=th)
        m = g.mask.cpu().numpy()
        if prev is not None:
            assert np.all(m <= prev)
        prev = m
    assert prev.sum() == 0


def test_determinism(P):
    xb = W.gradient(512, 1024, 77, tiny_half=True)
    for gran in ("sub1x128", "block128", "tensor"):
        _, a = P.run_gpu(xb, gran)
        _, b = P.run_gpu(xb, gran)
        for f in ("fp8", "bf16", "scale", "amax", "nnz", "mask"):
            assert torch.equal(getattr(a, f), getattr(b, f)), (gran, f)


def test_bf16_null_and_alias(P):
    from paper_2512_22804_amd import binding as B
    xb = W.gradient(128, 256, 3, tiny_half=True)
    params, ref = P.run_gpu(xb, "sub1x128")
    _, g = P.run_gpu(xb, "sub1x128", want_bf16=False)
    assert g.bf16 is None and torch.equal(g.mask, ref.mask) and torch.equal(g.fp8, ref.fp8)
    x = P.to_dev(xb)
    out = B.alloc_outputs(params, x.device, want_bf16=False)
    out.bf16 = x                                              # aliasing the input: writes are skipped
    B.mor_analyze_quantize(params, x, out)
    torch.cuda.synchronize()
    assert np.array_equal(P.u16(x), xb) and torch.equal(out.mask, ref.mask)


# ------------------------------------------------------------------ argument errors (host side, nothing launched)

def test_argument_errors(P):
    from paper_2512_22804_amd import binding as B
    xb = W.activation(128, 256, 1)
    x = P.to_dev(xb)

    def status(params, xx=None, mutate=None):
        out = B.alloc_outputs(B.make_params(128, 256, "sub1x128"), x.device)
        if mutate:
            mutate(out)
        try:
            B.mor_analyze_quantize(params, x if xx is None else xx, out)
        except B.MorError as e:
            return e.status
        return 0

    assert status(B.make_params(128, 256, "sub1x128")) == 0
    assert status(B.make_params(128, 200, "sub1x128")) == 2            # cols % 128
    assert status(B.make_params(100, 256, "block128")) == 2            # rows % 128
    assert status(B.make_params(128, 256, "sub1x128", ld=128)) == 2    # ld < cols
    assert status(B.make_params(128, 256, "sub1x128", ld=260)) == 3    # ld % 8
    assert status(B.make_params(128, 256, 7)) == 4
    assert status(B.make_params(128, 256, "sub1x128", formats=B.MOR_FMT_E4M3 | B.MOR_FMT_E5M2)) == 4     # no BF16 at the end
    assert status(B.make_params(128, 256, "sub1x128", formats=B.MOR_FMT_E4M3)) == 4
    bad_flags = B.make_params(128, 256, "sub1x128"); bad_flags.flags = 4
    assert status(bad_flags) == 4
    assert status(B.make_params(128, 260, "sub1x128", ld=264, ragged=True)) == 2                       # cols % 8
    assert status(B.make_params(128, 256, "sub1x128", scaling=3)) == 4
    assert status(B.make_params(128, 256, "sub1x128", crit=5)) == 4
    assert status(B.make_params(128, 256, "sub1x128"), xx=x.view(-1)[1:]) == 3   # misaligned input

    def drop_mask(o): o.mask = None
    assert status(B.make_params(128, 256, "sub1x128"), mutate=drop_mask) == 1
    assert status(B.make_params(128, 256, "sub1x128", crit="e4m3_vs_e5m2")) == 1  # err5_sum missing
    p_t = B.make_params(128, 256, "tensor")
    assert B.mor_workspace_bytes(p_t) > 0 and status(p_t) == 5                    # workspace missing
    torch.cuda.synchronize()


# ------------------------------------------------------------------ de-quantize and statistics

@pytest.mark.parametrize("gran", ["sub1x128", "block128", "tensor"])
def test_dequantize_parity(P, oracle, gran):
    from paper_2512_22804_amd import binding as B
    for name, xb in (("grad_half", W.gradient(256, 512, 31, tiny_half=True)), ("act", W.activation(128, 384, 32)),
                     ("patterns", np.random.default_rng(1).permutation(all_patterns()).reshape(256, 256))):
        a = oracle.analyze_quantize(xb, gran, threshold=TH, bf16_fill=0x1111)
        want = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, gran)
        params = B.make_params(xb.shape[0], xb.shape[1], gran)
        y = torch.full(xb.shape, 0x2222, dtype=torch.int16, device="cuda")
        B.mor_dequantize(params, torch.from_numpy(a.fp8).cuda(), torch.from_numpy(a.scale).cuda(),
                         torch.from_numpy(a.mask).cuda(), P.to_dev(a.bf16), y)
        torch.cuda.synchronize()
        assert np.array_equal(P.u16(y), want), (gran, name)


@pytest.mark.parametrize("gran,shape", [("sub1x128", (1024, 2048)), ("block128", (1024, 1024)), ("tensor", (64, 128))])
def test_select_stats_parity(P, oracle, gran, shape):
    from paper_2512_22804_amd import binding as B
    xb = W.gradient(shape[0], shape[1], 55, tiny_half=True)
    a = oracle.analyze_quantize(xb, gran, threshold=TH)
    err32 = a.err_sum.astype(np.float32)
    want = oracle.select_stats(err32, a.nnz, a.mask, shape[0], shape[1], gran, threshold=TH, near_tol=1e-2)
    params = B.make_params(shape[0], shape[1], gran, threshold=TH)
    out = torch.full((B.STATS_BYTES,), 0xFF, dtype=torch.uint8, device="cuda")
    for _ in range(2):                                        # second call must fully overwrite the first
        B.mor_select_stats(params, torch.from_numpy(err32).cuda(), torch.from_numpy(a.nnz.view(np.int32)).cuda(),
                           torch.from_numpy(a.mask).cuda(), 1e-2, out)
    got = B.read_stats(out)
    for k in ("n_part", "n_fp8_part", "n_bf16_part", "n_elem_fp8", "n_elem_bf16", "nnz_total", "n_near_threshold", "hist"):
        assert got[k] == want[k], (k, got[k], want[k])
    assert got["flags"] == 0
    assert got["err_sum_total"] == pytest.approx(want["err_sum_total"], rel=1e-12)
    assert got["mean_err"] == pytest.approx(want["mean_err"], rel=1e-12)


def test_select_stats_handworked(P):
    from paper_2512_22804_amd import binding as B
    err = np.array([0.0, 0.63, 0.64, 5.75, 5.76, 7.04, 7.05, 100.0, 0.0, np.inf], dtype=np.float32)
    nnz = np.array([128, 128, 128, 128, 128, 128, 128, 128, 0, 128], dtype=np.int32)
    mask = np.array([0, 0, 0, 0, 1, 1, 1, 1, 0, 1], dtype=np.uint8)
    out = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device="cuda")
    B.mor_select_stats(B.make_params(10, 128, "sub1x128", threshold=TH), torch.from_numpy(err).cuda(),
                       torch.from_numpy(nnz).cuda(), torch.from_numpy(mask).cuda(), 1e-3, out)
    got = B.read_stats(out)
    assert got["hist"] == [3, 1, 0, 0, 0, 0, 0, 0, 1, 1, 0, 4] and got["n_near_threshold"] == 1
    assert got["n_fp8_part"] == 5 and got["n_elem_bf16"] == 5 * 128 and got["nnz_total"] == 9 * 128
    assert np.isinf(got["err_sum_total"])


# ------------------------------------------------------------------ full benchmark sizes

def test_full_cfg1(P):
    for _, xb, gran in W.cfg1():
        P.compare(xb, gran, threshold=TH, label="cfg1")


def test_full_cfg2(P):
    (_, xb, gran), = W.cfg2()
    r = P.compare(xb, gran, threshold=TH, label="cfg2")
    print("cfg2:", {k: v for k, v in r.items() if k not in ("gpu", "oracle", "params")})


def test_full_cfg3(P):
    for _, xb, gran in W.cfg3():
        r = P.compare(xb, gran, threshold=TH, label="cfg3")
        print("cfg3:", gran, {k: v for k, v in r.items() if k not in ("gpu", "oracle", "params")})


def test_full_cfg4(P):
    for _, xb, gran in W.cfg4():
        r = P.compare(xb, gran, threshold=TH, label="cfg4")
        print("cfg4:", gran, {k: v for k, v in r.items() if k not in ("gpu", "oracle", "params")})
    xb = W.cfg4(rows=2048, tiny_half=True)[0][1]
    r = P.compare(xb, "sub1x128", threshold=TH, label="cfg4b")
    assert 0 < r["n_bf16"] < r["P"]


def test_full_configurations_with_eq3(P):
    """Every benchmark configuration once more with the E4M3-versus-E5M2 criterion (two-way recipe)."""
    cases = list(W.cfg1()) + list(W.cfg2()) + list(W.cfg3()) + list(W.cfg4())
    for name, xb, gran in cases:
        r = P.compare(xb, gran, crit="e4m3_vs_e5m2", label=f"{name}-eq3")
        print(name, gran, {k: v for k, v in r.items() if k not in ("gpu", "oracle", "params")})


@pytest.mark.parametrize("frac", [0.0, 0.02, 0.03, 0.042, 0.0455, 0.047, 0.06, 0.2, 1.0])
def test_per_tensor_fallback_with_and_without_proof(P, frac):
    """Per-tensor operands whose flushed fraction sweeps across the threshold: below it the error of the
    surviving values decides, just above it the decision is BF16 without the flush-count proof, well above
    it the proof triggers and the fallback is written by the quantize pass.  All must match the oracle."""
    rng = np.random.default_rng(int(frac * 1e4) + 1)
    rows, cols = 768, 1024
    x = np.exp2(rng.uniform(-3.0, 3.0, size=(rows, cols))).astype(np.float32) * (rng.integers(0, 2, size=(rows, cols)) * 2 - 1)
    x[0, 0] = 8.0                                                  # exact values inside the range: error 0 for them
    x = np.where(rng.random((rows, cols)) < 0.5, np.round(x * 4) / 4, x).astype(np.float32)
    tiny = rng.random((rows, cols)) < frac
    x[tiny] = np.float32(2.0 ** -40) * (1 + rng.random(int(tiny.sum())).astype(np.float32))
    x[rng.random((rows, cols)) < 0.03] = 0.0
    xb = W.f32_to_bf16_bits(x)
    r = P.compare(xb, "tensor", threshold=TH, label=f"flush-{frac}")
    if 0.06 <= frac < 1.0:                       # at 1.0 every value is tiny, so nothing flushes
        assert r["n_bf16"] == 1
    P.compare(xb, "tensor", crit="e4m3_vs_e5m2", label=f"flush-{frac}-eq3")
    P.compare(xb, "tensor", threshold=0.5, label=f"flush-{frac}-th0.5")


@pytest.mark.parametrize("frac", [0.0, 0.04, 0.2])
def test_lean_fp8_payload(P, frac):
    """MOR_FLAG_LEAN_FP8: every output equals the oracle's; the FP8 payload of a per-tensor operand whose BF16
    decision the amax pass proves is left untouched, any other operand's payload is written as usual."""
    from paper_2512_22804_amd import binding as B
    from oracle import mor_oracle as O
    rng = np.random.default_rng(int(frac * 1e4) + 7)
    rows, cols = 520, 1024
    x = np.exp2(rng.uniform(-3.0, 3.0, size=(rows, cols))).astype(np.float32) * (rng.integers(0, 2, size=(rows, cols)) * 2 - 1)
    tiny = rng.random((rows, cols)) < frac
    x[tiny] = np.float32(2.0 ** -40)
    xb = W.f32_to_bf16_bits(x)
    for gran in ("tensor", "block128"):
        if gran == "block128":
            xb = np.ascontiguousarray(xb[:512])
        params = B.make_params(xb.shape[0], cols, gran, threshold=TH, lean_fp8=True)
        xd = P.to_dev(xb)
        out = B.alloc_outputs(params, xd.device, want_bf16=True, bf16_fill=P.FILL)
        out.fp8.fill_(0xAA)
        st = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=xd.device)
        items = B.make_batch([(params, xd, out, st)])
        ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=xd.device)
        B.mor_analyze_quantize_batch(items, 1e-5, ws)
        torch.cuda.synchronize()
        stats = B.read_stats(st)
        a = O.analyze_quantize(xb, gran, "partition", "mean_rel_err", TH, bf16_fill=P.FILL)
        assert np.array_equal(out.mask.cpu().numpy(), a.mask) and np.array_equal(out.scale.cpu().numpy(), a.scale)
        assert np.array_equal(out.nnz.cpu().numpy().view(np.uint32), a.nnz)
        assert np.allclose(out.err_sum.cpu().numpy().astype(np.float64), a.err_sum, rtol=1e-5, atol=0)
        assert np.array_equal(P.u16(out.bf16), a.bf16)
        proven = bool(stats["flags"] & B.MOR_STATS_FLAG_FUSED_FALLBACK)
        fp8 = out.fp8.cpu().numpy()
        if gran == "tensor" and frac >= 0.2:
            assert proven and a.mask[0] == 1 and np.all(fp8 == 0xAA)
        else:
            assert not proven and np.array_equal(fp8, a.fp8)
            assert gran != "tensor" or a.mask[0] == (1 if frac > 0 else 0)      # 4 % flushed: BF16, but not proven beforehand


def test_operand_beyond_2_to_32_bytes(P):
    """Maximum sizes: one operand of 34 816 x 65 536 elements (2.28 G elements, 4.6 GB of BF16), so that element indices
    pass 2^31 and byte offsets pass 2^32 in the input, the payload and the fallback buffer; per-tensor, 128 x 128, 1 x 128
    and per-channel rows (of 65 536 elements), every output against the oracle.  The operand is 34 row bands of one random 1024-row band, each band in its own
    binade, a fifth of the 128 x 128 blocks carrying values that flush."""
    from paper_2512_22804_amd import binding as B
    from oracle import mor_oracle as O
    rows0, cols, bands = 1024, 65536, 34
    rng = np.random.default_rng(2512)
    base = rng.standard_normal((rows0, cols), dtype=np.float32)
    blk = rng.random((rows0 // 128, cols // 128)) < 0.2
    tiny = (rng.random((rows0, cols), dtype=np.float32) < 0.3) & np.repeat(np.repeat(blk, 128, 0), 128, 1)
    base[tiny] *= np.float32(2.0 ** -24)
    band = W.f32_to_bf16_bits(base)
    del base, tiny
    xb = np.empty((rows0 * bands, cols), np.uint16)
    for k in range(bands):
        # band k scaled by 2^(k - 17): the exponent field moves, zeros stay zeros (no value is near the ends of the range)
        xb[k * rows0:(k + 1) * rows0] = np.where((band & 0x7FFF) != 0, (band.astype(np.int32) + ((k - 17) << 7)).astype(np.uint16), band)
    assert xb.size > 2 ** 31
    xd = P.to_dev(xb)
    for gran in ("tensor", "block128", "sub1x128", "channel_row"):
        print(f"[parity] large operand {xb.shape} gran={gran}", flush=True)
        params = B.make_params(xb.shape[0], cols, gran, threshold=TH)
        out = B.alloc_outputs(params, xd.device, want_bf16=True, bf16_fill=P.FILL)
        B.mor_analyze_quantize(params, xd, out)
        torch.cuda.synchronize()
        a = O.analyze_quantize(xb, gran, "partition", "mean_rel_err", TH, bf16_fill=P.FILL)
        assert np.array_equal(out.amax.cpu().numpy().view(np.uint32), a.amax.view(np.uint32))
        assert np.array_equal(out.scale.cpu().numpy().view(np.uint32), a.scale.view(np.uint32))
        assert np.array_equal(out.nnz.cpu().numpy().view(np.uint32), a.nnz)
        assert np.array_equal(out.mask.cpu().numpy(), a.mask)             # no block is near the threshold (checked below)
        metric = a.err_sum / np.maximum(a.nnz, 1)
        assert np.all(np.abs(metric - TH) > 1e-3 * TH)
        assert np.allclose(out.err_sum.cpu().numpy().astype(np.float64), a.err_sum, rtol=1e-5, atol=0)
        assert np.array_equal(out.fp8.cpu().numpy(), a.fp8), "fp8 payload differs"
        assert np.array_equal(P.u16(out.bf16), a.bf16), "BF16 fallback differs"
        if gran in ("block128", "sub1x128"):
            assert 0.1 < a.mask.mean() < 0.3                              # both kinds of block occur
        del out, a
