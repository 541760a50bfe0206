"""A lone dense 1x128 operand in a batch call: its block kernel gathers the selection statistics (Section 4.1.3) of its
workgroups itself and one small launch combines them.  The statistics must equal those of the separate statistics call
on the same per-block outputs (integers exactly, the binary64 sums up to the order of summation) and the oracle's
statistics of the oracle's own outputs."""
import numpy as np
import pytest
import torch

from paper_2512_22804_amd import workloads as W

pytestmark = pytest.mark.gpu
NEAR = 1e-2
INT_KEYS = ("n_part", "n_fp8_part", "n_bf16_part", "n_e5m2_part", "n_elem_fp8", "n_elem_bf16", "n_elem_e5m2", "nnz_total",
            "hist", "n_near_threshold")


def _mixed(rows, cols, seed):
    """Heavy-tailed gradient whose chosen sub-channels are half shrunk: a mixed mask at 1x128."""
    return W.gradient(rows, cols, seed, tiny_frac=0.3, tiny_half=True)


def _check(oracle, xb, crit="mean_rel_err", th=0.045, scaling="fp32_amax", fake=False, calls=2, gam_group_rows=0):
    import parity
    from paper_2512_22804_amd import binding as B
    dev = torch.device("cuda:0")
    rows, cols = xb.shape
    params = B.make_params(rows, cols, "sub1x128", "partition", crit, th, scaling=scaling, gam_group_rows=gam_group_rows)
    x = parity.to_dev(xb)
    out = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
    st = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev)
    fake_y = torch.full((rows, cols), 0x5A5A, dtype=torch.int16, device=dev) if fake else None
    items = B.make_batch([(params, x, out, st, fake_y)])
    ws = torch.full((B.mor_batch_workspace_bytes(items),), 0xA7, dtype=torch.uint8, device=dev)
    for _ in range(calls):
        st.fill_(0xEE)
        B.mor_analyze_quantize_batch(items, NEAR, ws)
    torch.cuda.synchronize()
    got = B.read_stats(st)
    # (1) the separate statistics call on the very same per-block outputs
    st2 = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev)
    B.mor_select_stats(params, out.err_sum, out.nnz, out.mask, NEAR, st2)
    torch.cuda.synchronize()
    want = B.read_stats(st2)
    for k in want:
        if k == "flags":
            continue
        if k in ("err_sum_total", "mean_err"):
            assert got[k] == pytest.approx(want[k], rel=1e-12) or (np.isinf(got[k]) and np.isinf(want[k])) or \
                (np.isnan(got[k]) and np.isnan(want[k])), (k, got[k], want[k])
        else:
            assert got[k] == want[k], (k, got[k], want[k])
    # (2) the oracle, on its own analysis of the same input
    a = oracle.analyze_quantize(xb, "sub1x128", "partition", crit, th, scaling=scaling, gam_group_rows=gam_group_rows,
                                want_fake=fake)
    mask = out.mask.cpu().numpy()
    err = out.err_sum.cpu().numpy()
    assert np.array_equal(out.nnz.cpu().numpy(), a.nnz)
    # the per-block outputs and the payloads of this kernel variant, bit for bit
    assert np.array_equal(out.scale.cpu().numpy().view(np.uint32), a.scale.view(np.uint32))
    assert np.array_equal(out.amax.cpu().numpy().view(np.uint32), a.amax.view(np.uint32))
    finite = np.isfinite(a.err_sum)
    assert np.allclose(err[finite], a.err_sum[finite], rtol=1e-5, atol=128 * 2.0 ** -23)
    if np.array_equal(mask, a.mask):
        if fake:
            assert np.array_equal(parity.u16(fake_y), a.fake)
        else:
            assert np.array_equal(out.fp8.cpu().numpy(), a.fp8)
            rows_bf16 = np.repeat(a.mask.reshape(rows, cols // 128) == 1, 128, axis=1)
            got_bf16 = parity.u16(out.bf16)
            assert np.array_equal(got_bf16[rows_bf16], xb[rows_bf16])
            assert (got_bf16[~rows_bf16] == parity.FILL).all()
    if np.array_equal(mask, a.mask):
        ref = oracle.select_stats(err, a.nnz, a.mask, rows, cols, "sub1x128", th, NEAR)
        for k in INT_KEYS:
            if k in ref:
                assert got[k] == ref[k], (k, got[k], ref[k])
        ref_o = oracle.select_stats(a.err_sum, a.nnz, a.mask, rows, cols, "sub1x128", th, NEAR)
        if np.isfinite(ref_o["err_sum_total"]):
            assert got["err_sum_total"] == pytest.approx(ref_o["err_sum_total"], rel=1e-5, abs=1e-6)
    return got


@pytest.mark.parametrize("rows, cols", [(1, 4096), (2, 4096), (3, 4096), (8, 4096), (33, 4096), (256, 4096), (1024, 4096), (2, 2048)])
def test_lone_operand_small_and_ragged_unit_counts(oracle, rows, cols):
    """1, 2, 3 ... units: fewer units than waves of a workgroup, one workgroup, several, many."""
    got = _check(oracle, _mixed(rows, cols, 900 + rows))
    assert got["n_part"] == rows * cols // 128


def test_lone_operand_more_units_than_resident_waves(oracle):
    """8192 x 4096: 8192 units over the launch's 1536 workgroups (some waves take two units); a mixed mask."""
    got = _check(oracle, _mixed(8192, 4096, 77), calls=3)
    assert 0 < got["n_bf16_part"] < got["n_part"]


def test_lone_activation_full_size(oracle):
    (name, xb, gran), = W.cfg2()
    got = _check(oracle, xb)
    assert got["n_part"] == 262144


def test_lone_gradient_full_size_mixed_mask(oracle):
    """The benchmark's cfg4b call: 8192 x 14336, about 10 % of the 1x128 blocks fall back."""
    xb = W.cfg4(tiny_half=True)[0][1]
    got = _check(oracle, xb, calls=1)
    assert got["n_part"] == 917504 and 0.05 < got["n_bf16_part"] / got["n_part"] < 0.15


@pytest.mark.parametrize("crit", ["mean_rel_err", "e4m3_vs_e5m2"])
@pytest.mark.parametrize("fake", [False, True])
def test_lone_operand_criteria_and_fake_quantization(oracle, crit, fake):
    _check(oracle, _mixed(512, 2048, 5), crit=crit, fake=fake)


@pytest.mark.parametrize("scaling, bands", [("gam", 0), ("e8m0", 0), ("gam", 64)])
def test_lone_operand_other_scalings(oracle, scaling, bands):
    _check(oracle, _mixed(512, 2048, 6), scaling=scaling, gam_group_rows=bands)


def test_lone_operand_with_nonfinite_blocks_and_zero_blocks(oracle):
    xb = _mixed(64, 4096, 7).copy()
    xb[3, 128:256] = 0                       # an all-zero block
    xb[5, 7] = 0x7F80                        # +Inf
    xb[9, 300] = 0x7FC1                      # NaN
    xb[11, 0:128] = 0x0001                   # smallest subnormals only
    got = _check(oracle, xb)
    assert got["hist"][11] >= 2


def test_threshold_extremes(oracle):
    xb = _mixed(128, 4096, 8)
    all_fp8 = _check(oracle, xb, th=1.5)
    assert all_fp8["n_bf16_part"] == 0
    none_fp8 = _check(oracle, xb, th=0.0)
    assert none_fp8["n_fp8_part"] == 0


def test_alternating_sizes_on_one_workspace(oracle):
    """Many launches of different grid sizes in a row: no launch may read a record an earlier, larger launch left behind."""
    shapes = [(1024, 4096), (3, 4096), (256, 4096), (8192, 4096), (1, 4096)]
    xs = {s: _mixed(s[0], s[1], 31 + s[0]) for s in shapes}
    for rep in range(3):
        for s in shapes:
            _check(oracle, xs[s], calls=1)


def test_not_alone_or_not_eligible_still_right(oracle):
    """Two 1x128 operands in one batch (shared launch, separate statistics kernels), and a lone operand whose block count
    is not a multiple of 32 (the general kernel takes the tail): the statistics go the ordinary way."""
    import parity
    from paper_2512_22804_amd import binding as B
    dev = torch.device("cuda:0")
    entries, keep = [], []
    for seed, (rows, cols) in enumerate([(256, 4096), (128, 2048)]):
        xb = _mixed(rows, cols, 50 + seed)
        params = B.make_params(rows, cols, "sub1x128", "partition", "mean_rel_err", 0.045)
        out = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
        st = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev)
        entries.append((params, parity.to_dev(xb), out, st))
        keep.append(xb)
    items = B.make_batch(entries)
    ws = torch.empty(B.mor_batch_workspace_bytes(items), dtype=torch.uint8, device=dev)
    B.mor_analyze_quantize_batch(items, NEAR, ws)
    torch.cuda.synchronize()
    for (params, x, out, st), xb in zip(entries, keep):
        a = oracle.analyze_quantize(xb, "sub1x128", "partition", "mean_rel_err", 0.045)
        got = B.read_stats(st)
        if np.array_equal(out.mask.cpu().numpy(), a.mask):
            ref = oracle.select_stats(out.err_sum.cpu().numpy(), a.nnz, a.mask, xb.shape[0], xb.shape[1], "sub1x128", 0.045, NEAR)
            for k in INT_KEYS:
                if k in ref:
                    assert got[k] == ref[k], k
    _check(oracle, _mixed(5, 640, 60))       # 25 blocks: no whole unit
    _check(oracle, _mixed(9, 640, 61))       # 45 blocks: one unit and a tail


def test_lone_operand_in_a_graph_and_deterministic():
    """The lone-operand call only launches kernels: captured in a HIP graph, every replay into scrubbed buffers (with
    eager work in between, and with the workspace overwritten) gives the eager call's outputs and statistics bit for bit."""
    import parity
    from paper_2512_22804_amd import binding as B
    dev = torch.device("cuda:0")
    xb = _mixed(2048, 4096, 99)
    params = B.make_params(2048, 4096, "sub1x128", "partition", "mean_rel_err", 0.045)
    out = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
    st = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)
    x = parity.to_dev(xb)                     # (kept alive: the item array only holds its address)
    items = B.make_batch([(params, x, out, st)])
    ws = torch.empty(B.mor_batch_workspace_bytes(items), dtype=torch.uint8, device=dev)
    fields = ("fp8", "bf16", "scale", "amax", "nnz", "mask", "err_sum")

    def snapshot():
        torch.cuda.synchronize()
        return [getattr(out, f).clone() for f in fields] + [st.clone()]

    def scrub(fill):
        out.fp8.zero_(); out.mask.fill_(9); out.err_sum.fill_(-1.0); st.fill_(fill); ws.fill_(fill)
        out.bf16.fill_(parity.FILL if parity.FILL < 0x8000 else parity.FILL - 0x10000)

    scrub(0x11)
    B.mor_analyze_quantize_batch(items, NEAR, ws)
    want = snapshot()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.mor_analyze_quantize_batch(items, NEAR, ws)
    for rep in range(3):
        scrub(0x22 + rep)
        graph.replay()
        for a, b in zip(want, snapshot()):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
        scrub(0x55)
        B.mor_analyze_quantize_batch(items, NEAR, ws)       # eager work between the replays
        for a, b in zip(want, snapshot()):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


@pytest.mark.parametrize("seed", range(40))
def test_random_lone_operands(oracle, seed):
    """Random shapes (whole units, units and a tail, no whole unit), criteria, scalings, thresholds and output kinds."""
    rng = np.random.default_rng(31000 + seed)
    cols = 128 * int(rng.integers(1, 41))
    rows = int(rng.integers(1, 400))
    xb = W.gradient(rows, cols, 4000 + seed, tiny_frac=float(rng.choice([0.0, 0.1, 0.5])), tiny_half=bool(rng.integers(0, 2)))
    crit = ["mean_rel_err", "e4m3_vs_e5m2"][int(rng.integers(0, 2))]
    scaling = ["fp32_amax", "gam", "e8m0"][int(rng.integers(0, 3))]
    th = float(rng.choice([0.045, 0.02, 0.1, 0.5]))
    _check(oracle, xb, crit=crit, th=th, scaling=scaling, fake=bool(rng.integers(0, 2)), calls=1)
