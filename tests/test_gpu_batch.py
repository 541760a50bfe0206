"""The batch entry point must give exactly what operand-by-operand calls give (which the parity tests
check against the oracle), for every mix of granularity, criterion, scope and layout."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2512_22804_amd import workloads as W

pytestmark = pytest.mark.gpu

TH = 0.045


def build_cases():
    g1 = W.gradient(256, 512, 11, tiny_half=True)
    cases = [
        ("act-sub", W.activation(200, 1024, 1), "sub1x128", "partition", "mean_rel_err", None),          # 1600 blocks: ragged tail unit
        ("grad-sub", g1, "sub1x128", "partition", "mean_rel_err", None),
        ("grad-sub-eq3", g1, "sub1x128", "partition", "e4m3_vs_e5m2", None),
        ("w-block", W.weight(384, 512, 3), "block128", "partition", "mean_rel_err", None),
        ("grad-block", W.gradient(256, 768, 4), "block128", "partition", "mean_rel_err", None),
        ("grad-block-eq3", g1, "block128", "partition", "e4m3_vs_e5m2", None),
        ("w-tensor", W.weight(300, 520, 5), "tensor", "partition", "mean_rel_err", None),
        ("grad-tensor", W.gradient(256, 1024, 6), "tensor", "partition", "mean_rel_err", None),
        ("grad-tensor-eq3", g1, "tensor", "partition", "e4m3_vs_e5m2", None),
        ("tiny-tensor", W.activation(1, 8, 7), "tensor", "partition", "mean_rel_err", None),
        ("sub-tensor-scope", g1, "sub1x128", "tensor", "mean_rel_err", None),
        ("block-tensor-scope", g1, "block128", "tensor", "e4m3_vs_e5m2", None),
        ("strided-sub", W.gradient(128, 640, 8, tiny_half=True), "sub1x128", "partition", "mean_rel_err", 512),
        ("strided-block", W.gradient(128, 640, 9, tiny_half=True), "block128", "partition", "mean_rel_err", 512),
        ("strided-tensor", W.gradient(128, 640, 10), "tensor", "partition", "mean_rel_err", 512),
        ("patterns-sub", np.random.default_rng(1).permutation(np.arange(65536, dtype=np.uint32).astype(np.uint16)).reshape(512, 128),
         "sub1x128", "partition", "mean_rel_err", None),
    ]
    return cases


def test_batch_equals_single_calls(oracle):
    import parity
    from paper_2512_22804_amd import binding as B
    cases = build_cases()
    dev = torch.device("cuda:0")
    entries, singles, keep = [], [], []
    for name, xb, gran, scope, crit, cols in cases:
        rows, ld = xb.shape
        cols = ld if cols is None else cols
        params = B.make_params(rows, cols, gran, scope, crit, TH, ld=ld)
        x = parity.to_dev(xb)
        out_b = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
        out_s = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
        st_b = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev)
        st_s = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev)
        entries.append((params, x, out_b, st_b))
        singles.append((params, x, out_s, st_s))
        keep.append((name, xb, gran, scope, crit, cols))
    items = B.make_batch(entries)
    nbytes = B.mor_batch_workspace_bytes(items)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    for _ in range(2):                      # twice: the workspace is reusable without re-initialisation
        B.mor_analyze_quantize_batch(items, 1e-2, ws)
    for params, x, out, st in singles:
        B.mor_analyze_quantize(params, x, out)
        B.mor_select_stats(params, out.err_sum, out.nnz, out.mask, 1e-2, st)
    torch.cuda.synchronize()
    for (name, xb, gran, scope, crit, cols), (_, _, ob, sb), (_, _, os_, ss) in zip(keep, entries, singles):
        for f in ("fp8", "bf16", "scale", "amax", "nnz", "mask", "err_sum", "err5_sum"):
            a, b = getattr(ob, f), getattr(os_, f)
            if a is None:
                continue
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (name, f)
        got, want = B.read_stats(sb), B.read_stats(ss)
        for k in want:
            if k == "flags":
                continue                        # informational: the batch may fuse the fallback copy
            if k in ("err_sum_total", "mean_err"):
                assert got[k] == pytest.approx(want[k], rel=1e-12) or (np.isinf(got[k]) and np.isinf(want[k])), (name, k)
            else:
                assert got[k] == want[k], (name, k, got[k], want[k])
        # and the statistics agree with the oracle's on the oracle's own per-block outputs
        a = oracle.analyze_quantize(xb, gran, scope, crit, TH, ld=xb.shape[1], cols=cols)
        if np.array_equal(a.mask, ob.mask.cpu().numpy()):
            ref = oracle.select_stats(ob.err_sum.cpu().numpy(), a.nnz, a.mask, xb.shape[0], cols, gran, TH, 1e-2)
            for k in ("n_part", "n_fp8_part", "n_bf16_part", "n_elem_fp8", "n_elem_bf16", "nnz_total", "hist", "n_near_threshold"):
                assert got[k] == ref[k], (name, k)


def test_batch_argument_errors():
    import parity
    from paper_2512_22804_amd import binding as B
    xb = W.activation(128, 256, 1)
    x = parity.to_dev(xb)
    params = B.make_params(128, 256, "tensor")
    out = B.alloc_outputs(params, x.device)
    items = B.make_batch([(params, x, out, None)])
    with pytest.raises(B.MorError) as e:
        B.mor_analyze_quantize_batch(items, 1e-5, None)
    assert e.value.status == 5                                   # workspace missing
    bad = B.make_batch([(B.make_params(128, 200, "sub1x128"), x, out, None)])
    assert B.mor_batch_workspace_bytes(bad) == 0
    with pytest.raises(B.MorError) as e:
        B.mor_analyze_quantize_batch(bad, 1e-5, None)
    assert e.value.status == 2
    torch.cuda.synchronize()


def test_dequantize_batch_equals_single_calls(oracle):
    """One mor_dequantize_batch call over operands of every partition (incl. ragged edges, three types, the stored
    GAM form) gives bit for bit what the single-operand calls give, which in turn match the oracle."""
    import parity
    from paper_2512_22804_amd import binding as B
    rng = np.random.default_rng(17)
    cases = [("sub1x128", W.gradient(256, 512, 31, tiny_half=True), {}),
             ("block128", W.gradient(256, 512, 32, tiny_half=True), {}),
             ("block64", W.activation(130, 200, 33), {"ragged": True}),
             ("channel_row", W.activation(77, 1032, 34), {}),
             ("tensor", W.weight(128, 256, 35), {}),
             ("sub128x1", W.gradient(256, 384, 36, tiny_half=True), {}),
             ("channel_col", W.gradient(300, 264 - 8, 37), {}),
             ("sub1x128", W.gradient(128, 512, 38, tiny_half=True), {"crit": "e4m3_vs_e5m2", "formats": "e4m3|e5m2|bf16"}),
             ("block128", W.gradient(256, 256, 39, tiny_half=True), {"scaling": "gam", "stored": True})]
    entries, singles = [], []
    for gran, xb, kw in cases:
        stored = kw.pop("stored", False)
        params, g = parity.run_gpu(xb, gran, **kw)
        a = oracle.analyze_quantize(xb, gran, bf16_fill=parity.FILL, **kw)
        y_b = torch.full(xb.shape, 0x2222, dtype=torch.int16, device="cuda")
        y_s = torch.full(xb.shape, 0x2222, dtype=torch.int16, device="cuda")
        entries.append((params, g, y_b, stored))
        if stored:
            B.mor_dequantize_e8m0(params, g.fp8, g.scale_e8m0, g.group_mantissa, g.mask, g.bf16, y_s)
        else:
            B.mor_dequantize(params, g.fp8, g.scale, g.mask, g.bf16, y_s)
        singles.append((gran, xb, kw, a, g, y_s))
    B.mor_dequantize_batch(B.make_dequant_batch(entries))
    torch.cuda.synchronize()
    for (gran, xb, kw, a, g, y_s), (_, _, y_b, _) in zip(singles, entries):
        assert torch.equal(y_b, y_s), gran
        if np.array_equal(g.mask.cpu().numpy(), a.mask):
            want = oracle.dequantize(a.fp8, a.scale, a.mask, a.bf16, gran, ragged=kw.get("ragged", False))
            assert np.array_equal(parity.u16(y_b), want), gran


def test_cfg5_full_size_batch_matches_oracle(oracle):
    """The benchmark's own launch configuration: the twelve full-size operands of the layer sweep in one
    mor_analyze_quantize_batch call with statistics, every output of every operand against the oracle."""
    import parity
    from paper_2512_22804_amd import binding as B
    from paper_2512_22804_amd import workloads as W
    dev = torch.device("cuda:0")
    sweep = W.cfg5()
    entries = []
    for name, xb, gran in sweep:
        params = B.make_params(xb.shape[0], xb.shape[1], gran, "partition", "mean_rel_err", TH)
        out = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
        st = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)
        entries.append((params, parity.to_dev(xb), out, st))
    items = B.make_batch(entries)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    for _ in range(2):                       # the second call reuses the workspace as the benchmark's loop does
        B.mor_analyze_quantize_batch(items, 1e-5, ws)
    torch.cuda.synchronize()
    n_fp8 = n_all = 0
    for (name, xb, gran), (params, _, out, st) in zip(sweep, entries):
        r = parity.compare(xb, gran, threshold=TH, label="cfg5-batch-" + name, gpu=(params, out))
        got = B.read_stats(st)
        a = r["oracle"]
        ref = oracle.select_stats(out.err_sum.cpu().numpy(), a.nnz, a.mask, xb.shape[0], xb.shape[1], gran, TH, 1e-5)
        for k in ("n_part", "n_fp8_part", "n_bf16_part", "n_elem_fp8", "n_elem_bf16", "nnz_total", "hist"):
            assert got[k] == ref[k], (name, k, got[k], ref[k])
        n_fp8 += got["n_elem_fp8"]; n_all += xb.size
        del r
    assert n_all == 503316480 and abs(n_fp8 / n_all - 0.5) < 0.01      # forward operands FP8, gradients BF16


def test_batch_call_can_be_captured_in_a_graph():
    """The library only launches kernels (no allocation, memset or synchronization), so a batch call can be captured
    in a HIP graph; every replay, with eager work and synchronizations in between, gives the eager call's outputs."""
    import parity
    from paper_2512_22804_amd import binding as B
    dev = torch.device("cuda:0")
    entries = []
    for name, xb, gran, scope, crit, cols in build_cases():
        rows, ld = xb.shape
        params = B.make_params(rows, ld if cols is None else cols, gran, scope, crit, TH, ld=ld)
        out = B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
        st = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)
        entries.append((params, parity.to_dev(xb), out, st))
    items = B.make_batch(entries)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    fields = ("fp8", "bf16", "scale", "amax", "nnz", "mask", "err_sum", "err5_sum")

    def snapshot():
        torch.cuda.synchronize()
        return [[getattr(o, f).clone() for f in fields if getattr(o, f) is not None] + [st.clone()] for _, _, o, st in entries]

    def scrub():
        for _, _, o, st in entries:
            o.fp8.zero_(); o.mask.fill_(9); o.err_sum.fill_(-1.0); st.zero_()
            o.bf16.fill_(parity.FILL if parity.FILL < 0x8000 else parity.FILL - 0x10000)

    B.mor_analyze_quantize_batch(items, 1e-2, ws)
    want = snapshot()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.mor_analyze_quantize_batch(items, 1e-2, ws)
    for _ in range(3):
        scrub()
        graph.replay()
        got = snapshot()
        for a, b in zip(want, got):
            for ta, tb in zip(a, b):
                assert torch.equal(ta.view(torch.uint8), tb.view(torch.uint8))
        B.mor_analyze_quantize_batch(items, 1e-2, ws)       # eager work between the replays
        torch.cuda.synchronize()


def test_cfg5_full_size_batch_is_deterministic():
    """Five runs of the benchmark's batch call into scrubbed buffers give bit-identical outputs (payloads, metadata,
    statistics): no result depends on timing or on what the buffers or the workspace held before."""
    from paper_2512_22804_amd import binding as B
    from paper_2512_22804_amd import workloads as W
    dev = torch.device("cuda:0")
    entries = []
    for name, xb, gran in W.cfg5():
        params = B.make_params(xb.shape[0], xb.shape[1], gran, "partition", "mean_rel_err", TH)
        x = torch.from_numpy(xb.view(np.int16)).to(dev)
        entries.append((params, x, B.alloc_outputs(params, dev, bf16_fill=0), torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)))
    items = B.make_batch(entries)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    fields = ("fp8", "bf16", "scale", "amax", "nnz", "mask", "err_sum")
    B.mor_analyze_quantize_batch(items, 1e-5, ws)
    torch.cuda.synchronize()
    want = [[getattr(o, f).clone() for f in fields] + [st.clone()] for _, _, o, st in entries]
    for run in range(4):
        ws.fill_(0x5A + run)
        for _, _, o, st in entries:
            o.fp8.fill_(run); o.bf16.zero_(); o.mask.fill_(7); o.err_sum.fill_(-1.0); st.zero_()
        B.mor_analyze_quantize_batch(items, 1e-5, ws)
        torch.cuda.synchronize()
        for (_, _, o, st), ref in zip(entries, want):
            for f, r in zip(fields, ref):
                assert torch.equal(getattr(o, f), r), (run, f)
            assert torch.equal(st, ref[-1]), (run, "stats")


def test_batch_with_more_operands_than_one_launch_group_holds():
    """60 operands (20 per-tensor, 20 at 128 x 128, 20 at 1 x 128, two of each kind with statistics only on some):
    more than any kernel's descriptor table holds, so every kind is split over several launches; results must equal
    operand-by-operand calls."""
    import parity
    from paper_2512_22804_amd import binding as B
    dev = torch.device("cuda:0")
    entries, singles = [], []
    for i in range(60):
        gran = ("tensor", "block128", "sub1x128")[i % 3]
        rows = 128 * (1 + i % 4)
        cols = 128 * (2 + i % 5)
        xb = W.gradient(rows, cols, 1000 + i, tiny_half=(i % 2 == 0)) if i % 7 else W.activation(rows, cols, 1000 + i)
        crit = "e4m3_vs_e5m2" if i % 5 == 0 else "mean_rel_err"
        params = B.make_params(rows, cols, gran, "partition", crit, TH)
        x = parity.to_dev(xb)
        want_stats = i % 4 != 1
        ob, os_ = B.alloc_outputs(params, dev, bf16_fill=parity.FILL), B.alloc_outputs(params, dev, bf16_fill=parity.FILL)
        sb = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev) if want_stats else None
        ss = torch.full((B.STATS_BYTES,), 0xEE, dtype=torch.uint8, device=dev) if want_stats else None
        entries.append((params, x, ob, sb))
        singles.append((params, x, os_, ss))
    items = B.make_batch(entries)
    ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
    B.mor_analyze_quantize_batch(items, 1e-2, ws)
    for params, x, out, st in singles:
        B.mor_analyze_quantize(params, x, out)
        if st is not None:
            B.mor_select_stats(params, out.err_sum, out.nnz, out.mask, 1e-2, st)
    torch.cuda.synchronize()
    for i, ((_, _, ob, sb), (_, _, os_, ss)) in enumerate(zip(entries, singles)):
        for f in ("fp8", "bf16", "scale", "amax", "nnz", "mask", "err_sum", "err5_sum"):
            a, b = getattr(ob, f), getattr(os_, f)
            if a is not None:
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (i, f)
        if sb is not None:
            got, want = B.read_stats(sb), B.read_stats(ss)
            for k in want:
                if k == "flags":
                    continue
                if k in ("err_sum_total", "mean_err"):
                    assert got[k] == pytest.approx(want[k], rel=1e-12) or (np.isinf(got[k]) and np.isinf(want[k])), (i, k)
                else:
                    assert got[k] == want[k], (i, k, got[k], want[k])
