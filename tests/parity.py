"""Shared helper of the GPU parity tests: run one operand through the HIP library (via the C ABI
binding) and through the CPU oracle, and compare to the acceptance bar:

  amax, scale, FP8 bytes, nnz, BF16 payload   bit-exact
  err_sum / err5_sum                          1e-5 relative (absolute floor 2^-23 per non-zero
                                              element when the metric is below 1e-2 * th)
  mask                                        bit-exact except blocks whose metric lies within
                                              1e-5 * th of the threshold (Eq. 2) or whose two
                                              error totals agree to 1e-5 (Eq. 3); those are
                                              counted and returned
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import mor_oracle as O
from paper_2512_22804_amd import binding as B

REL_TOL = 1e-5
FILL = 0x5A5A        # pattern pre-filled into the BF16 fallback buffer to detect stray writes
GUARD = 512          # bytes of canary on either side of every output buffer and of the workspace
CANARY = 0xC3


class Guards:
    """Output buffers carved out of larger canary-filled allocations: `check()` fails if a kernel wrote outside one."""

    def __init__(self, device):
        self.device = device
        self.bufs = []

    def carve(self, name, shape, dtype, fill=None):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        body = (n + 255) // 256 * 256                  # keeps the view 256-byte aligned and the tail guard whole
        raw = torch.full((GUARD + body + GUARD,), CANARY, dtype=torch.uint8, device=self.device)
        view = raw[GUARD:GUARD + n].view(dtype).reshape(shape)
        if fill is not None:
            view.fill_(fill)
        self.bufs.append((name, raw, n))
        return view

    def check(self):
        for name, raw, n in self.bufs:
            assert bool((raw[:GUARD] == CANARY).all()), f"write BEFORE the start of {name}"
            assert bool((raw[GUARD + n:] == CANARY).all()), f"write BEYOND the end of {name}"


def guarded_outputs(params, device, want_bf16=True, bf16_fill=None, want_fp8=True):
    """The buffers of binding.alloc_outputs (dense leading dimensions), each between two guard bands."""
    g = Guards(device)
    rows, cols = params.rows, params.cols
    P = B.mor_params_num_partitions(params)
    fp8 = g.carve("fp8", (rows, cols), torch.uint8) if want_fp8 else None
    bf16 = None
    if want_bf16:
        bf16 = g.carve("bf16", (rows, cols), torch.int16,
                       None if bf16_fill is None else (bf16_fill if bf16_fill < 0x8000 else bf16_fill - 0x10000))
    err5 = g.carve("err5_sum", (P,), torch.float32) if params.criterion == B.MOR_CRIT_E4M3_VS_E5M2 else None
    nbytes = B.mor_workspace_bytes(params)
    ws = g.carve("workspace", (nbytes,), torch.uint8, 0xFF) if nbytes else None     # nothing may depend on what the workspace held before
    e8m0 = gmant = None
    if params.scaling != B.MOR_SCALE_FP32_AMAX:
        e8m0 = g.carve("scale_e8m0", (P,), torch.uint8, 0xEE)
        gmant = g.carve("group_mantissa", (2 * B.gam_groups(params),), torch.int32, -1)
    amin = g.carve("amin", (P,), torch.float32, -1.0) if params.formats & B.MOR_FMT_E5M2 else None
    out = B.MorResult(fp8, bf16, g.carve("scale", (P,), torch.float32), g.carve("amax", (P,), torch.float32),
                      g.carve("err_sum", (P,), torch.float32), g.carve("nnz", (P,), torch.int32), g.carve("mask", (P,), torch.uint8),
                      err5, ws, params, e8m0, gmant, amin)
    return out, g


def to_dev(xb: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(xb.view(np.int16)).cuda()


def u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


def block_map(gran: str, rows: int, cols: int) -> np.ndarray:
    """(rows, cols) array of block numbers, row-major over the block grid (edge blocks smaller)."""
    pr, pc = {"tensor": (rows, cols), "sub1x128": (1, 128), "block128": (128, 128), "channel_row": (1, cols),
              "channel_col": (rows, 1), "sub128x1": (128, 1), "block64": (64, 64)}[gran]
    gc = -(-cols // pc)
    return (np.arange(rows)[:, None] // pr) * gc + (np.arange(cols)[None, :] // pc)


def run_gpu(xb: np.ndarray, gran: str, scope: str = "partition", crit: str = "mean_rel_err", threshold: float = 0.045,
            cols: int | None = None, want_bf16: bool = True, scaling: str = "fp32_amax", formats: str = "e4m3|bf16",
            ragged: bool = False, gam_group_rows: int = 0):
    """xb: (rows, ld) uint16.  Returns (params, MorResult) with outputs still on the device."""
    rows, ld = xb.shape
    cols = ld if cols is None else cols
    params = B.make_params(rows, cols, gran, scope, crit, threshold, ld=ld, scaling=scaling, formats=formats, ragged=ragged,
                           gam_group_rows=gam_group_rows)
    x = to_dev(xb)
    out, guards = guarded_outputs(params, x.device, want_bf16=want_bf16, bf16_fill=FILL)
    B.mor_analyze_quantize(params, x, out)
    torch.cuda.synchronize()
    guards.check()
    return params, out


def compare(xb: np.ndarray, gran: str, scope: str = "partition", crit: str = "mean_rel_err", threshold: float = 0.045,
            cols: int | None = None, label: str = "", scaling: str = "fp32_amax", formats: str = "e4m3|bf16",
            ragged: bool = False, gpu=None, gam_group_rows: int = 0) -> dict:
    """``gpu``: (params, outputs) of a call already made (e.g. one operand of a batch call; its fallback buffer pre-filled
    with FILL); by default the operand is run through mor_analyze_quantize here."""
    rows, ld = xb.shape
    cols = ld if cols is None else cols
    print(f"[parity] {label} shape={rows}x{cols} ld={ld} gran={gran} scope={scope} crit={crit} th={threshold} "
          f"scaling={scaling} formats={formats} ragged={ragged} gam_group_rows={gam_group_rows}", flush=True)
    if gpu is None:
        params, g = run_gpu(xb, gran, scope, crit, threshold, cols, scaling=scaling, formats=formats, ragged=ragged,
                            gam_group_rows=gam_group_rows)
    else:
        params, g = gpu
    a = O.analyze_quantize(xb, gran, scope, crit, threshold, bf16_fill=FILL, ld=ld, cols=cols, scaling=scaling,
                           formats=formats, ragged=ragged, gam_group_rows=gam_group_rows)
    P = a.mask.size
    three = formats != "e4m3|bf16"
    bmap = block_map(gran, rows, cols)
    g_mask = g.mask.cpu().numpy()
    agree = g_mask == a.mask                # with three types, payload and scale follow the choice
    g_amax = g.amax.cpu().numpy(); g_scale = g.scale.cpu().numpy()
    assert np.array_equal(g_amax.view(np.uint32), a.amax.view(np.uint32)), "amax differs"
    assert np.array_equal(g_scale.view(np.uint32)[agree], a.scale.view(np.uint32)[agree]), "scale differs"
    if scaling != "fp32_amax":      # stored form of the scales: one E8M0 byte per block, shared 23-bit mantissas
        assert np.array_equal(g.scale_e8m0.cpu().numpy()[agree], a.e8m0[agree]), "E8M0 exponents differ"
        gm = g.group_mantissa.cpu().numpy().view(np.uint32)
        assert np.array_equal(gm.reshape(-1, 2), a.group_mantissas), "group mantissas differ"
    g_fp8 = g.fp8.cpu().numpy()
    same = agree[bmap]
    if not np.array_equal(g_fp8[same], a.fp8[same]):
        bad = np.argwhere((g_fp8 != a.fp8) & same)
        r, c = bad[0]
        raise AssertionError(f"fp8 differs at {len(bad)} elements, first ({r},{c}): gpu {g_fp8[r, c]:#x} oracle "
                             f"{a.fp8[r, c]:#x} x={xb[r, c]:#06x}")
    g_nnz = g.nnz.cpu().numpy().view(np.uint32)
    assert np.array_equal(g_nnz, a.nnz), "nnz differs"
    if three:                                 # smallest non-zero magnitude of the blocks that failed M_1
        failed = (a.mask != 0) & (g_mask != 0)
        assert np.array_equal(g.amin.cpu().numpy().view(np.uint32)[failed], a.amin.view(np.uint32)[failed]), "amin differs"

    def check_err(ge, oe, what):
        ge = ge.astype(np.float64)
        both_inf = np.isinf(ge) & np.isinf(oe)
        with np.errstate(invalid="ignore"):
            diff = np.abs(ge - oe)
        diff[both_inf] = 0.0
        ok = diff <= REL_TOL * np.abs(oe)
        metric = np.where(a.nnz > 0, oe / np.maximum(a.nnz, 1), 0.0)
        floor = (~ok) & (metric < 1e-2 * threshold) & (diff <= 2.0 ** -23 * np.maximum(a.nnz, 1))
        bad = ~(ok | floor)
        assert not bad.any(), (f"{what} differs in {bad.sum()} blocks, first p={np.argmax(bad)} gpu={ge[np.argmax(bad)]!r} "
                               f"oracle={oe[np.argmax(bad)]!r}")
        with np.errstate(invalid="ignore", divide="ignore"):
            rel = np.where(oe > 0, diff / oe, 0.0)
        return int(floor.sum()), float(np.nanmax(rel[~floor & np.isfinite(rel)], initial=0.0))

    n_floor, max_rel = check_err(g.err_sum.cpu().numpy(), a.err_sum, "err_sum")
    if crit == "e4m3_vs_e5m2":
        f5, r5 = check_err(g.err5_sum.cpu().numpy(), a.err5_sum, "err5_sum")
        n_floor += f5; max_rel = max(max_rel, r5)

    # blocks (or the tensor) where the M_1 decision may legitimately differ
    if scope == "tensor":
        es, e5, n = a.err_sum.sum(), a.err5_sum.sum(), a.nnz.sum()
        es, e5, n = np.full(P, es), np.full(P, e5), np.full(P, n)
    else:
        es, e5, n = a.err_sum, a.err5_sum, a.nnz
    if crit == "e4m3_vs_e5m2":
        with np.errstate(invalid="ignore"):
            near = np.abs(es - e5) <= REL_TOL * np.maximum(es, e5)
    else:
        with np.errstate(invalid="ignore"):
            metric = np.where(n > 0, es / np.maximum(n, 1), 0.0)
        near = np.abs(metric - np.float32(threshold)) <= REL_TOL * np.float32(threshold)
    mism = ~agree
    assert not (mism & ~near).any(), f"mask differs in {(mism & ~near).sum()} blocks away from the threshold"
    assert not (mism & (g_mask != 0) & (a.mask != 0)).any(), "E5M2 / BF16 choice (Eq. 4) differs"
    assert set(np.unique(g_mask)) <= ({0, 1, 2} if three else {0, 1})

    # BF16 payload: input bits exactly where the GPU's own mask says BF16, untouched elsewhere
    g_bf16 = u16(g.bf16)
    m2 = g_mask[bmap] == 1
    xin = xb[:, :cols]
    assert np.array_equal(g_bf16[m2], xin[m2]), "BF16 fallback payload differs from the input"
    assert np.all(g_bf16[~m2] == FILL), "BF16 buffer written outside fallback blocks"
    if not mism.any():
        assert np.array_equal(g_bf16, a.bf16)
    return {"P": P, "n_bf16": int((g_mask == 1).sum()), "n_e5m2": int((g_mask == 2).sum()), "n_near": int(near.sum()),
            "n_mask_mismatch_near": int(mism.sum()), "n_floor": n_floor, "max_rel_err": max_rel, "gpu": g, "oracle": a,
            "params": params}


def compare_fake(xb: np.ndarray, gran: str, scope: str = "partition", crit: str = "mean_rel_err", threshold: float = 0.045,
                 cols: int | None = None, label: str = "", scaling: str = "fp32_amax", formats: str = "e4m3|bf16",
                 ragged: bool = False, gam_group_rows: int = 0) -> dict:
    """mor_fake_quantize against the oracle's fake-quantized tensor, and against the library's own
    analyze + de-quantize pair (which must give the same bits)."""
    rows, ld = xb.shape
    cols = ld if cols is None else cols
    print(f"[parity-fake] {label} shape={rows}x{cols} ld={ld} gran={gran} scope={scope} crit={crit} th={threshold} "
          f"scaling={scaling} formats={formats} ragged={ragged}", flush=True)
    params = B.make_params(rows, cols, gran, scope, crit, threshold, ld=ld, scaling=scaling, formats=formats, ragged=ragged,
                           gam_group_rows=gam_group_rows)
    x = to_dev(xb)
    meta, guards = guarded_outputs(params, x.device, want_bf16=False, want_fp8=False)
    y = guards.carve("fake_y", (rows, cols), torch.int16, FILL if FILL < 0x8000 else FILL - 0x10000)
    B.mor_fake_quantize(params, x, y, meta)
    torch.cuda.synchronize()
    guards.check()
    a = O.analyze_quantize(xb, gran, scope, crit, threshold, ld=ld, cols=cols, scaling=scaling, formats=formats,
                           ragged=ragged, want_fake=True, gam_group_rows=gam_group_rows)
    g_mask = meta.mask.cpu().numpy()
    assert np.array_equal(meta.amax.cpu().numpy().view(np.uint32), a.amax.view(np.uint32)), "amax differs"
    assert np.array_equal(meta.nnz.cpu().numpy().view(np.uint32), a.nnz), "nnz differs"
    agree = g_mask == a.mask
    same = agree[block_map(gran, rows, cols)]
    gy = u16(y)
    if not np.array_equal(gy[same], a.fake[same]):
        bad = np.argwhere((gy != a.fake) & same)
        r, c = bad[0]
        raise AssertionError(f"fake-quantized tensor differs at {len(bad)} elements, first ({r},{c}): gpu {gy[r, c]:#06x} "
                             f"oracle {a.fake[r, c]:#06x} x={xb[r, c]:#06x}")
    # the analyse + de-quantize pair of the library gives the same tensor
    _, g = run_gpu(xb, gran, scope, crit, threshold, cols, scaling=scaling, formats=formats, ragged=ragged, gam_group_rows=gam_group_rows)
    y2 = torch.full_like(y, 0x1111)
    B.mor_dequantize(params, g.fp8, g.scale, g.mask, g.bf16, y2)
    torch.cuda.synchronize()
    assert torch.equal(g.mask, meta.mask) and torch.equal(y2, y), "fake quantization differs from analyse + de-quantize"
    assert torch.equal(g.err_sum, meta.err_sum) and torch.equal(g.scale, meta.scale)
    return {"n_mismatch": int((~agree).sum()), "n_bf16": int((g_mask == 1).sum()), "n_e5m2": int((g_mask == 2).sum()), "y": y,
            "meta": meta, "oracle": a}
