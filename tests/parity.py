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


def to_dev(xb: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(xb.view(np.int16)).cuda()


def u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


def run_gpu(xb: np.ndarray, gran: str, scope: str = "partition", crit: str = "mean_rel_err", threshold: float = 0.045,
            cols: int | None = None, want_bf16: bool = True, scaling: str = "fp32_amax"):
    """xb: (rows, ld) uint16.  Returns (params, MorResult) with outputs still on the device."""
    rows, ld = xb.shape
    cols = ld if cols is None else cols
    params = B.make_params(rows, cols, gran, scope, crit, threshold, ld=ld, scaling=scaling)
    x = to_dev(xb)
    out = B.alloc_outputs(params, x.device, want_bf16=want_bf16, bf16_fill=FILL)
    B.mor_analyze_quantize(params, x, out)
    torch.cuda.synchronize()
    return params, out


def compare(xb: np.ndarray, gran: str, scope: str = "partition", crit: str = "mean_rel_err", threshold: float = 0.045,
            cols: int | None = None, label: str = "", scaling: str = "fp32_amax") -> dict:
    rows, ld = xb.shape
    cols = ld if cols is None else cols
    print(f"[parity] {label} shape={rows}x{cols} ld={ld} gran={gran} scope={scope} crit={crit} th={threshold} "
          f"scaling={scaling}", flush=True)
    params, g = run_gpu(xb, gran, scope, crit, threshold, cols, scaling=scaling)
    a = O.analyze_quantize(xb, gran, scope, crit, threshold, bf16_fill=FILL, ld=ld, cols=cols, scaling=scaling)
    P = a.mask.size
    if scaling != "fp32_amax":      # stored form of the scales: one E8M0 byte per block, one 23-bit mantissa
        assert np.array_equal(g.scale_e8m0.cpu().numpy(), a.e8m0), "E8M0 exponents differ"
        assert int(g.group_mantissa.cpu().numpy().view(np.uint32)[0]) == a.group_mantissa, "group mantissa differs"

    g_amax = g.amax.cpu().numpy(); g_scale = g.scale.cpu().numpy()
    assert np.array_equal(g_amax.view(np.uint32), a.amax.view(np.uint32)), "amax differs"
    assert np.array_equal(g_scale.view(np.uint32), a.scale.view(np.uint32)), "scale differs"
    g_fp8 = g.fp8.cpu().numpy()
    if not np.array_equal(g_fp8, a.fp8):
        bad = np.argwhere(g_fp8 != a.fp8)
        r, c = bad[0]
        raise AssertionError(f"fp8 differs at {len(bad)} elements, first ({r},{c}): gpu {g_fp8[r, c]:#x} oracle "
                             f"{a.fp8[r, c]:#x} x={xb[r, c]:#06x}")
    g_nnz = g.nnz.cpu().numpy().view(np.uint32)
    assert np.array_equal(g_nnz, a.nnz), "nnz differs"

    def check_err(ge, oe, what):
        ge = ge.astype(np.float64)
        both_inf = np.isinf(ge) & np.isinf(oe)
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

    g_mask = g.mask.cpu().numpy()
    # blocks (or the tensor) where the decision may legitimately differ
    if scope == "tensor":
        es, e5, n = a.err_sum.sum(), a.err5_sum.sum(), a.nnz.sum()
        es, e5, n = np.full(P, es), np.full(P, e5), np.full(P, n)
    else:
        es, e5, n = a.err_sum, a.err5_sum, a.nnz
    if crit == "e4m3_vs_e5m2":
        near = np.abs(es - e5) <= REL_TOL * np.maximum(es, e5)
    else:
        with np.errstate(invalid="ignore"):
            metric = np.where(n > 0, es / np.maximum(n, 1), 0.0)
        near = np.abs(metric - np.float32(threshold)) <= REL_TOL * np.float32(threshold)
    mism = g_mask != a.mask
    assert not (mism & ~near).any(), f"mask differs in {(mism & ~near).sum()} blocks away from the threshold"
    assert set(np.unique(g_mask)) <= {0, 1}

    # BF16 payload: input bits exactly where the GPU's own mask says BF16, untouched elsewhere
    g_bf16 = u16(g.bf16)
    pr, pc = {"tensor": (rows, cols), "sub1x128": (1, 128), "block128": (128, 128)}[gran]
    m2 = np.repeat(np.repeat(g_mask.reshape(rows // pr, cols // pc), pr, axis=0), pc, axis=1).astype(bool)
    xin = xb[:, :cols]
    assert np.array_equal(g_bf16[m2], xin[m2]), "BF16 fallback payload differs from the input"
    assert np.all(g_bf16[~m2] == FILL), "BF16 buffer written outside fallback blocks"
    if not mism.any():
        assert np.array_equal(g_bf16, a.bf16)
    return {"P": P, "n_bf16": int(g_mask.sum()), "n_near": int(near.sum()), "n_mask_mismatch_near": int(mism.sum()),
            "n_floor": n_floor, "max_rel_err": max_rel, "gpu": g, "oracle": a, "params": params}
