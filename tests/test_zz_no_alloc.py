"""mor_analyze_quantize_static -- the entry point that allocates nothing (its scratch is a fixed array inside the
library's device image) -- against mor_analyze_quantize on a caller-provided workspace: every output must be
identical, on two calls in a row that share the built-in scratch, the second with a smaller input, for every kind of
operand that uses scratch at all.  Collected last so that a failure here cannot hide another test."""
import numpy as np
import pytest
import torch

import parity
from paper_2512_22804_amd import binding as B
from paper_2512_22804_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(xb, gran, scope="partition", crit="mean_rel_err", threshold=0.045, scaling="fp32_amax"):
    rows, cols = xb.shape
    params = B.make_params(rows, cols, gran, scope, crit, threshold, scaling=scaling)
    assert 0 < B.mor_workspace_bytes(params) <= B.MOR_STATIC_SCRATCH_BYTES
    x = parity.to_dev(xb)
    ref = B.alloc_outputs(params, x.device, want_bf16=True, bf16_fill=parity.FILL)
    ref.workspace.fill_(0xFF)
    B.mor_analyze_quantize(params, x, ref)
    got = B.alloc_outputs(params, x.device, want_bf16=True, bf16_fill=parity.FILL)
    got.workspace = None                                    # not passed, not used
    B.mor_analyze_quantize_static(params, x, got)
    torch.cuda.synchronize()
    for name in ("fp8", "bf16", "scale", "amax", "err_sum", "nnz", "mask", "err5_sum", "scale_e8m0", "group_mantissa"):
        a, b = getattr(ref, name), getattr(got, name)
        if a is None:
            continue
        # bit patterns, so that equal NaNs / infinities compare equal
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"{name} differs ({gran}, {scope}, {crit}, {scaling}, {rows}x{cols})"
    return ref


CASES = [
    # (gran, scope, crit, scaling): each uses the scratch for something else
    ("tensor", "partition", "mean_rel_err", "fp32_amax"),        # amax / error partials of the two-pass per-tensor path
    ("tensor", "partition", "e4m3_vs_e5m2", "gam"),
    ("block128", "tensor", "mean_rel_err", "gam"),                # pre-pass partials, group mantissas, tensor-level sums
    ("sub1x128", "tensor", "e4m3_vs_e5m2", "fp32_amax"),          # tensor-level sums
    ("channel_col", "partition", "mean_rel_err", "fp32_amax"),    # column amax / scales / error partials
]


@pytest.mark.parametrize("gran, scope, crit, scaling", CASES)
def test_two_calls_in_a_row_match_the_workspace_entry_point(gran, scope, crit, scaling):
    print(f"[no-alloc] {gran} {scope} {crit} {scaling}: 512x1024 then 128x256", flush=True)
    big = W.gradient(512, 1024, W.seed_for(4, 7), tiny_half=True)
    r1 = _both(big, gran, scope, crit, 0.045, scaling)
    small = W.activation(128, 256, W.seed_for(2, 7))
    r2 = _both(small, gran, scope, crit, 0.045, scaling)
    # and against the oracle, to the usual bar (the workspace entry point's outputs are the static one's, bit for bit)
    parity.compare(small, gran, scope, crit, 0.045, scaling=scaling, label="no-alloc", gpu=(r2.params, r2))
    parity.compare(big, gran, scope, crit, 0.045, scaling=scaling, label="no-alloc", gpu=(r1.params, r1))


def test_operand_without_scratch_and_oversized_request():
    xb = W.activation(64, 256, W.seed_for(2, 8))
    params = B.make_params(64, 256, "sub1x128")
    assert B.mor_workspace_bytes(params) == 0
    x = parity.to_dev(xb)
    got = B.alloc_outputs(params, x.device, want_bf16=True, bf16_fill=parity.FILL)
    B.mor_analyze_quantize_static(params, x, got)
    torch.cuda.synchronize()
    parity.compare(xb, "sub1x128", label="no-alloc, no scratch", gpu=(params, got))
    # per-channel columns of a large operand need more than the built-in scratch holds: refused, nothing launched
    rows, cols = 8192, 4096
    params = B.make_params(rows, cols, "channel_col")
    assert B.mor_workspace_bytes(params) > B.MOR_STATIC_SCRATCH_BYTES
    x = torch.zeros((rows, cols), dtype=torch.int16, device="cuda")
    out = B.alloc_outputs(params, x.device, want_bf16=False)
    out.mask.fill_(7)
    with pytest.raises(B.MorError) as e:
        B.mor_analyze_quantize_static(params, x, out)
    torch.cuda.synchronize()
    assert e.value.status == 5 and bool((out.mask == 7).all())
