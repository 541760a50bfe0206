"""Seeded synthetic BF16 operands shaped like transformer-training GEMM operands.

This module only draws random numbers and rounds them to BF16 bit patterns.  It
holds none of the method's arithmetic (no amax, scale, FP8 conversion, error
metric or selection) and imports neither the HIP binding nor the CPU oracle, so
the tests and the benchmark can feed exactly the same bits to both.

The paper applies MoR to the activation, weight and gradient operands of the
four linear layers of every transformer block (Section 4, first paragraph) of a
model whose tensors are not public; the generators below stand in for those
operands with Llama-style 8B shapes (hidden 4096, ffn 14336, 8192 tokens) and
distributions with outliers, heavy tails, exact zeros and underflowing
sub-channels.

All tensors are returned as C-contiguous ``numpy.uint16`` arrays of BF16 bit
patterns, shape ``(rows, cols)``.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 2_280_400


def seed_for(cfg: int, tensor_idx: int = 0) -> int:
    """Seed of tensor ``tensor_idx`` of workload ``cfg``."""
    return SEED_BASE + 100 * cfg + tensor_idx


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 values to BF16 (round-to-nearest-even), return uint16 bits.

    NaNs are mapped to a quiet NaN with the sign kept.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    out = np.empty(a.shape, dtype=np.uint16)
    # process in slabs to bound temporary memory on big operands
    flat_u = u.reshape(-1)
    flat_o = out.reshape(-1)
    step = 1 << 24
    for i in range(0, flat_u.size, step):
        w = flat_u[i:i + step].astype(np.uint64)
        lsb = (w >> np.uint64(16)) & np.uint64(1)
        r = (w + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
        r = r.astype(np.uint32)
        isnan = (flat_u[i:i + step] & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        if isnan.any():
            r = np.where(isnan, ((flat_u[i:i + step] >> np.uint32(16)) | np.uint32(0x0040)), r)
        flat_o[i:i + step] = r.astype(np.uint16)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of BF16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _normal_f32(rng: np.random.Generator, shape, scale: float = 1.0) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a


def outlier_normal(rows: int, cols: int, seed: int, frac: float = 1e-3, gain: float = 100.0) -> np.ndarray:
    """N(0,1) with a fraction ``frac`` of uniformly placed entries times ``gain`` (random sign)."""
    rng = _rng(seed)
    a = _normal_f32(rng, (rows, cols))
    n = rows * cols
    k = int(round(frac * n))
    if k:
        pos = rng.choice(n, size=k, replace=False)
        sign = rng.integers(0, 2, size=k).astype(np.float32) * 2.0 - 1.0
        flat = a.reshape(-1)
        flat[pos] *= np.float32(gain) * sign
    return f32_to_bf16_bits(a)


def activation(rows: int, cols: int, seed: int, n_outlier_channels: int = 4, gain: float = 50.0) -> np.ndarray:
    """tokens x hidden activations: N(0,1) times a per-channel log-normal(0,1) scale,
    with ``n_outlier_channels`` random channels additionally scaled by ``gain``."""
    rng = _rng(seed)
    a = _normal_f32(rng, (rows, cols))
    ch = np.exp(rng.standard_normal(size=cols)).astype(np.float32)
    hot = rng.choice(cols, size=min(n_outlier_channels, cols), replace=False)
    ch[hot] *= np.float32(gain)
    a *= ch[None, :]
    return f32_to_bf16_bits(a)


def weight(rows: int, cols: int, seed: int, std: float = 0.02, spike_frac: float = 1e-4) -> np.ndarray:
    """N(0, std) weights with a fraction ``spike_frac`` of entries replaced by N(0,1) spikes."""
    rng = _rng(seed)
    a = _normal_f32(rng, (rows, cols), std)
    n = rows * cols
    k = int(round(spike_frac * n))
    if k:
        pos = rng.choice(n, size=k, replace=False)
        a.reshape(-1)[pos] = rng.standard_normal(size=k).astype(np.float32)
    return f32_to_bf16_bits(a)


def gradient(rows: int, cols: int, seed: int, nu: float = 3.0, scale: float = 1e-4,
             zero_frac: float = 0.05, tiny_frac: float = 0.10, tiny_gain: float = 1e-6,
             tiny_half: bool = False) -> np.ndarray:
    """Heavy-tailed gradients: Student-t(nu) times ``scale``, ``zero_frac`` exact zeros, and a
    fraction ``tiny_frac`` of the 1x128 sub-channels (drawn once per tensor) scaled by
    ``tiny_gain`` so that, under coarser scaling, they land near or below the smallest E4M3
    subnormal.  With ``tiny_half`` only a random half of each chosen sub-channel is shrunk,
    which makes those sub-channels fall back even at 1x128 granularity (a mixed mask)."""
    if cols % 128:
        raise ValueError("gradient(): cols must be a multiple of 128")
    rng = _rng(seed)
    a = np.empty((rows, cols), dtype=np.float32)
    slab = max(1, (1 << 24) // cols)
    for r0 in range(0, rows, slab):
        r1 = min(rows, r0 + slab)
        a[r0:r1] = rng.standard_t(nu, size=(r1 - r0, cols)).astype(np.float32)
    a *= np.float32(scale)
    zero = rng.random(size=(rows, cols), dtype=np.float32) < np.float32(zero_frac)
    a[zero] = 0.0
    del zero
    nsub = rows * (cols // 128)
    tiny = rng.random(size=nsub) < tiny_frac
    g = np.ones((nsub, 1), dtype=np.float32)
    g[tiny] = np.float32(tiny_gain)
    v = a.reshape(nsub, 128)
    if tiny_half:
        half = rng.random(size=(nsub, 128), dtype=np.float32) < np.float32(0.5)
        gm = np.where(half & tiny[:, None], np.float32(tiny_gain), np.float32(1.0))
        v *= gm
    else:
        v *= g
    return f32_to_bf16_bits(a)


# --------------------------------------------------------------------------------------
# The five workloads.  Granularity / scope names are plain strings here so that this module
# needs no knowledge of the library's enums: "tensor", "sub1x128", "block128".
# --------------------------------------------------------------------------------------

def cfg1():
    """Single 1024x1024 tensor, per-tensor and 128x128-block granularity."""
    x = outlier_normal(1024, 1024, seed_for(1))
    return [("x_1024", x, "tensor"), ("x_1024", x, "block128")]


def cfg2(rows: int = 8192, cols: int = 4096):
    """Activation operand, 1x128 sub-channels along the hidden dimension."""
    return [("act", activation(rows, cols, seed_for(2)), "sub1x128")]


def cfg3(rows: int = 14336, cols: int = 4096):
    """Weight operand, 128x128 blocks; also per-tensor on the same data."""
    w = weight(rows, cols, seed_for(3))
    return [("weight", w, "block128"), ("weight", w, "tensor")]


def cfg4(rows: int = 8192, cols: int = 14336, tiny_half: bool = False):
    """Gradient operand, 1x128 and 128x128 partitions on the same tensor."""
    g = gradient(rows, cols, seed_for(4, 1 if tiny_half else 0), tiny_half=tiny_half)
    return [("grad", g, "sub1x128"), ("grad", g, "block128")]


LAYER_SWEEP = (
    # name,      rows,  cols,  kind,        granularity
    ("X",        8192,  4096,  "act",       "sub1x128"),
    ("W_qkv",    6144,  4096,  "weight",    "block128"),
    ("W_o",      4096,  4096,  "weight",    "block128"),
    ("W_gate",   14336, 4096,  "weight",    "block128"),
    ("W_up",     14336, 4096,  "weight",    "block128"),
    ("W_down",   4096,  14336, "weight",    "block128"),
    ("dX",       8192,  4096,  "grad",      "tensor"),
    ("dW_qkv",   6144,  4096,  "grad",      "tensor"),
    ("dW_o",     4096,  4096,  "grad",      "tensor"),
    ("dW_gate",  14336, 4096,  "grad",      "tensor"),
    ("dW_up",    14336, 4096,  "grad",      "tensor"),
    ("dW_down",  4096,  14336, "grad",      "tensor"),
)


def cfg5(row_div: int = 1):
    """Operand sweep of one Llama-style layer (hidden 4096, ffn 14336, 8192 tokens): the
    activation, the five weights and one same-shape gradient per listed operand, with mixed
    granularity (activations 1x128, weights 128x128, gradients per-tensor).

    ``row_div`` > 1 divides every row count (kept a multiple of 128) for reduced-size tests.
    """
    out = []
    for i, (name, rows, cols, kind, gran) in enumerate(LAYER_SWEEP):
        r = max(128, (rows // row_div) // 128 * 128)
        seed = seed_for(5, i)
        if kind == "act":
            t = activation(r, cols, seed)
        elif kind == "weight":
            t = weight(r, cols, seed)
        else:
            t = gradient(r, cols, seed)
        out.append((name, t, gran))
    return out
