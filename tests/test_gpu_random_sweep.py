"""Seeded random sweep over the whole parameter space of the analyse-select-quantize entry points (granularity,
scope, criterion, scaling, GAM groups, type list, ragged shapes, padded leading dimensions, fake quantization): every case is
compared with the CPU oracle to the usual bar.  Small shapes, many combinations."""
import numpy as np
import pytest
import torch

from paper_2512_22804_amd import workloads as W

pytestmark = pytest.mark.gpu

TH = 0.045
GRANS = ["tensor", "sub1x128", "block128", "channel_row", "channel_col", "sub128x1", "block64"]
BLOCK = {"tensor": (1, 8), "sub1x128": (1, 128), "block128": (128, 128), "channel_row": (1, 8), "channel_col": (1, 8),
         "sub128x1": (128, 8), "block64": (64, 64)}


@pytest.fixture(scope="module")
def P():
    import parity
    from paper_2512_22804_amd import binding as B
    B.load()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return parity


def operand(rng, rows, ld):
    """Magnitudes over a few binades per 32-column group, some groups with a tail of tiny values (E4M3 flushes, E5M2
    may hold), some zeros, now and then a very large or a non-finite value."""
    x = rng.standard_normal((rows, ld)).astype(np.float32)
    x *= np.exp2(rng.integers(-6, 6, size=(rows, 1))).astype(np.float32)
    groups = -(-ld // 32)
    kind = np.repeat(rng.integers(0, 4, size=(rows, groups)), 32, axis=1)[:, :ld]
    tail = rng.random((rows, ld)) < 0.4
    x[(kind == 1) & tail] *= np.float32(2.0 ** -21)
    x[(kind == 2) & tail] *= np.float32(2.0 ** -33)
    x[rng.random((rows, ld)) < 0.04] = 0.0
    xb = W.f32_to_bf16_bits(x)
    roll = rng.random()
    if roll < 0.08:
        xb[rng.integers(0, rows), rng.integers(0, ld)] = 0x7F80          # +inf
    elif roll < 0.16:
        xb[rng.integers(0, rows), rng.integers(0, ld)] = 0x7E80          # 2^126: the careful element path
    return xb


@pytest.mark.parametrize("seed", range(420))
def test_random_case(P, seed):
    rng = np.random.default_rng(9000 + seed)
    gran = GRANS[seed % len(GRANS)]
    ragged = bool(rng.integers(0, 2))
    pr, pc = BLOCK[gran]
    if ragged:
        rows = int(rng.integers(1, 330))
        cols = 8 * int(rng.integers(1, 140))
    else:
        rows = pr * int(rng.integers(1, max(2, 330 // pr)))
        cols = pc * int(rng.integers(1, max(2, 1100 // pc)))
    ld = cols + 8 * int(rng.integers(0, 3)) * int(rng.integers(0, 2))
    three = bool(rng.integers(0, 3) == 0)
    scope = "partition" if three or rng.integers(0, 3) else "tensor"
    crit = ("mean_rel_err", "e4m3_vs_e5m2")[int(rng.integers(0, 2))]
    scaling = ("fp32_amax", "gam", "e8m0")[int(rng.integers(0, 3))]
    th = float((0.045, 0.02, 0.2)[int(rng.integers(0, 3))])
    fake = bool(rng.integers(0, 3) == 0)
    xb = operand(rng, rows, ld)
    kw = dict(scope=scope, crit=crit, threshold=th, scaling=scaling, formats="e4m3|e5m2|bf16" if three else "e4m3|bf16",
              ragged=ragged, cols=cols, label=f"sweep-{seed}")
    # GAM: half of the cases take bands of rows as the groups of Algorithm 1 (drawn from a generator of its own, so that the
    # operands of the cases above stay what they were)
    rng_band = np.random.default_rng(77000 + seed)
    if scaling == "gam" and gran in ("sub1x128", "block128", "channel_row", "sub128x1", "block64") and rng_band.integers(0, 2):
        kw["gam_group_rows"] = pr * int(rng_band.integers(1, max(2, rows // pr + 1)))
    if fake:
        P.compare_fake(xb, gran, **kw)
    else:
        P.compare(xb, gran, **kw)
