"""Test-only third implementation of the analyse-select-quantize definitions in exact rational
arithmetic (``fractions``), for tiny inputs.  Independent of both the C oracle and the HIP path:
it is written directly from the format definitions (Section 1-2 of the paper) and Eq. (1)-(3).
Only the two binary32 roundings the method fixes (scale = fl32(q_amax/amax), y = fl32(x*s)) use
numpy float32 as a library primitive; the de-quantize / de-scale half (Section 4, Figure 4) does every
rounding (binary32 and BF16) in exact rationals."""
from fractions import Fraction
import bisect
import math

import numpy as np


def fp8_values(ebits, mbits):
    """code -> exact value for all non-negative finite codes, from the format definition."""
    bias = 2 ** (ebits - 1) - 1
    vals = {}
    for code in range(128):
        e = code >> mbits
        m = code & (2 ** mbits - 1)
        if ebits == 4 and e == 15 and m == 7:
            continue                      # E4M3: S.1111.111 is NaN, there are no infinities
        if ebits == 5 and e == 31:
            continue                      # E5M2: inf / NaN
        if e == 0:
            v = Fraction(m, 2 ** mbits) * Fraction(2) ** (1 - bias)
        else:
            v = (1 + Fraction(m, 2 ** mbits)) * Fraction(2) ** (e - bias)
        vals[code] = v
    return vals


_TABLES = {}


def _table(ebits, mbits):
    key = (ebits, mbits)
    if key not in _TABLES:
        vals = fp8_values(ebits, mbits)
        codes = sorted(vals, key=lambda c: vals[c])
        _TABLES[key] = (codes, [vals[c] for c in codes])
    return _TABLES[key]


def fp8_encode(y, ebits, mbits):
    """Nearest representable value, ties to the even code, clip beyond the largest finite value."""
    y = float(y)
    sign = 0x80 if math.copysign(1.0, y) < 0 else 0
    if math.isnan(y):
        return sign | 0x7F
    codes, values = _table(ebits, mbits)
    if math.isinf(y):
        return sign | codes[-1]
    a = abs(Fraction(y))
    if a >= values[-1]:
        return sign | codes[-1]
    i = bisect.bisect_right(values, a) - 1          # values[i] <= a < values[i+1]
    dlo, dhi = a - values[i], values[i + 1] - a
    if dlo < dhi:
        pick = codes[i]
    elif dhi < dlo:
        pick = codes[i + 1]
    else:
        pick = codes[i] if codes[i] % 2 == 0 else codes[i + 1]
    return sign | pick


def fp8_decode(code, ebits, mbits):
    codes, values = _table(ebits, mbits)
    v = fp8_values(ebits, mbits)[code & 0x7F]
    return -v if code & 0x80 else v


def bf16_to_f32(b):
    return np.array([int(b) << 16], dtype=np.uint32).view(np.float32)[0]


def scale_of(amax, qmax):
    amax = np.float32(amax)
    if not np.isfinite(amax) or amax == 0:
        return np.float32(1.0)
    with np.errstate(over="ignore"):
        s = np.float32(qmax) / amax
    return np.float32(np.finfo(np.float32).max) if np.isinf(s) else s


def _mant_exp(v):
    """v = m * 2^e with 1 <= m < 2, exactly, for a positive Fraction v."""
    e = 0
    while v >= 2 ** (e + 1):
        e += 1
    while v < Fraction(2) ** e:
        e -= 1
    return v / Fraction(2) ** e, e


def gam_scale(b_amax, g_amax, qmax, e8m0_only=False):
    """Algorithm 1 with one group, in exact rationals: (applied scale, exponent e, m_g)."""
    m_g = Fraction(1) if e8m0_only else _mant_exp(Fraction(float(scale_of(g_amax, qmax))))[0]
    m_b, e = _mant_exp(Fraction(float(scale_of(b_amax, qmax))))
    if m_g > m_b:
        e -= 1
    return m_g * Fraction(2) ** e, e, m_g


def analyze_block(bits, crit="mean_rel_err", threshold=0.045, scaling="fp32_amax", g_amax=None, three_way=False):
    """bits: iterable of BF16 bit patterns of ONE block.  Returns dict with exact-rational sums.
    scaling 'gam' / 'e8m0' take the block's scale from Algorithm 1 (g_amax = amax of the tensor).
    three_way: type list [E4M3, E5M2, BF16] of Section 3.2; out['choice'] is 'e4m3', 'e5m2' or 'bf16'
    and out['codes'] / out['scale'] describe the chosen payload (E4M3's when BF16 is chosen)."""
    bits = [int(b) for b in bits]
    a = max(b & 0x7FFF for b in bits)
    amax = bf16_to_f32(a)
    out = {"amax": float(amax), "nnz": sum(1 for b in bits if b & 0x7FFF)}

    def run(qmax, ebits, mbits):
        if scaling == "fp32_amax":
            s = scale_of(amax, qmax)
        else:
            sf = gam_scale(amax, amax if g_amax is None else g_amax, qmax, scaling == "e8m0")[0]
            s = np.float32(float(sf))
            assert Fraction(float(s)) == sf          # the applied scale is a binary32 number
        codes, total = [], Fraction(0)
        for b in bits:
            with np.errstate(over="ignore", under="ignore", invalid="ignore"):
                y = np.float32(bf16_to_f32(b) * s)
            c = fp8_encode(y, ebits, mbits)
            codes.append(c)
            if b & 0x7FFF == 0:
                continue
            q = fp8_decode(c, ebits, mbits)
            if q == 0:
                total += 1
            else:
                yy = Fraction(float(y))
                total += abs(yy - q) / abs(yy)
        return float(s), codes, total

    s, codes, err = run(448.0, 4, 3)
    out.update(scale=s, codes=codes, err_sum=err)
    if crit == "e4m3_vs_e5m2":
        _, _, err5 = run(57344.0, 5, 2)
        out["err5_sum"] = err5
        out["fp8"] = err < err5
    else:
        metric = err / out["nnz"] if out["nnz"] else Fraction(0)
        out["metric"] = metric
        out["fp8"] = metric < Fraction(float(np.float32(threshold)))
    out["choice"] = "e4m3" if out["fp8"] else "bf16"
    if three_way and not out["fp8"]:
        # Eq. (4): max|b| / min|b| < 57344 / 2^-14 over the non-zero elements, in exact rationals
        mags = [Fraction(float(bf16_to_f32(b & 0x7FFF))) for b in bits if b & 0x7FFF and (b & 0x7FFF) < 0x7F80]
        finite = all((b & 0x7FFF) < 0x7F80 for b in bits)
        fits = finite and (not mags or max(mags) / min(mags) < Fraction(57344) / Fraction(1, 2 ** 14))
        if fits:
            s5, codes5, _ = run(57344.0, 5, 2)
            out.update(choice="e5m2", scale=s5, codes=codes5)
    return out


# ---------------------------------------------------------------- de-quantize / de-scale (Section 4, Figure 4)

def round_to_binary(v, sig_bits, emin, emax):
    """Exact round-to-nearest-even of the rational ``v`` to a binary floating-point grid with ``sig_bits``
    significant bits, smallest normal exponent ``emin`` (values below 2^emin sit on the subnormal grid
    2^(emin - sig_bits + 1)) and largest exponent ``emax`` (beyond it: infinity).  Returns a Fraction, or
    +-math.inf.  Written from the IEEE-754 definition; no floating-point arithmetic is used."""
    v = Fraction(v)
    if v == 0:
        return Fraction(0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    _, e = _mant_exp(a)
    e = max(e, emin)
    ulp = Fraction(2) ** (e - (sig_bits - 1))
    n = a / ulp                                     # position on the grid of this binade
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    r = lo * ulp
    if r >= Fraction(2) ** (emax + 1):
        return sign * math.inf
    return sign * r


def fl32(v):
    """binary32 rounding of a rational."""
    return round_to_binary(v, 24, -126, 127)


def bf16_rne_bits(v):
    """BF16 bit pattern (8 significant bits, binary32's exponent range) of the rational ``v``, round to nearest even.
    ``negative_zero`` cannot be expressed by a Fraction: callers pass the sign separately when v == 0."""
    r = round_to_binary(v, 8, -126, 127)
    if r in (math.inf, -math.inf):
        return 0x7F80 | (0x8000 if r < 0 else 0)
    f = np.float32(float(r))                         # exact: r is on the BF16 grid
    assert Fraction(float(f)) == r
    bits = int(np.array([f], np.float32).view(np.uint32)[0])
    assert bits & 0xFFFF == 0
    return bits >> 16


def dequantize_block(codes, scale, ebits=4, mbits=3):
    """De-quantize and de-scale the FP8 codes of one block: value(code) times fl32(1 / scale), rounded to binary32,
    then to BF16 round-to-nearest-even -- every rounding done in exact rationals.  Returns BF16 bit patterns.
    The sign of a zero result is the sign of the code (a product of a signed zero and a positive number)."""
    s = Fraction(float(np.float32(scale)))
    assert s > 0
    s_inv = fl32(1 / s)
    out = []
    for c in codes:
        q = fp8_decode(int(c), ebits, mbits)
        v = fl32(q * s_inv)
        bits = bf16_rne_bits(v)
        if v == 0 and (int(c) & 0x80):
            bits |= 0x8000
        out.append(bits)
    return out
