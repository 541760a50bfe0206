"""ctypes front end of the CPU oracle (``mor_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this module.  It never touches the HIP library and the HIP binding never
touches it.  Argument marshalling only: all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mor_oracle.c")
_LIB = os.path.join(_HERE, "libmor_oracle.so")

GRAN = {"tensor": 0, "sub1x128": 1, "block128": 2, "channel_row": 3, "channel_col": 4, "sub128x1": 5, "block64": 6}
FORMATS = {"e4m3|bf16": 1 | 4, "e4m3|e5m2|bf16": 1 | 2 | 4}
CRIT = {"mean_rel_err": 0, "e4m3_vs_e5m2": 1}
SCOPE = {"partition": 0, "tensor": 1}
SCALING = {"fp32_amax": 0, "gam": 1, "e8m0": 2}


_SANITIZE = os.environ.get("MOR_ORACLE_SANITIZE", "") not in ("", "0")
if _SANITIZE:
    # host-only checking build (AddressSanitizer + UndefinedBehaviorSanitizer, any finding aborts): run the CPU tests as
    #   MOR_ORACLE_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
    #       python -m pytest tests -m "not gpu" -q
    _LIB = os.path.join(_HERE, "libmor_oracle_san.so")


_PREBUILT = os.environ.get("MOR_ORACLE_LIB")      # a library built elsewhere from (a variant of) mor_oracle.c: mutation runs of the pins
if _PREBUILT:
    _LIB = _PREBUILT


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if _PREBUILT:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        if _SANITIZE:
            cmd[2:3] = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Stats(C.Structure):
    _fields_ = [("n_part", C.c_uint64), ("n_fp8_part", C.c_uint64), ("n_bf16_part", C.c_uint64),
                ("n_elem_fp8", C.c_uint64), ("n_elem_bf16", C.c_uint64), ("nnz_total", C.c_uint64),
                ("n_near_threshold", C.c_uint64),
                ("err_sum_total", C.c_double), ("mean_err", C.c_double),
                ("hist", C.c_uint32 * 12), ("pad_", C.c_uint32),
                ("n_e5m2_part", C.c_uint64), ("n_elem_e5m2", C.c_uint64)]


class _Params(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("gran", C.c_int32), ("scope", C.c_int32), ("crit", C.c_int32), ("scaling", C.c_int32),
                ("formats", C.c_uint32), ("ragged", C.c_int32), ("threshold", C.c_float), ("group_rows", C.c_int32)]


class _Out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("fp8", "bf16", "scale", "amax", "err_sum", "nnz", "mask", "err5_sum",
                                          "err_sum_unscaled", "e8m0", "group_mantissa", "amin", "fake")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.mor_oracle_e4m3_encode.argtypes = [C.c_float]; L.mor_oracle_e4m3_encode.restype = C.c_uint8
        L.mor_oracle_e5m2_encode.argtypes = [C.c_float]; L.mor_oracle_e5m2_encode.restype = C.c_uint8
        L.mor_oracle_e4m3_decode.argtypes = [C.c_uint8]; L.mor_oracle_e4m3_decode.restype = C.c_double
        L.mor_oracle_e5m2_decode.argtypes = [C.c_uint8]; L.mor_oracle_e5m2_decode.restype = C.c_double
        L.mor_oracle_f32_to_bf16.argtypes = [C.c_float]; L.mor_oracle_f32_to_bf16.restype = C.c_uint16
        L.mor_oracle_scale.argtypes = [C.c_float, C.c_float]; L.mor_oracle_scale.restype = C.c_float
        L.mor_oracle_num_partitions.argtypes = [C.c_int, C.c_int64, C.c_int64]
        L.mor_oracle_num_partitions.restype = C.c_int64
        L.mor_oracle_num_partitions_ex.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int]
        L.mor_oracle_num_partitions_ex.restype = C.c_int64
        L.mor_oracle_run.argtypes = [C.POINTER(_Params), C.c_void_p, C.POINTER(_Out)]
        L.mor_oracle_run.restype = C.c_int
        L.mor_oracle_dequantize_ex.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]
        L.mor_oracle_dequantize_ex.restype = C.c_int
        L.mor_oracle_select_stats_ex.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                                 C.c_int, C.c_int, C.c_float, C.c_float, C.POINTER(_Stats)]
        L.mor_oracle_select_stats_ex.restype = C.c_int
        L.mor_oracle_histogram_update.argtypes = [C.c_void_p, C.c_float, C.c_int64, C.c_int64]
        L.mor_oracle_histogram_update.restype = None
        L.mor_oracle_analyze_quantize.argtypes = [
            C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_float,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p]
        L.mor_oracle_analyze_quantize.restype = C.c_int
        L.mor_oracle_analyze_quantize_ex.argtypes = [
            C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.mor_oracle_analyze_quantize_ex.restype = C.c_int
        L.mor_oracle_group_mantissa.argtypes = [C.c_float, C.c_float, C.c_int]
        L.mor_oracle_group_mantissa.restype = C.c_double
        L.mor_oracle_gam_block_scale.argtypes = [C.c_float, C.c_float, C.c_double, C.POINTER(C.c_int)]
        L.mor_oracle_gam_block_scale.restype = C.c_float
        L.mor_oracle_dequantize.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int64, C.c_int64, C.c_int, C.c_void_p]
        L.mor_oracle_dequantize.restype = C.c_int
        L.mor_oracle_select_stats.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                              C.c_int, C.c_float, C.c_float, C.POINTER(_Stats)]
        L.mor_oracle_select_stats.restype = C.c_int
        L.mor_oracle_threads.restype = C.c_int
        L.mor_oracle_set_threads.argtypes = [C.c_int]
        L.mor_oracle_set_threads.restype = None
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def e4m3_encode(y: float) -> int:
    return int(lib().mor_oracle_e4m3_encode(float(np.float32(y))))


def e5m2_encode(y: float) -> int:
    return int(lib().mor_oracle_e5m2_encode(float(np.float32(y))))


def e4m3_decode(code: int) -> float:
    return float(lib().mor_oracle_e4m3_decode(int(code)))


def e5m2_decode(code: int) -> float:
    return float(lib().mor_oracle_e5m2_decode(int(code)))


def e4m3_encode_array(y: np.ndarray) -> np.ndarray:
    f = lib().mor_oracle_e4m3_encode
    y = np.asarray(y, dtype=np.float32)
    return np.fromiter((f(float(v)) for v in y.reshape(-1)), dtype=np.uint8, count=y.size).reshape(y.shape)


def e5m2_encode_array(y: np.ndarray) -> np.ndarray:
    f = lib().mor_oracle_e5m2_encode
    y = np.asarray(y, dtype=np.float32)
    return np.fromiter((f(float(v)) for v in y.reshape(-1)), dtype=np.uint8, count=y.size).reshape(y.shape)


def f32_to_bf16(v: float) -> int:
    return int(lib().mor_oracle_f32_to_bf16(float(np.float32(v))))


def scale(amax: float, q_amax: float = 448.0) -> float:
    return float(lib().mor_oracle_scale(float(np.float32(amax)), float(q_amax)))


def group_mantissa(g_amax: float, q_amax: float = 448.0, scaling: str = "gam") -> float:
    """m_g of Algorithm 1 as a number in [1, 2)."""
    return float(lib().mor_oracle_group_mantissa(float(np.float32(g_amax)), float(q_amax), SCALING[scaling]))


def gam_block_scale(b_amax: float, m_g: float, q_amax: float = 448.0) -> tuple[float, int]:
    """Applied scale m_g * 2^e and the exponent e of one block (Algorithm 1, block loop)."""
    e = C.c_int(0)
    s = lib().mor_oracle_gam_block_scale(float(np.float32(b_amax)), float(q_amax), float(m_g), C.byref(e))
    return float(s), int(e.value)


def num_partitions(gran: str, rows: int, cols: int, ragged: bool = False) -> int:
    return int(lib().mor_oracle_num_partitions_ex(GRAN[gran], rows, cols, 1 if ragged else 0))


def threads() -> int:
    return int(lib().mor_oracle_threads())


def set_threads(n: int) -> None:
    lib().mor_oracle_set_threads(int(n))


@dataclass
class Analysis:
    fp8: np.ndarray            # (rows, cols) uint8: E4M3 codes of every block, E5M2 codes where mask == 2
    bf16: np.ndarray           # (rows, cols) uint16, input bits where mask == 1, `fill` elsewhere
    scale: np.ndarray          # (P,) float32: scale of the payload in fp8
    amax: np.ndarray           # (P,) float32
    err_sum: np.ndarray        # (P,) float64
    nnz: np.ndarray            # (P,) uint32
    mask: np.ndarray           # (P,) uint8, 0 = E4M3, 1 = BF16, 2 = E5M2
    err5_sum: np.ndarray       # (P,) float64 (zeros unless criterion is e4m3_vs_e5m2)
    err_sum_unscaled: np.ndarray  # (P,) float64, Eq. (2) evaluated in the unscaled domain
    e8m0: np.ndarray | None = None          # (P,) uint8 block exponents + 127 (GAM / E8M0 scaling)
    group_mantissa: int | None = None       # 23 fraction bits of m_g (GAM / E8M0 scaling) of the first (or only) group
    group_mantissa5: int | None = None      # the same for the E5M2 scales
    amin: np.ndarray | None = None          # (P,) float32 smallest non-zero magnitude (0 if none)
    fake: np.ndarray | None = None          # (rows, cols) uint16 fake-quantized tensor, on request
    group_mantissas: np.ndarray | None = None   # (n_groups, 2) uint32: fraction bits of m_g for E4M3 / E5M2, for every group of Algorithm 1

    def metric(self) -> np.ndarray:
        n = self.nnz.astype(np.float64)
        with np.errstate(invalid="ignore", divide="ignore"):
            return np.where(n > 0, self.err_sum / np.maximum(n, 1), 0.0)


def analyze_quantize(x: np.ndarray, gran: str, scope: str = "partition", crit: str = "mean_rel_err",
                     threshold: float = 0.045, bf16_fill: int = 0, ld: int | None = None,
                     cols: int | None = None, scaling: str = "fp32_amax", formats: str = "e4m3|bf16",
                     ragged: bool = False, want_fake: bool = False, gam_group_rows: int = 0) -> Analysis:
    """Run the oracle on BF16 bit patterns ``x`` (2-D uint16).  ``ld``/``cols`` allow a padded
    leading dimension: ``x`` is then (rows, ld) and only the first ``cols`` columns are used."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    rows = x.shape[0]
    ld = x.shape[1] if ld is None else ld
    cols = x.shape[1] if cols is None else cols
    P = num_partitions(gran, rows, cols, ragged)
    if P < 0:
        raise ValueError(f"bad shape {rows}x{cols} for granularity {gran}")
    fp8 = np.zeros((rows, cols), np.uint8)
    bf16 = np.full((rows, cols), bf16_fill, np.uint16)
    sc = np.zeros(P, np.float32); am = np.zeros(P, np.float32); mn = np.zeros(P, np.float32)
    es = np.zeros(P, np.float64); e5 = np.zeros(P, np.float64); eu = np.zeros(P, np.float64)
    nz = np.zeros(P, np.uint32); mk = np.zeros(P, np.uint8)
    ex = np.zeros(P, np.uint8)
    n_groups = -(-rows // gam_group_rows) if (gam_group_rows and scaling == "gam") else 1
    gm = np.zeros(2 * n_groups, np.uint32)
    fake = np.zeros((rows, cols), np.uint16) if want_fake else None
    pp = _Params(rows, cols, ld, GRAN[gran], SCOPE[scope], CRIT[crit], SCALING[scaling], FORMATS[formats],
                 1 if ragged else 0, float(np.float32(threshold)), int(gam_group_rows))
    oo = _Out(*[None if a is None else a.ctypes.data for a in (fp8, bf16, sc, am, es, nz, mk, e5, eu, ex, gm, mn, fake)])
    rc = lib().mor_oracle_run(C.byref(pp), _p(x), C.byref(oo))
    if rc != 0:
        raise ValueError("mor_oracle_run rejected the arguments")
    if scaling == "fp32_amax":
        return Analysis(fp8, bf16, sc, am, es, nz, mk, e5, eu, amin=mn, fake=fake)
    return Analysis(fp8, bf16, sc, am, es, nz, mk, e5, eu, ex, int(gm[0]), int(gm[1]), mn, fake, gm.reshape(n_groups, 2))


def dequantize(fp8: np.ndarray, scale_: np.ndarray, mask: np.ndarray, bf16: np.ndarray | None,
               gran: str, fill: int = 0, ragged: bool = False) -> np.ndarray:
    fp8 = np.ascontiguousarray(fp8, dtype=np.uint8)
    rows, cols = fp8.shape
    y = np.full((rows, cols), fill, np.uint16)
    scale_ = np.ascontiguousarray(scale_, np.float32)
    mask = np.ascontiguousarray(mask, np.uint8)
    if bf16 is not None:
        bf16 = np.ascontiguousarray(bf16, np.uint16)
    rc = lib().mor_oracle_dequantize_ex(_p(fp8), _p(scale_), _p(mask), _p(bf16), rows, cols, GRAN[gran],
                                        1 if ragged else 0, _p(y))
    if rc != 0:
        raise ValueError("mor_oracle_dequantize rejected the arguments")
    return y


def select_stats(err_sum: np.ndarray, nnz: np.ndarray, mask: np.ndarray, rows: int, cols: int, gran: str,
                 threshold: float = 0.045, near_tol: float = 1e-5, ragged: bool = False) -> dict:
    err_sum = np.ascontiguousarray(err_sum, np.float32)
    nnz = np.ascontiguousarray(nnz, np.uint32)
    mask = np.ascontiguousarray(mask, np.uint8)
    st = _Stats()
    rc = lib().mor_oracle_select_stats_ex(_p(err_sum), _p(nnz), _p(mask), rows, cols, GRAN[gran], 1 if ragged else 0,
                                          float(np.float32(threshold)), float(np.float32(near_tol)), C.byref(st))
    if rc != 0:
        raise ValueError("mor_oracle_select_stats rejected the arguments")
    d = {k: getattr(st, k) for k, _ in _Stats._fields_ if k not in ("hist", "pad_")}
    d["hist"] = [int(v) for v in st.hist]
    return d


def histogram_update(hist12: np.ndarray, tensor_metric: float, step: int, reset_interval: int) -> None:
    """Running per-tensor histogram over mini-batches (in place; hist12 is uint32[12])."""
    assert hist12.dtype == np.uint32 and hist12.size == 12 and hist12.flags.c_contiguous
    lib().mor_oracle_histogram_update(_p(hist12), float(np.float32(tensor_metric)), int(step), int(reset_interval))


if __name__ == "__main__":
    print(build(force=True))
