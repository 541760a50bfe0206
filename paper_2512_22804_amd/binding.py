"""Thin ctypes binding of ``libmor.so`` (the C ABI declared in ``include/mor.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch is used for
device memory and the current stream, nothing else.  There is no CPU fallback: if the library is
missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MOR_LIB_PATH", os.path.join(_HERE, "libmor.so"))

MOR_GRAN_TENSOR, MOR_GRAN_SUB_1x128, MOR_GRAN_BLOCK_128x128 = 0, 1, 2
MOR_GRAN_CHANNEL_ROW, MOR_GRAN_CHANNEL_COL, MOR_GRAN_SUB_128x1, MOR_GRAN_BLOCK_64x64 = 3, 4, 5, 6
MOR_FMT_E4M3, MOR_FMT_E5M2, MOR_FMT_BF16 = 1, 2, 4
MOR_FLAG_RAGGED = 1
MOR_FLAG_LEAN_FP8 = 2
MOR_CRIT_MEAN_REL_ERR, MOR_CRIT_E4M3_VS_E5M2 = 0, 1
MOR_SCOPE_PARTITION, MOR_SCOPE_TENSOR = 0, 1
MOR_SCALE_FP32_AMAX, MOR_SCALE_GAM, MOR_SCALE_E8M0 = 0, 1, 2

GRAN = {"tensor": MOR_GRAN_TENSOR, "sub1x128": MOR_GRAN_SUB_1x128, "block128": MOR_GRAN_BLOCK_128x128,
        "channel_row": MOR_GRAN_CHANNEL_ROW, "channel_col": MOR_GRAN_CHANNEL_COL, "sub128x1": MOR_GRAN_SUB_128x1,
        "block64": MOR_GRAN_BLOCK_64x64}
FORMATS = {"e4m3|bf16": MOR_FMT_E4M3 | MOR_FMT_BF16, "e4m3|e5m2|bf16": MOR_FMT_E4M3 | MOR_FMT_E5M2 | MOR_FMT_BF16}
CRIT = {"mean_rel_err": MOR_CRIT_MEAN_REL_ERR, "e4m3_vs_e5m2": MOR_CRIT_E4M3_VS_E5M2}
SCOPE = {"partition": MOR_SCOPE_PARTITION, "tensor": MOR_SCOPE_TENSOR}
SCALING = {"fp32_amax": MOR_SCALE_FP32_AMAX, "gam": MOR_SCALE_GAM, "e8m0": MOR_SCALE_E8M0}

EXPORTS = ("mor_num_partitions", "mor_params_num_partitions", "mor_workspace_bytes", "mor_analyze_quantize",
           "mor_analyze_quantize_static",
           "mor_analyze_quantize_profiled", "mor_batch_workspace_bytes", "mor_analyze_quantize_batch", "mor_fake_quantize",
           "mor_dequantize", "mor_dequantize_e8m0", "mor_dequantize_batch", "mor_select_stats", "mor_histogram_update", "mor_status_string")
MOR_BATCH_MAX = 64
MOR_PROFILE_MAX = 16
MOR_STATS_FLAG_FUSED_FALLBACK = 1

KERNEL_NAMES = {1: "sub1x128", 2: "block128", 3: "tensor_amax", 4: "tensor_quant", 5: "tensor_finalize",
                6: "fallback_copy", 7: "scope_reduce", 8: "scope_decide", 9: "scope_fill_mask",
                10: "stats_partial", 11: "stats_final", 12: "group_amax", 13: "group_mantissa", 14: "team_block",
                15: "column_tile", 16: "column_combine"}


class MorParams(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("granularity", C.c_int32), ("scope", C.c_int32), ("criterion", C.c_int32), ("scaling", C.c_int32),
                ("formats", C.c_uint32), ("threshold", C.c_float), ("flags", C.c_uint32), ("gam_group_rows", C.c_uint32)]


class MorOutputs(C.Structure):
    _fields_ = [("fp8", C.c_void_p), ("ld_fp8", C.c_int64), ("bf16", C.c_void_p), ("ld_bf16", C.c_int64),
                ("scale", C.c_void_p), ("amax", C.c_void_p), ("err_sum", C.c_void_p), ("nnz", C.c_void_p),
                ("mask", C.c_void_p), ("err5_sum", C.c_void_p), ("scale_e8m0", C.c_void_p), ("group_mantissa", C.c_void_p),
                ("amin", C.c_void_p)]


class MorStats(C.Structure):
    _fields_ = [("n_part", C.c_uint64), ("n_fp8_part", C.c_uint64), ("n_bf16_part", C.c_uint64),
                ("n_elem_fp8", C.c_uint64), ("n_elem_bf16", C.c_uint64), ("nnz_total", C.c_uint64),
                ("n_near_threshold", C.c_uint64), ("err_sum_total", C.c_double), ("mean_err", C.c_double),
                ("hist", C.c_uint32 * 12), ("flags", C.c_uint32), ("reserved", C.c_uint32),
                ("n_e5m2_part", C.c_uint64), ("n_elem_e5m2", C.c_uint64)]


STATS_BYTES = C.sizeof(MorStats)     # 144


class MorProfile(C.Structure):
    _fields_ = [("capacity", C.c_int32), ("count", C.c_int32), ("start", C.c_void_p * MOR_PROFILE_MAX),
                ("stop", C.c_void_p * MOR_PROFILE_MAX), ("kernel", C.c_int32 * MOR_PROFILE_MAX)]


class MorBatchItem(C.Structure):
    _fields_ = [("params", MorParams), ("x", C.c_void_p), ("out", MorOutputs), ("stats", C.c_void_p),
                ("fake_y", C.c_void_p), ("ld_fake_y", C.c_int64)]


class MorDequantItem(C.Structure):
    _fields_ = [("params", MorParams), ("fp8", C.c_void_p), ("ld_fp8", C.c_int64), ("scale", C.c_void_p),
                ("scale_e8m0", C.c_void_p), ("group_mantissa", C.c_void_p), ("mask", C.c_void_p), ("bf16", C.c_void_p),
                ("ld_bf16", C.c_int64), ("y", C.c_void_p), ("ld_y", C.c_int64)]


class MorError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = load().mor_status_string(self.status).decode()
        super().__init__(f"{where}: {msg} (status {self.status})")


_lib = None


def load():
    """Load libmor.so (built in-tree by ``paper_2512_22804_amd.build``).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2512_22804_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.mor_num_partitions.argtypes = [C.c_int32, C.c_int64, C.c_int64]
        L.mor_num_partitions.restype = C.c_int64
        L.mor_params_num_partitions.argtypes = [C.POINTER(MorParams)]
        L.mor_params_num_partitions.restype = C.c_int64
        L.mor_fake_quantize.argtypes = [C.POINTER(MorParams), C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(MorOutputs), C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        L.mor_fake_quantize.restype = C.c_int
        L.mor_histogram_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p]
        L.mor_histogram_update.restype = C.c_int
        L.mor_workspace_bytes.argtypes = [C.POINTER(MorParams)]
        L.mor_workspace_bytes.restype = C.c_size_t
        L.mor_analyze_quantize.argtypes = [C.POINTER(MorParams), C.c_void_p, C.POINTER(MorOutputs), C.c_void_p,
                                           C.c_size_t, C.c_void_p]
        L.mor_analyze_quantize.restype = C.c_int
        L.mor_analyze_quantize_static.argtypes = [C.POINTER(MorParams), C.c_void_p, C.POINTER(MorOutputs), C.c_void_p]
        L.mor_analyze_quantize_static.restype = C.c_int
        L.mor_analyze_quantize_profiled.argtypes = [C.POINTER(MorParams), C.c_void_p, C.POINTER(MorOutputs), C.c_void_p,
                                                    C.c_size_t, C.c_void_p, C.POINTER(MorProfile)]
        L.mor_analyze_quantize_profiled.restype = C.c_int
        L.mor_batch_workspace_bytes.argtypes = [C.POINTER(MorBatchItem), C.c_int32]
        L.mor_batch_workspace_bytes.restype = C.c_size_t
        L.mor_analyze_quantize_batch.argtypes = [C.POINTER(MorBatchItem), C.c_int32, C.c_float, C.c_void_p, C.c_size_t,
                                                 C.c_void_p, C.POINTER(MorProfile)]
        L.mor_analyze_quantize_batch.restype = C.c_int
        L.mor_dequantize.argtypes = [C.POINTER(MorParams), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
        L.mor_dequantize.restype = C.c_int
        L.mor_dequantize_e8m0.argtypes = [C.POINTER(MorParams), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
        L.mor_dequantize_e8m0.restype = C.c_int
        L.mor_dequantize_batch.argtypes = [C.POINTER(MorDequantItem), C.c_int32, C.c_void_p]
        L.mor_dequantize_batch.restype = C.c_int
        L.mor_select_stats.argtypes = [C.POINTER(MorParams), C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p,
                                       C.c_void_p]
        L.mor_select_stats.restype = C.c_int
        L.mor_status_string.argtypes = [C.c_int]
        L.mor_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def make_params(rows: int, cols: int, gran: str | int, scope: str | int = "partition", crit: str | int = "mean_rel_err",
                threshold: float = 0.045, ld: int | None = None, formats: int | str = MOR_FMT_E4M3 | MOR_FMT_BF16,
                scaling: str | int = MOR_SCALE_FP32_AMAX, ragged: bool = False, lean_fp8: bool = False,
                gam_group_rows: int = 0) -> MorParams:
    g = GRAN[gran] if isinstance(gran, str) else gran
    s = SCOPE[scope] if isinstance(scope, str) else scope
    c = CRIT[crit] if isinstance(crit, str) else crit
    sc = SCALING[scaling] if isinstance(scaling, str) else scaling
    f = FORMATS[formats] if isinstance(formats, str) else formats
    return MorParams(rows, cols, cols if ld is None else ld, g, s, c, sc, f, threshold,
                     (MOR_FLAG_RAGGED if ragged else 0) | (MOR_FLAG_LEAN_FP8 if lean_fp8 else 0), int(gam_group_rows))


def mor_num_partitions(gran: str | int, rows: int, cols: int) -> int:
    g = GRAN[gran] if isinstance(gran, str) else gran
    return int(load().mor_num_partitions(g, rows, cols))


def mor_params_num_partitions(params: MorParams) -> int:
    return int(load().mor_params_num_partitions(C.byref(params)))


def mor_workspace_bytes(params: MorParams) -> int:
    return int(load().mor_workspace_bytes(C.byref(params)))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class MorResult:
    """Device buffers written by :func:`mor_analyze_quantize`."""
    fp8: torch.Tensor        # (rows, ld_fp8) uint8 E4M3 codes
    bf16: torch.Tensor | None  # (rows, ld_bf16) int16 BF16 bits, written only where mask == 1
    scale: torch.Tensor      # (P,) float32
    amax: torch.Tensor       # (P,) float32
    err_sum: torch.Tensor    # (P,) float32
    nnz: torch.Tensor        # (P,) int32 (bit pattern of uint32)
    mask: torch.Tensor       # (P,) uint8
    err5_sum: torch.Tensor | None
    workspace: torch.Tensor | None
    params: MorParams
    scale_e8m0: torch.Tensor | None = None      # (P,) uint8, GAM / E8M0 scaling only
    group_mantissa: torch.Tensor | None = None  # (2 * n_groups,) int32, GAM / E8M0 scaling only: per group E4M3's, E5M2's
    amin: torch.Tensor | None = None            # (P,) float32, three-way recipe only


def gam_groups(params: MorParams) -> int:
    """Number of groups of Algorithm 1 for these parameters (1 unless GAM scaling with bands of rows as groups)."""
    if params.scaling != MOR_SCALE_GAM or params.gam_group_rows == 0 or params.gam_group_rows >= params.rows:
        return 1
    return -(-params.rows // params.gam_group_rows)


def alloc_outputs(params: MorParams, device, want_bf16: bool = True, bf16_fill: int | None = None,
                  want_fp8: bool = True) -> MorResult:
    """Allocate the output buffers of one call (dense leading dimensions)."""
    rows, cols = params.rows, params.cols
    P = mor_params_num_partitions(params)
    if P < 0:
        raise MorError(2, "alloc_outputs")
    fp8 = torch.empty((rows, cols), dtype=torch.uint8, device=device) if want_fp8 else None
    bf16 = None
    if want_bf16:
        bf16 = (torch.empty((rows, cols), dtype=torch.int16, device=device) if bf16_fill is None else
                torch.full((rows, cols), bf16_fill if bf16_fill < 0x8000 else bf16_fill - 0x10000, dtype=torch.int16, device=device))
    f32 = lambda: torch.empty(P, dtype=torch.float32, device=device)
    err5 = f32() if params.criterion == MOR_CRIT_E4M3_VS_E5M2 else None
    nbytes = mor_workspace_bytes(params)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None
    e8m0 = gmant = None
    if params.scaling != MOR_SCALE_FP32_AMAX:
        e8m0 = torch.full((P,), 0xEE, dtype=torch.uint8, device=device)
        gmant = torch.full((2 * gam_groups(params),), -1, dtype=torch.int32, device=device)
    amin = torch.full((P,), -1.0, dtype=torch.float32, device=device) if params.formats & MOR_FMT_E5M2 else None
    return MorResult(fp8, bf16, f32(), f32(), f32(), torch.empty(P, dtype=torch.int32, device=device),
                     torch.empty(P, dtype=torch.uint8, device=device), err5, ws, params, e8m0, gmant, amin)


def _outputs_struct(out: MorResult) -> MorOutputs:
    return MorOutputs(_ptr(out.fp8), out.fp8.stride(0) if out.fp8 is not None else 0, _ptr(out.bf16),
                      out.bf16.stride(0) if out.bf16 is not None else 0,
                      _ptr(out.scale), _ptr(out.amax), _ptr(out.err_sum), _ptr(out.nnz), _ptr(out.mask), _ptr(out.err5_sum),
                      _ptr(out.scale_e8m0), _ptr(out.group_mantissa), _ptr(out.amin))


def mor_analyze_quantize(params: MorParams, x: torch.Tensor, out: MorResult) -> None:
    """Enqueue the analyse-select-quantize pass of ``x`` (int16/bfloat16 device tensor holding BF16 bits,
    row stride ``params.ld``) on the current stream, writing into ``out``."""
    if not x.is_cuda:
        raise ValueError("x must live in device memory")
    o = _outputs_struct(out)
    ws = out.workspace
    rc = load().mor_analyze_quantize(C.byref(params), _ptr(x), C.byref(o), _ptr(ws), ws.numel() if ws is not None else 0,
                                     _stream())
    if rc != 0:
        raise MorError(rc, "mor_analyze_quantize")


MOR_STATIC_SCRATCH_BYTES = 1 << 20


def mor_analyze_quantize_static(params: MorParams, x: torch.Tensor, out: MorResult) -> None:
    """The same call on the library's built-in scratch (``out.workspace`` is not used; nothing is allocated)."""
    if not x.is_cuda:
        raise ValueError("x must live in device memory")
    o = _outputs_struct(out)
    rc = load().mor_analyze_quantize_static(C.byref(params), _ptr(x), C.byref(o), _stream())
    if rc != 0:
        raise MorError(rc, "mor_analyze_quantize_static")


def mor_analyze_quantize_profiled(params: MorParams, x: torch.Tensor, out: MorResult, profile: MorProfile) -> None:
    """Same call with the caller's HIP events recorded around each kernel (see :class:`HipEvents`)."""
    if not x.is_cuda:
        raise ValueError("x must live in device memory")
    o = _outputs_struct(out)
    ws = out.workspace
    rc = load().mor_analyze_quantize_profiled(C.byref(params), _ptr(x), C.byref(o), _ptr(ws),
                                              ws.numel() if ws is not None else 0, _stream(), C.byref(profile))
    if rc != 0:
        raise MorError(rc, "mor_analyze_quantize_profiled")


def mor_fake_quantize(params: MorParams, x: torch.Tensor, y: torch.Tensor, meta: MorResult) -> None:
    """Enqueue the fake-quantization pass: ``y`` (same shape as ``x``, BF16 bits) = de-quantize(quantize(x));
    the [P] arrays of ``meta`` are written as by :func:`mor_analyze_quantize` (its fp8 / bf16 buffers are not used)."""
    if not x.is_cuda or not y.is_cuda:
        raise ValueError("x and y must live in device memory")
    o = _outputs_struct(meta)
    ws = meta.workspace
    rc = load().mor_fake_quantize(C.byref(params), _ptr(x), _ptr(y), y.stride(0), C.byref(o), _ptr(ws),
                                  ws.numel() if ws is not None else 0, _stream())
    if rc != 0:
        raise MorError(rc, "mor_fake_quantize")


def mor_histogram_update(hist12: torch.Tensor, stats_dev: torch.Tensor, step: int, reset_interval: int) -> None:
    """``hist12``: device int32/uint32[12]; ``stats_dev``: device mor_stats of this step's call for the tensor."""
    rc = load().mor_histogram_update(_ptr(hist12), _ptr(stats_dev), step, reset_interval, _stream())
    if rc != 0:
        raise MorError(rc, "mor_histogram_update")


def make_batch(entries) -> "C.Array":
    """entries: sequence of (params, x, out: MorResult, stats: torch.Tensor | None[, fake_y: torch.Tensor | None]).
    Returns the host item array."""
    arr = (MorBatchItem * len(entries))()
    for i, entry in enumerate(entries):
        params, x, out, stats = entry[:4]
        fake_y = entry[4] if len(entry) > 4 else None
        arr[i].params = params
        arr[i].x = x.data_ptr()
        arr[i].out = _outputs_struct(out)
        arr[i].stats = stats.data_ptr() if stats is not None else None
        arr[i].fake_y = fake_y.data_ptr() if fake_y is not None else None
        arr[i].ld_fake_y = fake_y.stride(0) if fake_y is not None else 0
    return arr


def mor_batch_workspace_bytes(items) -> int:
    return int(load().mor_batch_workspace_bytes(items, len(items)))


def mor_analyze_quantize_batch(items, near_tol: float, workspace: torch.Tensor | None, profile: MorProfile | None = None) -> None:
    """Enqueue the analyse-select-quantize pass (and, where an item carries a stats buffer, its selection
    statistics) of every operand in ``items`` (from :func:`make_batch`) on the current stream."""
    rc = load().mor_analyze_quantize_batch(items, len(items), near_tol, _ptr(workspace),
                                           workspace.numel() if workspace is not None else 0, _stream(),
                                           C.byref(profile) if profile is not None else None)
    if rc != 0:
        raise MorError(rc, "mor_analyze_quantize_batch")


class HipEvents:
    """Raw hipEvent_t handles (timing enabled) created through the HIP runtime that PyTorch already loaded; they can
    be recorded by the library on the stream its kernels run on."""

    def __init__(self):
        self.rt = C.CDLL("libamdhip64.so")
        self.rt.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.rt.hipEventDestroy.argtypes = [C.c_void_p]
        self.rt.hipEventSynchronize.argtypes = [C.c_void_p]
        self.rt.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.rt.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.events = []

    def create(self) -> C.c_void_p:
        ev = C.c_void_p()
        rc = self.rt.hipEventCreate(C.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        self.events.append(ev)
        return ev

    def record(self, ev, stream=None) -> None:
        rc = self.rt.hipEventRecord(ev, _stream() if stream is None else stream)
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed ({rc})")

    def new_profile(self, capacity: int = 8) -> MorProfile:
        pr = MorProfile()
        pr.capacity = capacity
        for i in range(capacity):
            pr.start[i] = self.create().value
            pr.stop[i] = self.create().value
        return pr

    def elapsed_ms(self, a, b) -> float:
        ms = C.c_float()
        self.rt.hipEventSynchronize(C.c_void_p(b) if isinstance(b, int) else b)
        rc = self.rt.hipEventElapsedTime(C.byref(ms), C.c_void_p(a) if isinstance(a, int) else a,
                                         C.c_void_p(b) if isinstance(b, int) else b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def destroy(self) -> None:
        for ev in self.events:
            self.rt.hipEventDestroy(ev)
        self.events = []


def mor_dequantize(params: MorParams, fp8: torch.Tensor, scale: torch.Tensor, mask: torch.Tensor,
                   bf16: torch.Tensor | None, y: torch.Tensor) -> None:
    rc = load().mor_dequantize(C.byref(params), _ptr(fp8), fp8.stride(0), _ptr(scale), _ptr(mask), _ptr(bf16),
                               bf16.stride(0) if bf16 is not None else 0, _ptr(y), y.stride(0), _stream())
    if rc != 0:
        raise MorError(rc, "mor_dequantize")


def mor_dequantize_e8m0(params: MorParams, fp8: torch.Tensor, scale_e8m0: torch.Tensor, group_mantissa: torch.Tensor,
                        mask: torch.Tensor, bf16: torch.Tensor | None, y: torch.Tensor) -> None:
    """De-quantize from the stored form of GAM / E8M0 scaling (one byte per block + one shared mantissa)."""
    rc = load().mor_dequantize_e8m0(C.byref(params), _ptr(fp8), fp8.stride(0), _ptr(scale_e8m0), _ptr(group_mantissa),
                                    _ptr(mask), _ptr(bf16), bf16.stride(0) if bf16 is not None else 0, _ptr(y),
                                    y.stride(0), _stream())
    if rc != 0:
        raise MorError(rc, "mor_dequantize_e8m0")


def make_dequant_batch(entries) -> "C.Array":
    """entries: sequence of (params, result: MorResult, y: torch.Tensor[, stored: bool]); ``stored`` selects the E8M0 byte +
    group mantissa form of the scales.  Returns the host item array for :func:`mor_dequantize_batch`."""
    arr = (MorDequantItem * len(entries))()
    for i, entry in enumerate(entries):
        params, r, y = entry[:3]
        stored = entry[3] if len(entry) > 3 else False
        arr[i].params = params
        arr[i].fp8 = r.fp8.data_ptr(); arr[i].ld_fp8 = r.fp8.stride(0)
        arr[i].scale = None if stored else r.scale.data_ptr()
        arr[i].scale_e8m0 = r.scale_e8m0.data_ptr() if stored else None
        arr[i].group_mantissa = r.group_mantissa.data_ptr() if stored else None
        arr[i].mask = r.mask.data_ptr()
        arr[i].bf16 = r.bf16.data_ptr() if r.bf16 is not None else None
        arr[i].ld_bf16 = r.bf16.stride(0) if r.bf16 is not None else 0
        arr[i].y = y.data_ptr(); arr[i].ld_y = y.stride(0)
    return arr


def mor_dequantize_batch(items) -> None:
    rc = load().mor_dequantize_batch(items, len(items), _stream())
    if rc != 0:
        raise MorError(rc, "mor_dequantize_batch")


def mor_select_stats(params: MorParams, err_sum: torch.Tensor, nnz: torch.Tensor, mask: torch.Tensor,
                     near_tol: float, out_dev: torch.Tensor) -> None:
    """``out_dev``: device uint8 tensor of ``ctypes.sizeof(MorStats)`` bytes, 8-byte aligned."""
    if out_dev.numel() * out_dev.element_size() < C.sizeof(MorStats):
        raise ValueError("out_dev too small")
    rc = load().mor_select_stats(C.byref(params), _ptr(err_sum), _ptr(nnz), _ptr(mask), near_tol, _ptr(out_dev), _stream())
    if rc != 0:
        raise MorError(rc, "mor_select_stats")


def read_stats(out_dev: torch.Tensor) -> dict:
    """Copy a device mor_stats back to the host as a dict (synchronizes)."""
    raw = bytes(out_dev.cpu().numpy().tobytes()[:C.sizeof(MorStats)])
    st = MorStats.from_buffer_copy(raw)
    d = {k: getattr(st, k) for k, _ in MorStats._fields_ if k != "hist"}
    d["hist"] = [int(v) for v in st.hist]
    return d
