"""Host-only checks of the C-ABI library: it loads, exports every function include/mor.h declares,
and its pure host helpers behave.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2512_22804_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mor.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mor_[a-z_0-9]+)\s*\(", text)))


def test_exports_every_declared_symbol(B):
    lib = B.load()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts(B):
    assert C.sizeof(B.MorStats) == 144 == B.STATS_BYTES
    assert C.sizeof(B.MorParams) == 56
    assert C.sizeof(B.MorOutputs) == 104
    assert C.sizeof(B.MorProfile) == 8 + 16 * 8 * 2 + 16 * 4


def test_num_partitions(B):
    assert B.mor_num_partitions("tensor", 8192, 4096) == 1
    assert B.mor_num_partitions("sub1x128", 8192, 4096) == 262144
    assert B.mor_num_partitions("block128", 14336, 4096) == 3584
    assert B.mor_num_partitions("sub1x128", 8192, 14336) == 917504
    assert B.mor_num_partitions("block128", 8192, 14336) == 7168
    assert B.mor_num_partitions("sub1x128", 4, 100) == -1
    assert B.mor_num_partitions("block128", 100, 128) == -1
    assert B.mor_num_partitions("tensor", 3, 12) == -1
    assert B.mor_num_partitions("tensor", 0, 128) == -1
    assert B.mor_num_partitions(9, 128, 128) == -1
    assert B.mor_num_partitions("channel_row", 8192, 4096) == 8192
    assert B.mor_num_partitions("channel_row", 8, 65536) == 8
    assert B.mor_num_partitions("channel_row", 8, 65544) == -1               # rows longer than 65536 elements
    assert B.mor_num_partitions("channel_col", 8192, 4096) == 4096
    assert B.mor_num_partitions("sub128x1", 8192, 4096) == 64 * 4096
    assert B.mor_num_partitions("sub128x1", 100, 4096) == -1
    assert B.mor_num_partitions("block64", 8192, 14336) == 128 * 224
    assert B.mor_params_num_partitions(B.make_params(130, 200, "block64", ragged=True)) == 3 * 4
    assert B.mor_params_num_partitions(B.make_params(130, 200, "block64")) == -1
    assert B.mor_params_num_partitions(B.make_params(130, 204, "block64", ragged=True)) == -1   # 16-byte rows
    assert B.mor_params_num_partitions(B.make_params(3, 136, "sub1x128", ragged=True)) == 6


def test_workspace_bytes(B):
    assert B.mor_workspace_bytes(B.make_params(8192, 4096, "sub1x128")) == 0
    assert B.mor_workspace_bytes(B.make_params(8192, 4096, "block128")) == 0
    assert B.mor_workspace_bytes(B.make_params(8192, 4096, "sub1x128", scope="tensor")) > 0
    t = B.mor_workspace_bytes(B.make_params(8192, 14336, "tensor"))
    assert 0 < t < (1 << 22) and t % 16 == 0
    assert B.mor_workspace_bytes(B.make_params(8192, 100, "sub1x128")) == 0      # invalid -> 0
    assert B.mor_workspace_bytes(B.make_params(8192, 4096, "channel_row")) == 0
    assert B.mor_workspace_bytes(B.make_params(8192, 4096, "block64")) == 0
    c = B.mor_workspace_bytes(B.make_params(8192, 4096, "channel_col"))
    assert 0 < c < (1 << 23) and c % 16 == 0


def test_status_strings(B):
    lib = B.load()
    seen = {lib.mor_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and lib.mor_status_string(0).decode() == "ok"
    assert "unknown" in lib.mor_status_string(99).decode()


def test_argument_validation_without_a_gpu(B):
    """Argument errors are reported before anything is launched, so they can be checked on the host: fake but
    well-aligned device addresses are enough (they are never dereferenced)."""
    lib = B.load()
    base = 0x7F0000000000

    def call(params, x=base, **over):
        o = B.MorOutputs(fp8=base + (1 << 30), ld_fp8=params.cols, bf16=base + (2 << 30), ld_bf16=params.cols,
                         scale=base + (3 << 30), amax=base + (3 << 30) + 4096, err_sum=base + (3 << 30) + 8192,
                         nnz=base + (3 << 30) + 12288, mask=base + (3 << 30) + 16384, err5_sum=None,
                         scale_e8m0=None, group_mantissa=None, amin=None)
        for k, v in over.items():
            setattr(o, k, v)
        return lib.mor_analyze_quantize(C.byref(params), C.c_void_p(x), C.byref(o), None, 0, None)

    assert call(B.make_params(128, 200, "sub1x128")) == 2                     # cols not a whole number of blocks
    assert call(B.make_params(128, 200, "sub1x128", ragged=True), fp8=base + 4) == 3   # misaligned payload
    assert call(B.make_params(100, 256, "block64")) == 2
    assert call(B.make_params(128, 256, "channel_row", ld=128)) == 2          # ld < cols
    assert call(B.make_params(128, 256, "sub128x1", ld=260)) == 3             # ld % 8
    big = (1 << 22) + 8                                                       # above MOR_MAX_LD
    assert call(B.make_params(128, 256, "block128", ld=big)) == 2
    assert call(B.make_params(128, 256, "channel_col"), ld_fp8=big) == 2
    assert call(B.make_params(128, 256, "block64"), ld_bf16=big) == 2
    assert call(B.make_params(128, 256, "tensor", ld=big)) == 5              # no such limit where blocks do not span rows (passes validation)
    assert call(B.make_params(128, 256, 7)) == 4
    assert call(B.make_params(128, 256, "sub1x128", formats=B.MOR_FMT_E4M3 | B.MOR_FMT_E5M2)) == 4
    assert call(B.make_params(128, 256, "tensor", scope="tensor", crit="e4m3_vs_e5m2", formats="e4m3|e5m2|bf16"),
                err5_sum=base + (4 << 30)) == 4
    assert call(B.make_params(128, 256, "channel_col", scope="tensor", crit="e4m3_vs_e5m2", formats="e4m3|e5m2|bf16"),
                err5_sum=base + (4 << 30)) == 4
    assert call(B.make_params(128, 256, "sub1x128", scope="tensor", crit="e4m3_vs_e5m2", formats="e4m3|e5m2|bf16"),
                err5_sum=base + (4 << 30)) == 4
    assert call(B.make_params(128, 256, "sub1x128", scaling=3)) == 4
    assert call(B.make_params(128, 256, "sub1x128", crit=5)) == 4
    assert call(B.make_params(128, 256, "sub1x128"), x=base + 2) == 3
    assert call(B.make_params(128, 256, "sub1x128"), mask=None) == 1
    assert call(B.make_params(128, 256, "sub1x128", crit="e4m3_vs_e5m2")) == 1            # err5_sum missing
    assert call(B.make_params(128, 256, "tensor")) == 5                                   # workspace missing
    assert call(B.make_params(128, 256, "channel_col")) == 5
    assert call(B.make_params(128, 256, "block128", scope="tensor")) == 5
    p = B.make_params(128, 256, "sub1x128"); p.flags = 8
    assert call(p) == 4
    assert call(B.make_params(128, 256, "tensor", lean_fp8=True, ragged=True)) == 5       # both flags pass validation
    # GAM groups as bands of rows: whole blocks only, and not for partitions whose blocks span every band
    assert call(B.make_params(256, 256, "block128", scaling="gam", gam_group_rows=64)) == 2
    assert call(B.make_params(256, 256, "tensor", scaling="gam", gam_group_rows=128)) == 4
    assert call(B.make_params(256, 256, "channel_col", scaling="gam", gam_group_rows=128)) == 4
    assert call(B.make_params(256, 256, "block128", scaling="gam", gam_group_rows=128)) == 5     # valid: workspace missing
    # fake quantization: y must not alias x, needs 16-byte alignment and ld_y >= cols
    pr = B.make_params(128, 256, "block128")
    o = B.MorOutputs(scale=base, amax=base + 4096, err_sum=base + 8192, nnz=base + 12288, mask=base + 16384)
    fq = lambda x, y, ld: lib.mor_fake_quantize(C.byref(pr), C.c_void_p(x), C.c_void_p(y), ld, C.byref(o), None, 0, None)
    assert fq(base + (1 << 30), base + (1 << 30), 256) == 4
    assert fq(base + (1 << 30), base + (2 << 30) + 8, 256) == 3
    assert fq(base + (1 << 30), base + (2 << 30), 128) == 2
    assert fq(base + (1 << 30), None, 256) == 1
    # histogram: argument checks only
    assert lib.mor_histogram_update(None, C.c_void_p(base), 0, 6000, None) == 1
    assert lib.mor_histogram_update(C.c_void_p(base), C.c_void_p(base + 1024), -1, 6000, None) == 2
    assert lib.mor_histogram_update(C.c_void_p(base + 2), C.c_void_p(base + 1024), 0, 6000, None) == 3
