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
