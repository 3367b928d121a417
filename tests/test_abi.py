"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its pure host entry points behave."""
import ctypes
import os
import re

import pytest

from paper_2506_04985_amd import binding as fptq
from paper_2506_04985_amd import probe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fptq_[a-z0-9_]+)\s*\(", text)))


def test_libraries_export_every_declared_symbol():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["fptq.h", "fptq_probe.h", "fptq_testing.h"]
    for header, L, exports in (("fptq.h", fptq.lib(), fptq.EXPORTS), ("fptq_testing.h", fptq.lib(), fptq.TESTING_EXPORTS),
                               ("fptq_probe.h", probe.lib(), probe.EXPORTS)):
        names = header_symbols(header)
        assert set(names) == set(exports), header
        for n in names:
            assert getattr(L, n) is not None
    # the measurement aids are not part of the product library
    assert not hasattr(fptq.lib(), "fptq_probe_read")


def test_host_only_entry_points():
    L = fptq.lib()
    assert L.fptq_version() >= 100
    assert L.fptq_packed_bytes(1, 1) == 64
    assert L.fptq_packed_bytes(10, 128) == 640
    assert L.fptq_packed_bytes(10, 129) == 1280
    assert L.fptq_packed_bytes(57344, 8192) == 57344 * 8192 // 2
    assert L.fptq_packed_bytes(0, 8) == -2
    assert b"bad shape" in L.fptq_last_error()
    # validation happens before any launch, so these return without touching a device
    assert L.fptq_pack_weights(None, 4, 4, None, 0, None) == -1
    assert L.fptq_quantize_act(None, 4, 4, 1, 0.0, None, 1.0, None, 0, None, None) == -1
    assert L.fptq_unpack(None, 1, 1, None, None) == -1
    dummy = ctypes.c_void_p(256)
    assert L.fptq_quantize_act(dummy, 0, 4, 1, 0.0, None, 1.0, dummy, 0, None, None) == -2
    assert L.fptq_quantize_act(dummy, 4, 4, 9, 0.0, None, 1.0, dummy, 1 << 20, None, None) == -4
    assert L.fptq_quantize_act(dummy, 4, 4, 1, 0.0, None, -1.0, dummy, 1 << 20, None, None) == -6
    assert L.fptq_quantize_act(dummy, 4, 4, 1, 0.0, None, 1.0, dummy, 8, None, None) == -3
    assert L.fptq_w4a4_linear(dummy, dummy, 4, 0, 4, 1.0, dummy, None, dummy, None, None) == -2
    assert L.fptq_w4a4_linear(dummy, dummy, 4, 4, 4, float("inf"), dummy, None, dummy, None, None) == -6


def test_k_beyond_exact_int32_accumulation_is_refused():
    """|q w| <= 64, so INT32 sums are exact up to K = 2^25 - 1; with a zero point the epilogue's acc - z * sum_k w
    needs K <= 2^24 - 1.  Longer sums are refused before anything is launched."""
    L = fptq.lib()
    dummy = ctypes.c_void_p(4096)
    big, big_zp = (1 << 25) - 1, (1 << 24) - 1
    for fn in (L.fptq_w4a4_linear, L.fptq_w4a4_linear_ref):
        assert fn(dummy, dummy, 1, 1, big + 1, 1.0, dummy, None, dummy, None, None) == -2
        assert b"INT32" in L.fptq_last_error()
    assert L.fptq_w4a4_linear_ws(dummy, dummy, 1, 1, big + 1, 1.0, dummy, None, dummy, None, None, 0, None) == -2
    assert L.fptq_w4a4_linear_zp(dummy, dummy, 1, 1, big_zp + 1, 1.0, dummy, None, 3, dummy, dummy, None, None) == -2
    assert L.fptq_w4a4_linear_zp(dummy, dummy, 1, 1, big + 1, 1.0, dummy, None, 0, None, dummy, None, None) == -2
    assert L.fptq_linear_workspace_bytes(1, 1, big + 1) == -2
    assert L.fptq_linear_workspace_bytes(256, 1024, big) >= 0


def test_workspace_size_is_host_arithmetic():
    L = fptq.lib()
    f = L.fptq_linear_workspace_bytes
    assert f(256, 1024, 14336) == (1024 + 4 * 64 * 64 * 64) * 4     # 1024 counters, 64 tiles of 64 x 64, four K ranges of 28 K tiles
    assert f(129, 128, 12288) == (1024 + 4 * 6 * 64 * 64) * 4       # 6 tiles: the counter region has a fixed size
    assert f(512, 1024, 12288) == (1024 + 2 * 128 * 64 * 64) * 4    # 128 tiles leave room for two ranges
    assert f(256, 1024, 6144) == (1024 + 3 * 64 * 64 * 64) * 4      # 48 K tiles: three ranges of 16
    assert f(256, 1024, 4096) == 0 and f(256, 4096, 14336) == 0 and f(64, 1024, 14336) == 0 and f(2048, 11008, 4096) == 0
    assert f(0, 4096, 4096) == -2 and f(256, 4096, -1) == -2
    dummy = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4096 + 64)                                  # not 256-byte aligned
    assert L.fptq_w4a4_linear_ws(dummy, dummy, 256, 4096, 14336, 1.0, dummy, None, dummy, None, odd, 1 << 30, None) == -7
    assert L.fptq_w4a4_linear_ws(dummy, dummy, 256, 4096, 14336, 1.0, dummy, None, dummy, None, dummy, -5, None) == -3
    assert L.fptq_w4a4_linear_ws(None, dummy, 256, 4096, 14336, 1.0, dummy, None, dummy, None, dummy, 0, None) == -1


def test_testing_knobs_validate_and_the_launch_plan_is_host_arithmetic():
    L = fptq.lib()
    for bad in (-1, 9, 100):
        assert L.fptq_set_gemm_tile(bad) == -6
    for bad in (-1, 2):
        assert L.fptq_set_gemm_map(bad) == -6
    for bad in (1, 811 + 1000, 1631, 1615, 911):
        assert L.fptq_set_decode_shape(bad) == -6
    for ok in (811, 1624, 0):
        assert L.fptq_set_decode_shape(ok) == 0
    assert L.fptq_set_gemm_tile(0) == 0 and L.fptq_set_gemm_map(0) == 0
    # the shapes of the benchmark configurations on a 256-CU device: large tiles, two workgroups per CU or one
    plan = fptq.fptq_linear_launch_plan
    assert plan(8192, 57344, 8192) == ("GemmCfg<2, 2, 4, 4, 4, 1, 1, false>", 224 * 32, 256)
    assert plan(4096, 28672, 4096) == ("GemmCfg<2, 2, 4, 2, 3, 2, 1, false>", 112 * 32, 256)
    assert plan(8192, 8192, 28672) == ("GemmCfg<2, 2, 4, 4, 4, 1, 1, false>", 32 * 32, 256)
    assert plan(2048, 4096, 11008) == ("GemmCfg<2, 2, 4, 2, 3, 1, 2, false>", 16 * 16, 512)
    assert plan(256, 1024, 8192) == ("GemmCfg<1, 1, 2, 2, 4, 1, 4, false>", 64, 256)
    assert plan(256, 1024, 8192, True) == ("GemmCfg<1, 1, 2, 2, 4, 1, 4, true>", 64 * 4, 256)
    assert plan(8, 4096, 4096)[0] == "linear_decode_kernel" and plan(64, 28672, 4096)[0].startswith("GemmCfg")
    assert plan(300, 300, 200000)[0] == "linear_ref_kernel"
    with pytest.raises(fptq.FptqError):
        plan(0, 4, 4)
