"""The C-ABI libraries load without a GPU and export every function their headers declare."""
import ctypes
import os
import re

import pytest

from paper_2408_11200_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return ctypes.CDLL(binding.LIB_PATH)


@pytest.fixture(scope="module")
def bench_lib():
    if not os.path.exists(binding.BENCH_LIB_PATH):
        build.build()
    return ctypes.CDLL(binding.BENCH_LIB_PATH)


def declared_functions(header="kan.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith(("kan_", "ukan_"))})


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"kan_forward", "kan_backward", "ukan_cg_forward", "ukan_cg_backward"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_bench_library_exports_its_header(bench_lib, lib):
    names = declared_functions("kan_bench.h")
    assert {"kan_profile_enable", "kan_profile_read", "kan_dense_baseline_forward"} <= set(names)
    for n in names:
        assert hasattr(bench_lib, n), n
        assert not hasattr(lib, n), n + " belongs to the benchmark library only"
    assert set(binding.BENCH_EXPORTS) == set(names)


def test_layer_library_links_no_blas(lib):
    """Only the benchmark library may depend on rocBLAS."""
    import subprocess
    needed = subprocess.run(["readelf", "-d", binding.LIB_PATH], stdout=subprocess.PIPE, text=True).stdout
    assert "NEEDED" in needed and "blas" not in needed.lower()


def test_launch_observer_is_host_only(lib):
    lib.kan_set_launch_observer.restype = ctypes.c_int
    lib.kan_set_launch_observer.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.kan_set_launch_observer(None, None) == binding.KAN_OK


def test_host_only_calls(lib):
    """Calls that never touch the device: status strings and workspace sizes."""
    lib.kan_strerror.restype = ctypes.c_char_p
    assert lib.kan_strerror(0) == b"ok"
    assert b"workspace" in lib.kan_strerror(binding.KAN_ERR_WORKSPACE)
    lib.kan_workspace_bytes.restype = ctypes.c_size_t
    lib.kan_workspace_bytes.argtypes = [ctypes.POINTER(binding.KanLayerDesc), ctypes.c_int64, ctypes.c_int]
    d = binding.KanLayerDesc(512, 512, 20, 3, -1.0, 1.0, 1)
    fwd = lib.kan_workspace_bytes(ctypes.byref(d), 16384, binding.PASS_FORWARD)
    bwd = lib.kan_workspace_bytes(ctypes.byref(d), 16384, binding.PASS_BACKWARD)
    assert fwd >= 512 * 23 * 512 * 4 and fwd % 256 == 0
    assert bwd > fwd and bwd % 256 == 0
    assert lib.kan_workspace_bytes(None, 1, 0) == 0
    bad = binding.KanLayerDesc(512, 512, 0, 3, -1.0, 1.0, 1)
    assert lib.kan_workspace_bytes(ctypes.byref(bad), 1, 0) == 0
    lib.ukan_workspace_bytes.restype = ctypes.c_size_t
    lib.ukan_workspace_bytes.argtypes = [ctypes.POINTER(binding.UkanLayerDesc), ctypes.c_int64, ctypes.c_int32,
                                         ctypes.c_int]
    u = binding.UkanLayerDesc(128, 256, 3, 0.25, 32, 32, 64, 0)
    assert lib.ukan_workspace_bytes(ctypes.byref(u), 32768, 128, 1) > lib.ukan_workspace_bytes(
        ctypes.byref(u), 32768, 128, 0) > 128 * 128 * 4 * 256 * 4
    # B == 0 succeeds before any pointer is looked at; null descriptor is rejected
    lib.kan_forward.restype = ctypes.c_int
    assert lib.kan_forward(ctypes.byref(d), ctypes.c_int64(0), None, None, None, None, None, None,
                           ctypes.c_size_t(0), None) == binding.KAN_OK
    assert lib.kan_forward(None, ctypes.c_int64(0), None, None, None, None, None, None, ctypes.c_size_t(0),
                           None) == binding.KAN_ERR_INVALID_ARG


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError):
        binding.load()


def test_workspace_planning_limits(lib):
    """Host-side planning seen through the workspace queries: unsupported shapes report 0 bytes, tables too large
    for one partial table per chunk stay within the partial-table budget, and the degree-5 backward pass (two
    records per pair) asks for about twice the record space of the cubic one."""
    lib.kan_workspace_bytes.restype = ctypes.c_size_t
    lib.kan_workspace_bytes.argtypes = [ctypes.POINTER(binding.KanLayerDesc), ctypes.c_int64, ctypes.c_int]
    ws = lambda *a, B=1 << 17, which=binding.PASS_BACKWARD: lib.kan_workspace_bytes(
        ctypes.byref(binding.KanLayerDesc(*a)), B, which)
    assert ws(70000, 8, 5, 3, -1.0, 1.0, 1) == 0                       # more inputs than a launch dimension holds
    assert ws(4, 1 << 20, 1 << 12, 3, -1.0, 1.0, 1) == 0              # a table row range beyond 32-bit offsets
    assert ws(32, 32, 64, 6, -1.0, 1.0, 1) == 0                        # degree 6
    table = lambda G: 32 * (G + 4) * 32 * 4
    small, huge = ws(32, 32, 1 << 15, 3, -1.0, 1.0, 1), ws(32, 32, 1 << 18, 3, -1.0, 1.0, 1)
    assert small > 16 * table(1 << 15)                                  # one partial table per chunk of 8192 samples
    assert table(1 << 18) * 3 < huge < 5 << 30                          # shared partial tables: about 4 GiB, not 16 tables
    k3, k5 = ws(32, 32, 64, 3, -1.0, 1.0, 1, B=1 << 16), ws(32, 32, 64, 5, -1.0, 1.0, 1, B=1 << 16)
    assert 1.7 * k3 < k5 < 2.3 * k3
    lib.ukan_saved_bytes.restype = ctypes.c_size_t
    lib.ukan_saved_bytes.argtypes = [ctypes.POINTER(binding.UkanLayerDesc), ctypes.c_int32]
    u = binding.UkanLayerDesc(128, 256, 3, 0.25, 32, 32, 64, 0)
    assert lib.ukan_saved_bytes(ctypes.byref(u), 1) == 0
    a, b = lib.ukan_saved_bytes(ctypes.byref(u), 64), lib.ukan_saved_bytes(ctypes.byref(u), 128)
    assert 2 * 128 * 64 * 4 * 256 * 4 < a < b < 2.1 * a
