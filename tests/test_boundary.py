"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, sizes and
error paths behave.  No kernel is launched here (argument validation precedes any HIP call)."""
import ctypes
import os
import re

import pytest

import paper_2302_06646_amd as lc

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "longconv.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(longconv(?:2d)?_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = lc.lib()
    names = _declared()
    assert set(names) == set(lc.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_sizes_and_plan():
    assert lc.longconv_kspec_bytes(4, 1024, lc.F32) == 4 * 2048 * 8
    assert lc.longconv_kspec_bytes(4, 1000, lc.F32) == 0           # not a power of two
    assert lc.longconv_kspec_bytes(4, 128, lc.F32) == 0            # too short
    assert lc.longconv_kspec_bytes(4, 262144, lc.F16) == 0         # too long
    assert lc.longconv_workspace_bytes(2, 4, 1024, 7, False) == 0  # bad dtype
    for N in (256, 1024, 16384, 65536, 131072):
        for io in (lc.F32, lc.F16, lc.BF16):
            f = lc.longconv_workspace_bytes(3, 5, N, io, False)
            b = lc.longconv_workspace_bytes(3, 5, N, io, True)
            assert f >= lc.longconv_kspec_bytes(5, N, io) and b >= f
            assert "engine=" in lc.longconv_plan_string(N, io)
    assert "valu" in lc.longconv_plan_string(1024, lc.F32)
    assert "mfma" in lc.longconv_plan_string(1024, lc.BF16)
    assert "passes=3" in lc.longconv_plan_string(131072, lc.F16)
    assert lc.longconv_plan_string(100, lc.F32) == "invalid"


def test_spectrum_size_is_exact_per_dtype():
    # fp32 I/O stores fp32 complex bins, half I/O fp16 complex bins (matrix-core kernels) and, behind them, one
    # 32-bit exponent per head (the power of two left out of that head's stored values), rounded up to 16 bytes
    assert lc.longconv_kspec_bytes(3, 2048, lc.F32) == 3 * 4096 * 8
    for io in (lc.F16, lc.BF16):
        for N in (256, 1024, 16384, 65536):
            assert lc.longconv_kspec_bytes(3, N, io) == 3 * 2 * N * 4 + 16
        assert lc.longconv_kspec_bytes(8, 1024, io) == 8 * 2048 * 4 + 32


def test_options_switch_plans_and_reject_bad_input():
    try:
        assert "kernel=wave" in lc.longconv_plan_string(1024, lc.F16)
        lc.longconv_set_option("staged_kernel", 1)
        assert "kernel=" not in lc.longconv_plan_string(1024, lc.F16)
        assert lc.longconv_kspec_bytes(3, 1024, lc.F16) == 3 * 2048 * 8       # that kernel keeps fp32 bins
        lc.longconv_set_option("staged_kernel", 0)
        lc.longconv_set_option("inner_log2", 9)
        assert "passes=3" in lc.longconv_plan_string(1024, lc.F32)
        lc.longconv_set_option("inner_log2", 0)
        lc.longconv_set_option("engine", 1)
        assert "valu" in lc.longconv_plan_string(1024, lc.F16)
        lc.longconv_set_option("engine", 2)
        assert "valu" in lc.longconv_plan_string(1024, lc.F32)                # fp32 I/O never runs on fp16 operands
        L = lc.lib()
        assert L.longconv_set_option(b"no_such_switch", 1) == 2
        assert L.longconv_set_option(b"engine", 5) == 2
        assert L.longconv_set_option(None, 1) == 1
    finally:
        for name, value in lc.OPTION_DEFAULTS.items():
            lc.longconv_set_option(name, value)
    assert "kernel=wave" in lc.longconv_plan_string(1024, lc.F16)


def test_error_codes_before_any_launch():
    L = lc.lib()
    a = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    ws = ctypes.c_void_p(0x2000)
    big = 1 << 40
    f = L.longconv_fwd
    assert f(None, a, a, None, a, 2, 4, 1024, 0, ws, big, None) == 1            # NULL u
    assert f(a, None, a, None, a, 2, 4, 1024, 0, ws, big, None) == 1            # no k and no kspec
    assert f(a, a, a, None, a, 0, 4, 1024, 0, ws, big, None) == 2               # B < 1
    assert f(a, a, a, None, a, 2, 4, 1000, 0, ws, big, None) == 2               # N not a power of two
    assert f(a, a, a, None, a, 2, 70000, 1024, 0, ws, big, None) == 2           # H beyond 65535
    assert f(a, a, a, None, a, 1 << 12, 1 << 12, 1024, 1, ws, big, None) == 2   # more (head, pair) items than 2^22
    assert f(a, a, a, None, a, 2, 4, 1024, 9, ws, big, None) == 3               # dtype
    assert f(odd, a, a, None, a, 2, 4, 1024, 0, ws, big, None) == 4             # alignment
    assert f(a, a, a, None, a, 2, 4, 1024, 0, ws, 16, None) == 5                # workspace too small
    assert f(a, a, a, None, a, 2, 4, 1024, 0, None, big, None) == 5             # workspace missing
    b = L.longconv_bwd
    assert b(None, a, a, a, None, a, a, a, 2, 4, 1024, 0, ws, big, None) == 1   # NULL dy
    assert b(a, None, a, a, None, a, a, a, 2, 4, 1024, 0, ws, big, None) == 1   # dk wanted, no u
    assert b(a, a, a, a, None, a, a, a, 2, 4, 2048 + 1, 0, ws, big, None) == 2
    assert b(a, a, a, a, None, a, a, a, 2, 4, 1024, 0, ws, 8, None) == 5
    r = L.longconv_kreg_fwd
    lam = ctypes.c_float(0.01)
    assert r(None, None, a, 4, 1024, 1, lam, None) == 1                         # NULL k
    assert r(a, None, None, 4, 1024, 1, lam, None) == 1                         # NULL output
    assert r(a, None, a, 4, 1024, 33, lam, None) == 2                           # window too wide
    assert r(a, None, a, 4, 1024, -1, lam, None) == 2
    assert r(a, None, a, 4, 1024, 1, ctypes.c_float(-0.5), None) == 2           # negative lambda
    assert r(a, None, a, 4, 1000, 1, lam, None) == 2
    assert L.longconv_kreg_bwd(a, None, None, a, 4, 1024, 1, lam, None) == 1    # NULL dkbar
    assert L.longconv_kreg_bwd(a, None, a, a, 4, 1024, 40, lam, None) == 2
    k = L.longconv_kspec_compute
    assert k(None, a, a, 4, 1024, 0, ws, big, None) == 1
    assert k(a, a, a, 4, 3, 0, ws, big, None) == 2
    for code in range(8):
        assert L.longconv_status_string(code)


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(lc, "_lib", None)
    monkeypatch.setattr(lc, "LIB_PATH", "/nonexistent/liblongconv.so")
    with pytest.raises(lc.LongconvError):
        lc.lib()


def test_bench_reads_the_offline_traffic_table():
    # roofline.traffic of bench.py comes from the text table written with the rocprofv3 summaries under profiles/:
    # every launch group of the three profiled workloads has a figure, and it is not below the algorithmic bytes
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    import workloads as wl
    table = bench.load_offline_traffic()
    for key in ("2", "3", "4a"):
        w = wl.WORKLOADS[key]
        groups = bench.group_bytes(w)
        assert w.name in table
        for grp, measured in table[w.name].items():      # the groups this workload's plan launches
            assert grp in groups, (w.name, grp)
            assert measured >= 0.95 * groups[grp]
        assert "fwd" in table[w.name] and ("bwd" in table[w.name] or "bwd_dk" in table[w.name])
