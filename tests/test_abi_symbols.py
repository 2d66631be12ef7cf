"""The C-ABI library loads and exports every symbol include/gla.h declares (no GPU calls)."""
import ctypes
import os

import pytest

import paper_2405_18428_amd as gla


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(gla.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(gla.library_path())


def test_header_symbols_are_exported(lib):
    names = gla.lib_symbols()
    assert {"gla_fwd", "gla_fwd_ex", "gla_fwd_workspace_bytes", "gla_fwd_timed",
            "gla_status_string", "gla_version", "gla_set_option", "gla_get_option"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_host_only_entry_points():
    assert gla.gla_version() >= 100
    assert gla.gla_status_string(0) == "ok"
    for code in range(1, 7):
        assert gla.gla_status_string(code) not in ("ok", "unknown status")
    assert gla.gla_status_string(99) == "unknown status"
    # workspace bound: one state (dk*dv) and one decay vector (dk) per 64-token chunk, fp32
    n = gla.gla_fwd_workspace_bytes(1, 16, 16384, 36, 72)
    assert n >= 16 * 256 * (36 * 72 + 36) * 4
    assert n < 2 * 16 * 256 * (36 * 72 + 36) * 4
    assert gla.gla_fwd_workspace_bytes(0, 1, 1, 1, 1) == 0


def test_block_schedule_matches_the_oracle():
    """gla_block_scan_dir (host only) against the oracle's literal transposes / flips of Algorithms 1 and 4."""
    from oracle import gla_oracle
    for sched_lib, sched_ref in ((gla.SCHEDULE_BLOCK_PROCESS, gla_oracle.SCHEDULE_BLOCK_PROCESS),
                                 (gla.SCHEDULE_BLOCK_SCAN, gla_oracle.SCHEDULE_BLOCK_SCAN)):
        for block in range(1, 30):
            assert gla.gla_block_scan_dir(block, sched_lib) == gla_oracle.block_scan_dir(block, sched_ref, grid=3)
    for bad in ((0, 0), (-3, 1), (1, 2), (1, -1)):
        with pytest.raises(gla.GlaError):
            gla.gla_block_scan_dir(*bad)


def test_options_round_trip():
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 3)
    assert gla.gla_get_option(gla.OPT_CHUNKS_PER_SPAN) == 3
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 0)
    with pytest.raises(gla.GlaError):
        gla.gla_set_option(gla.OPT_ENGINE, 7)
    gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_IN_OUTPUT_PASS)
    assert gla.gla_get_option(gla.OPT_CARRY) == gla.CARRY_IN_OUTPUT_PASS
    gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_AUTO)
    gla.gla_set_option(gla.OPT_BWD_SPLIT, 1)
    assert gla.gla_get_option(gla.OPT_BWD_SPLIT) == 1
    gla.gla_set_option(gla.OPT_BWD_SPLIT, 0)
    with pytest.raises(gla.GlaError):
        gla.gla_set_option(gla.OPT_BWD_SPLIT, 2)
    with pytest.raises(gla.GlaError):
        gla.gla_set_option(gla.OPT_CARRY, 3)
    with pytest.raises(gla.GlaError):
        gla.gla_set_option(42, 0)


def test_argument_validation_needs_no_gpu():
    """Bad arguments are rejected on the host before anything is enqueued."""
    lib = gla.load_library()
    vp = ctypes.c_void_p
    ok_ptr = vp(4096)
    call = lambda q, T, gh, gw, dk, dv, sd: lib.gla_fwd(q, ok_ptr, ok_ptr, ok_ptr, 1, 1, T, dk, dv, gh, gw, sd,
                                                        ok_ptr, None, None)
    assert call(None, 4, 2, 2, 8, 8, 0) == 1          # NULL
    assert call(ok_ptr, 5, 2, 2, 8, 8, 0) == 2        # grid mismatch
    assert call(ok_ptr, 4, 2, 2, 8, 8, 4) == 2        # bad scan order
    assert call(ok_ptr, 4, 2, 2, 65, 8, 0) == 3       # dk too large
    assert call(ok_ptr, 4, 2, 2, 8, 129, 0) == 3      # dv too large
    lay = lambda layout, init: lib.gla_fwd_layout(ok_ptr, ok_ptr, ok_ptr, ok_ptr, 1, 1, 4, 8, 8, 2, 2, 0, 1, 0,
                                                  layout, init, ok_ptr, None, ok_ptr, 1 << 20, None)
    assert lay(2, None) == 2                          # unknown memory order
    assert lay(1, vp(4100)) == 4                      # initial state not 16-byte aligned
    assert call(vp(4100), 4, 2, 2, 8, 8, 0) == 4      # misaligned
    # gla_fwd_ex: missing / short workspace
    r = lib.gla_fwd_ex(ok_ptr, ok_ptr, ok_ptr, ok_ptr, 1, 1, 4, 8, 8, 2, 2, 0, 1, 0, ok_ptr, None, None, 0, None)
    assert r == 5
    r = lib.gla_fwd_ex(ok_ptr, ok_ptr, ok_ptr, ok_ptr, 1, 1, 4, 8, 8, 2, 2, 0, 1, 0, ok_ptr, None, ok_ptr, 16, None)
    assert r == 5
    r = lib.gla_fwd_ex(ok_ptr, ok_ptr, ok_ptr, ok_ptr, 1, 1, 4, 8, 8, 2, 2, 0, 5, 0, ok_ptr, None, ok_ptr, 1 << 20, None)
    assert r == 2
    # two-sided gate: the value-side tensor is mandatory and must be aligned
    g = lambda lb: lib.gla_fwd_gates(ok_ptr, ok_ptr, ok_ptr, ok_ptr, lb, 1, 1, 4, 8, 8, 2, 2, 0, 1, 0, 0, None,
                                     ok_ptr, None, ok_ptr, 1 << 20, None)
    assert g(None) == 1
    assert g(vp(4100)) == 4
    f = ctypes.c_float
    fg = lambda zb: lib.gla_fwd_fused_gates(ok_ptr, ok_ptr, ok_ptr, ok_ptr, zb, f(16.0), None, None, None, f(1e-5),
                                            1, 1, 4, 8, 8, 2, 2, 0, 1, 0, ok_ptr, None, ok_ptr, 1 << 20, None)
    assert fg(None) == 1
    assert fg(vp(4100)) == 4


def test_static_scratch_rejects_oversize_on_the_host():
    """gla_fwd_static: a plan that needs more than the static array is refused before any HIP call."""
    lib = gla.load_library()
    ok = ctypes.c_void_p(4096)
    # 4096 sequences of 1024 chunks, one span each: 4096 * (64 * 128 + 64 + 128) floats, far beyond 16 MiB
    assert lib.gla_fwd_static(ok, ok, ok, ok, 64, 64, 65536, 64, 128, 256, 256, 0, ok, None, None) == 5
    assert lib.gla_fwd_static(None, ok, ok, ok, 1, 1, 4, 8, 8, 2, 2, 0, ok, None, None) == 1
