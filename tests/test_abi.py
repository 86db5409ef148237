"""The C-ABI library without a GPU: it loads, exports what the header declares,
rejects bad arguments on the host, and plans launches sensibly (CPU only)."""
import ctypes
import os
import re

import pytest

import paper_2007_03179_amd as gs
from paper_2007_03179_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gespmm.h")


@pytest.fixture(scope="module")
def L():
    hip_build.build(force=False)
    return gs.lib()


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(gespmm_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = _declared_functions()
    assert {"gespmm_csr", "gespmm_csr_simple", "gespmm_plan", "gespmm_plan_ex", "gespmm_csr_ex", "gespmm_csr_arg_ex",
            "gespmm_csr_workspace_bytes", "gespmm_profiler_create", "gespmm_profiler_finish", "gespmm_status_string",
            "gespmm_calibration_copy", "gespmm_calibration_gather", "gespmm_csr_arg", "gespmm_csr_transposed", "gespmm_pool_backward",
            "gespmm_csr_transpose", "gespmm_csr_transpose_workspace_bytes", "gespmm_csr_transpose_noalloc",
            "gespmm_csr_b16", "gespmm_plan_b16", "gespmm_csr_arg_b16", "gespmm_csr_transpose_sorted",
            "gespmm_csr_transpose_sorted_workspace_bytes", "gespmm_version", "gespmm_csr_arg_ws"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_b16_entry_point_argument_errors_and_plan(L):
    p = ctypes.c_void_p(0x1000)
    call = L.gespmm_csr_b16
    assert call(4, 4, 8, 8, p, p, p, p, 3, p, 0, None) == 1          # unknown element type
    assert call(4, 4, 8, 8, p, p, p, p, -1, p, 0, None) == 1
    assert call(4, 4, 8, 8, p, p, p, None, 1, p, 0, None) == 2       # B NULL
    assert call(4, 4, 8, 8, p, p, p, p, 2, p, 9, None) == 1          # unknown op
    assert call(0, 4, 8, 0, p, p, p, p, 1, p, 0, None) == 0          # nothing to do
    assert call(4, 4, 8, 2**31, p, p, p, p, 1, p, 0, None) == 3
    # 8-byte loads of 4 columns; 16 lanes cover a 128-byte line = 64 columns, 32 lanes two lines beyond N = 256
    want = {8: (4, 2, 1), 16: (4, 4, 1), 32: (4, 8, 1), 64: (4, 16, 1), 128: (4, 16, 2), 256: (4, 16, 4), 512: (4, 32, 4),
            12: (4, 4, 1), 100: (4, 16, 2), 4: (4, 1, 1), 6: (1, 8, 1), 130: (1, 64, 3)}
    for N, (vec, G, blocks) in want.items():
        for dt in ("bf16", "f16"):
            q = gs.gespmm_plan_b16(10**6, N, 10**8, dt)
            assert (q["vec"], q["lanes_per_row"], q["tiles_per_lane"], q["col_blocks"]) == (vec, G, 1, blocks), (N, q)
    assert gs.gespmm_plan_b16(10**6, 64, 10**8, "bf16", aligned16=False)["vec"] == 1
    assert gs.gespmm_plan_b16(10**6, 64, 10**8, "f32") == gs.gespmm_plan(10**6, 64, 10**8)


def test_version_and_status_strings(L):
    assert gs.gespmm_version() >= 100
    seen = {gs.gespmm_status_string(s) for s in range(0, 5)}
    assert len(seen) == 5 and all(seen)
    assert "unknown" in gs.gespmm_status_string(99)


def test_argument_errors_come_before_any_device_work(L):
    p = ctypes.c_void_p(0x1000)      # never dereferenced on the host
    call = L.gespmm_csr
    assert call(-1, 4, 4, 0, p, p, p, p, p, 0, None) == 1
    assert call(4, 4, 4, -3, p, p, p, p, p, 0, None) == 1
    assert call(4, 4, 4, 8, p, p, p, p, p, 7, None) == 1          # unknown op
    assert call(4, 4, 4, 8, p, p, p, p, p, -1, None) == 1
    assert call(0, 4, 4, 8, p, p, p, p, p, 0, None) == 1          # entries without rows
    assert call(4, 4, 4, 8, None, p, p, p, p, 0, None) == 2       # rowptr NULL
    assert call(4, 4, 4, 8, p, None, p, p, p, 0, None) == 2       # colind NULL with nnz > 0
    assert call(4, 4, 4, 8, p, p, p, None, p, 0, None) == 2       # B NULL
    assert call(4, 4, 4, 8, p, p, p, p, None, 0, None) == 2       # C NULL
    assert call(2**31, 4, 4, 8, p, p, p, p, p, 0, None) == 3
    assert call(4, 2**31 + 1, 4, 8, p, p, p, p, p, 0, None) == 3
    assert call(4, 4, 4, 2**31, p, p, p, p, p, 0, None) == 3
    assert call(4, 4, 40_000_000, 8, p, p, p, p, p, 0, None) == 3  # more column blocks than a grid holds
    # nothing to do: success without touching a device
    assert call(0, 4, 4, 0, p, p, p, p, p, 0, None) == 0
    assert call(4, 4, 0, 8, p, p, p, p, p, 0, None) == 0
    assert L.gespmm_csr_simple(-1, 4, 4, p, p, p, p, p, 0, None) == 1
    assert L.gespmm_csr_simple(4, 4, 4, None, p, p, p, p, 0, None) == 2
    assert L.gespmm_csr_simple(0, 4, 4, p, p, p, p, p, 0, None) == 0
    # gradient-side entry points
    assert L.gespmm_csr_arg(4, 4, 4, 8, p, p, p, p, p, p, 0, None) == 1      # sum has no position
    assert L.gespmm_csr_arg(4, 4, 4, 8, p, p, p, p, p, None, 2, None) == 2   # arg NULL
    assert L.gespmm_csr_arg(4, 4, 4, -1, p, p, p, p, p, p, 2, None) == 1
    assert L.gespmm_csr_arg(0, 4, 4, 0, p, p, p, p, p, p, 3, None) == 0
    assert L.gespmm_csr_transposed(4, 4, 4, 8, p, p, p, p, p, 2, None) == 1  # max has no transposed sum
    assert L.gespmm_csr_transposed(4, 4, 4, 8, p, p, p, p, None, 0, None) == 2
    assert L.gespmm_csr_transposed(4, 4, 4, 8, None, p, p, p, p, 1, None) == 2
    assert L.gespmm_csr_transposed(4, 2**31 + 1, 4, 8, p, p, p, p, p, 0, None) == 3
    assert L.gespmm_csr_transposed(4, 0, 4, 0, p, p, p, p, p, 0, None) == 0
    assert L.gespmm_pool_backward(4, 4, 4, 8, p, p, None, p, p, None) == 2
    assert L.gespmm_pool_backward(4, 4, 4, 8, p, p, p, p, None, None) == 2
    assert L.gespmm_pool_backward(-4, 4, 4, 8, p, p, p, p, p, None) == 1
    assert L.gespmm_pool_backward(4, 4, 0, 8, p, p, p, p, p, None) == 0
    need = gs.gespmm_csr_transpose_workspace_bytes(4)
    assert need >= 4 * 4 and gs.gespmm_csr_transpose_workspace_bytes(10**6) >= 4 * 10**6
    assert L.gespmm_csr_transpose(4, 4, 8, p, p, p, 0, p, p, p, p, need - 1, None) == 4    # workspace too small
    assert L.gespmm_csr_transpose(4, 4, 8, p, p, p, 0, p, p, p, None, need, None) == 2
    assert L.gespmm_csr_transpose(4, 4, 8, p, p, p, 0, None, p, p, p, need, None) == 2
    assert L.gespmm_csr_transpose(4, 4, 8, p, p, p, 0, p, None, p, p, need, None) == 2
    assert L.gespmm_csr_transpose(4, -4, 8, p, p, p, 0, p, p, p, p, need, None) == 1
    assert L.gespmm_csr_transpose(4, 2**31, 8, p, p, p, 0, p, p, p, p, 2**40, None) == 3
    assert L.gespmm_csr_transpose_noalloc(4, 2097153, 8, p, p, p, 0, p, p, p, None) == 6    # beyond the built-in scratch
    assert L.gespmm_csr_transpose_noalloc(4, 4, 8, p, p, p, 0, p, None, p, None) == 2
    assert L.gespmm_plan(4, 4, 4, 1, None) == 2
    assert L.gespmm_profiler_finish(None, None, None) == 2        # no profiler
    assert L.gespmm_profiler_create(0, ctypes.byref(ctypes.c_void_p())) == 1
    assert L.gespmm_profiler_create(4, None) == 2
    ex = L.gespmm_csr_ex
    assert ex(4, 4, 4, 8, p, p, p, p, 7, p, 0, None, 0, None, None, None) == 1       # unknown element type
    assert ex(4, 4, 4, 8, p, p, p, None, 0, p, 0, None, 0, None, None, None) == 2    # B NULL
    assert ex(-4, 4, 4, 8, p, p, p, p, 0, p, 0, None, 0, None, None, None) == 1
    bad = gs.gespmm_tuning_t(3, -1, -1, -1, -1, -1)                                    # 3 lanes per row: no such kernel
    assert ex(4, 4, 4, 8, p, p, p, p, 0, p, 0, None, 0, ctypes.byref(bad), None, None) == 1
    forced = gs.gespmm_tuning_t(-1, -1, -1, -1, -1, 4)                                 # phases forced without a workspace
    assert ex(4, 4, 4, 8, p, p, p, p, 0, p, 0, None, 0, ctypes.byref(forced), None, None) == 4
    assert ex(4, 4, 4, 8, p, p, p, p, 0, p, 0, p, 8, ctypes.byref(forced), None, None) == 4   # workspace too small
    assert L.gespmm_csr_arg_ex(4, 4, 4, 8, p, p, p, p, 0, p, p, 0, None, None) == 1     # sum has no position
    assert L.gespmm_csr_arg_ex(4, 4, 4, 8, p, p, p, p, 0, p, p, 2, ctypes.byref(bad), None) == 1
    assert L.gespmm_calibration_copy(p, p, 24, None) == 1         # not a multiple of 16
    assert L.gespmm_calibration_copy(None, p, 32, None) == 2
    assert L.gespmm_calibration_copy(p, ctypes.c_void_p(0x1004), 32, None) == 1
    assert L.gespmm_calibration_copy(p, p, 0, None) == 0


@pytest.mark.parametrize("N,G,T,blocks", [(8, 2, 1, 1), (16, 4, 1, 1), (32, 8, 1, 1), (64, 8, 1, 2),
                                          (128, 16, 1, 2), (256, 16, 1, 4), (512, 16, 1, 8),
                                          (1024, 16, 1, 16), (4, 1, 1, 1), (100, 8, 1, 4)])
def test_plan_covers_all_columns_vectorised(N, G, T, blocks):
    p = gs.gespmm_plan(1000, N, 10_000)
    assert p["vec"] == 4 and (p["lanes_per_row"], p["tiles_per_lane"], p["col_blocks"]) == (G, T, blocks)
    if N == 128:              # exactly four lines of columns: one line per block when rows are long (mean row >= 28)
        q = gs.gespmm_plan(1000, N, 40_000)
        assert (q["lanes_per_row"], q["col_blocks"]) == (8, 4)
    assert p["vec"] * G * T * blocks >= N and p["slots"] * G == 64
    assert p["chunks"] == -(-(10_000 + 1000) // p["chunk_nnz"])      # items: stored entries + row ends
    assert p["grid_x"] * (p["block_threads"] // 64) >= p["chunks"]


@pytest.mark.parametrize("N,aligned", [(1, True), (3, True), (7, False), (33, True), (100, False), (64, False)])
def test_plan_scalar_path(N, aligned):
    p = gs.gespmm_plan(10, N, 50, aligned16=aligned)
    assert p["vec"] == (4 if (aligned and N % 4 == 0) else 1)
    assert p["vec"] * p["lanes_per_row"] * p["tiles_per_lane"] * p["col_blocks"] >= N


def test_tuning_override_is_validated():
    plan = lambda **t: gs.gespmm_plan_ex(1000, 1000, 64, 10_000, tuning=t)
    for bad in (dict(lanes_per_row=3), dict(tiles_per_lane=3), dict(lanes_per_row=2, tiles_per_lane=4),   # no such kernel
                dict(chunk_nnz=100), dict(chunk_nnz=2048), dict(chunk_nnz=8), dict(short_len=5000), dict(xcd_remap=5000),
                dict(k_parts=65)):
        with pytest.raises(gs.GespmmError):
            plan(**bad)
    p = plan(lanes_per_row=32, tiles_per_lane=1, xcd_remap=0)
    assert (p["lanes_per_row"], p["tiles_per_lane"], p["xcd_remap"], p["col_blocks"]) == (32, 1, 0, 1)
    p = plan(chunk_nnz=1024, short_len=5)
    assert (p["lanes_per_row"], p["chunk_nnz"], p["short_len"], p["chunks"]) == (8, 1024, 5, 11)
    assert p["lds_bytes"] == 4 * (1024 + 64) * 8
    assert gs.gespmm_plan(1000, 64, 10_000)["lanes_per_row"] == 8           # nothing sticks between calls
    assert plan(xcd_remap=16)["xcd_remap"] == 16                            # runs of 16 workgroups per XCD


def test_plan_xcd_mapping_rule():
    """Round-robin runs of workgroups per XCD on the plain path (shorter runs for small grids), one contiguous range
    per XCD for long rows, as dispatched on the K-phased path."""
    assert gs.gespmm_plan(1_000_000, 128, 6_000_000)["xcd_remap"] == 32
    assert gs.gespmm_plan(20_000, 128, 90_000)["xcd_remap"] in (2, 4, 8, 16)
    assert gs.gespmm_plan(100, 128, 400)["xcd_remap"] == 0
    assert gs.gespmm_plan(40_000, 128, 40_000 * 600)["xcd_remap"] == 1
    p = gs.gespmm_plan_ex(232_965, 232_965, 64, 114_000_000, workspace_bytes=1 << 30)
    assert p["k_parts"] > 1 and p["xcd_remap"] == 0


def test_two_threads_with_different_tunings_get_their_own_plans():
    """Tuning is an argument of the call, not process-wide state: plans computed at the same time from
    several threads with different overrides never see each other's values."""
    import threading
    wrong = []

    def worker(G, chunk):
        for _ in range(3000):
            p = gs.gespmm_plan_ex(5000, 5000, 256, 400_000, tuning=dict(lanes_per_row=G, chunk_nnz=chunk))
            if (p["lanes_per_row"], p["chunk_nnz"]) != (G, chunk):
                wrong.append((G, chunk, p))
            q = gs.gespmm_plan_ex(5000, 5000, 256, 400_000)
            if (q["lanes_per_row"], q["chunk_nnz"]) != (16, 256):
                wrong.append(("auto", q))

    threads = [threading.Thread(target=worker, args=a) for a in ((8, 64), (32, 1024), (64, 128), (4, 512))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not wrong, wrong[:3]


def test_k_phased_path_is_planned_for_large_features_and_long_rows():
    big = dict(workspace_bytes=1 << 40)
    p = gs.gespmm_plan_ex(232_965, 232_965, 64, 114_693_532, **big)             # workload 4: B is 60 MB, mean row 492
    assert p["k_parts"] >= 8 and p["lanes_per_row"] == 16 and p["col_blocks"] == 1 and p["workspace_bytes"] > 0
    assert p["workspace_bytes"] == gs.gespmm_csr_workspace_bytes(232_965, 232_965, 64, 114_693_532)
    assert p["workspace_bytes"] >= 4 * p["k_parts"] * (2 * 232_965 + 1)
    assert gs.gespmm_plan_ex(232_965, 232_965, 64, 114_693_532)["k_parts"] == 1     # no workspace, no phases
    assert gs.gespmm_plan_ex(232_965, 232_965, 64, 114_693_532, workspace_bytes=1000)["k_parts"] == 1
    assert gs.gespmm_plan_ex(232_965, 232_965, 64, 114_693_532, tuning=dict(k_parts=1), **big)["k_parts"] == 1
    assert gs.gespmm_plan_ex(232_965, 232_965, 64, 114_693_532, tuning=dict(k_parts=5), **big)["k_parts"] == 5
    # short rows or a B that fits the caches: the plain path
    assert gs.gespmm_plan_ex(1_000_000, 1_000_000, 32, 15_357_733, **big)["k_parts"] == 1
    assert gs.gespmm_plan_ex(20_000, 20_000, 64, 10_000_000, **big)["k_parts"] == 1
    assert gs.gespmm_csr_workspace_bytes(1_000_000, 1_000_000, 32, 15_357_733) == 0
    # 40,000 rows of 130 entries: two parts where the plain path's column block (256 bytes at N = 512) sees 10 MB of B,
    # none where it sees 5 MB (128-byte blocks at N = 128)
    assert gs.gespmm_plan_ex(40_000, 40_000, 512, 5_165_394, **big)["k_parts"] == 2
    assert gs.gespmm_plan_ex(40_000, 40_000, 256, 5_165_394, **big)["k_parts"] == 2
    assert gs.gespmm_plan_ex(40_000, 40_000, 128, 5_165_394, **big)["k_parts"] == 1


def test_whole_row_path_is_planned_only_from_a_bound_on_the_longest_row():
    plan = gs.gespmm_plan_ex
    assert plan(19_717, 19_717, 128, 88_648)["row_window"] == 0                       # nothing known: rows are split
    assert plan(19_717, 19_717, 128, 88_648, tuning=dict(longest_row=0))["row_window"] == 0
    p = plan(19_717, 19_717, 128, 88_648, tuning=dict(longest_row=173))               # a small problem: up to 1024
    assert p["row_window"] == p["chunk_nnz"] + 173 and p["lds_bytes"] == 4 * (p["row_window"] + 64) * 8
    assert plan(19_717, 19_717, 128, 88_648, tuning=dict(longest_row=1025))["row_window"] == 0
    # a problem that fills the chip: only rows that are short against a chunk, and a mean row of at least 8
    p = plan(1_000_000, 1_000_000, 128, 10_000_000, tuning=dict(longest_row=27))
    assert p["chunk_nnz"] == 256 and p["row_window"] == 256 + 27
    assert plan(1_000_000, 1_000_000, 128, 10_000_000, tuning=dict(longest_row=256))["row_window"] == 512
    assert plan(1_000_000, 1_000_000, 128, 10_000_000, tuning=dict(longest_row=257))["row_window"] == 0
    assert plan(1_000_000, 1_000_000, 128, 5_000_000, tuning=dict(longest_row=5))["row_window"] == 0
    # the K-phased path keeps its own kernels; 16-bit features have whole-row kernels too; LDS per workgroup stays within 64 KB
    assert plan(232_965, 232_965, 64, 114_693_532, workspace_bytes=1 << 40, tuning=dict(longest_row=100))["row_window"] == 0
    assert plan(19_717, 19_717, 128, 88_648, "bf16", tuning=dict(longest_row=173))["row_window"] > 0
    assert plan(1000, 1000, 64, 10_000, tuning=dict(longest_row=1000, chunk_nnz=1024))["row_window"] == 0
    assert plan(1000, 1000, 64, 10_000, tuning=dict(longest_row=960, chunk_nnz=1024))["row_window"] == 1984


def test_chunk_size_follows_width_and_problem_size():
    big = 100_000_000
    plans = [gs.gespmm_plan(10**6, N, big) for N in (8, 16, 32, 64, 128, 512)]
    assert [p["chunk_nnz"] for p in plans] == [1024, 512, 256, 256, 256, 256]
    # ... 1024 only while thousands of chunks remain, and up to N = 32 when the caller bounds the rows by 64 entries
    assert gs.gespmm_plan(169_343, 8, 2_330_033)["chunk_nnz"] == 512
    bounded = lambda N, L: gs.gespmm_plan_ex(524_288, 524_288, N, 2_099_988, tuning=dict(longest_row=L))["chunk_nnz"]
    assert [bounded(N, 16) for N in (8, 16, 32, 64)] == [1024, 1024, 1024, 256] and bounded(32, 65) == 256
    assert [p["short_len"] for p in plans] == [32, 32, 16, 16, 16, 16]
    # long rows (mean length >= 128): larger chunks, fewer split rows
    assert gs.gespmm_plan(232_965, 64, 114_693_532)["chunk_nnz"] == 512
    # the phases of the K-phased path: 1024 while a phase still has thousands of chunks
    assert gs.gespmm_plan_ex(232_965, 232_965, 64, 114_693_532, workspace_bytes=1 << 30)["chunk_nnz"] == 1024
    assert gs.gespmm_plan_ex(40_000, 40_000, 512, 5_165_394, workspace_bytes=1 << 30)["chunk_nnz"] == 512
    assert all(p["lds_bytes"] == 4 * (p["chunk_nnz"] + 64) * 8 for p in plans)
    assert all(p["chunks"] == -(-(big + 10**6) // p["chunk_nnz"]) for p in plans)
    # small problems: smaller chunks, so the rows spread over more wavefronts
    # (fewer than 2048 wavefronts over all column blocks -> halve, down to 64 entries)
    assert [gs.gespmm_plan(19717, N, 88_648)["chunk_nnz"] for N in (32, 64, 128, 256, 512)] == [64, 64, 64, 128, 256]
    assert gs.gespmm_plan(2708, 16, 10_556)["chunk_nnz"] == 64
    assert gs.gespmm_plan(65_536, 512, 649_959)["chunk_nnz"] == 256
    # ... unless the rows are long: every chunk a row crosses costs its outputs one more rounding
    assert gs.gespmm_plan(2, 8, 100_000)["chunk_nnz"] == 512
    # mean row of 17 .. 48 entries: one slot per row up to 32 entries
    assert [gs.gespmm_plan(262_144, N, 6_859_000)["short_len"] for N in (32, 128, 512)] == [32, 32, 32]
    assert gs.gespmm_plan(100_000, 128, 1_600_000)["short_len"] == 16
    assert gs.gespmm_plan(100_000, 128, 4_900_000)["short_len"] == 16
    p = gs.gespmm_plan(169_343, 128, 2_330_033)
    assert p["chunk_nnz"] == 256 and p["xcd_remap"] == 32        # runs of 32 workgroups per XCD
    # rows much longer than a chunk: consecutive chunks stay on one XCD
    assert gs.gespmm_plan(232_965, 64, 114_693_532)["xcd_remap"] == 1


def test_header_is_plain_c_and_cxx():
    """include/gespmm.h must compile on its own as C99 and as C++11 (no HIP or torch types in it)."""
    import subprocess
    for cmd in (["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", HEADER],
                ["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", HEADER]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    text = open(HEADER).read()
    assert "hip/" not in text and "torch" not in text.lower()


def test_run_time_reduce_host_side_argument_checks(L):
    handle = ctypes.c_void_p()
    log = ctypes.create_string_buffer(64)
    src = b"struct A { static __device__ float identity() { return 0.0f; } };"
    assert L.gespmm_custom_op_create(None, b"A", ctypes.byref(handle), log, 64) == 2
    assert L.gespmm_custom_op_create(src, None, ctypes.byref(handle), log, 64) == 2
    assert L.gespmm_custom_op_create(src, b"A", None, log, 64) == 2
    for bad in (b"", b"1A", b"A B", b"A;", b"A<int>", b":A"):
        assert L.gespmm_custom_op_create(src, bad, ctypes.byref(handle), None, 0) == 1, bad
        assert not handle.value
    assert L.gespmm_custom_op_destroy(None) == 0
    assert L.gespmm_csr_custom(None, 1, 1, 1, 0, None, None, None, None, None, None, None) == 2
    assert "compile" in gs.gespmm_status_string(7) and "libhiprtc" in gs.gespmm_status_string(8)


def test_embedded_device_header_is_the_header():
    """The text handed to the run-time compiler is include/gespmm_device.hpp, byte for byte."""
    path = hip_build.embed_device_header()
    pieces = re.findall(r'R"GESPMM_TEXT\((.*?)\)GESPMM_TEXT"\n', open(path).read(), flags=re.S)
    assert "".join(pieces) == open(os.path.join(ROOT, "include", "gespmm_device.hpp")).read()
    # device code only: nothing in it may need a host header when the run-time compiler reads it
    device = open(os.path.join(ROOT, "include", "gespmm_device.hpp")).read()
    includes = re.findall(r"#include\s*[<\"]([^>\"]+)[>\"]", device)
    assert sorted(includes) == ["cstdint", "hip/hip_runtime.h"], includes


def test_run_time_reduce_compiles_without_a_gpu():
    """The text of a user-defined reduce goes through the run-time compiler together with the embedded kernel header,
    for gfx950, on a machine without a GPU: a good text compiles, a broken one and one without step() are reported."""
    good = """struct SumOfSquares {
      static __device__ float identity() { return 0.0f; }
      static __device__ float step(float acc, float a, float b) { const float x = a * b; return acc + x * x; }
      static __device__ float merge(float x, float y) { return x + y; } };"""
    try:
        gs.gespmm_custom_op_check(good, "SumOfSquares")
    except gs.GespmmError as e:
        if e.status == 8:
            pytest.skip("libhiprtc.so is not installed here")
        raise
    with pytest.raises(gs.GespmmError) as e:
        gs.gespmm_custom_op_check("struct Broken { static __device__ float identity() { return 0.0f } };", "Broken")
    assert e.value.status == 7 and "error" in e.value.log
    with pytest.raises(gs.GespmmError) as e:
        gs.gespmm_custom_op_check("""struct NoStep { static __device__ float identity() { return 0.0f; }
                                     static __device__ float merge(float x, float y) { return x + y; } };""", "NoStep")
    assert e.value.status == 7 and "step" in e.value.log
    with pytest.raises(gs.GespmmError) as e:
        gs.gespmm_custom_op_check(good, "Sum Of Squares")
    assert e.value.status == 1
