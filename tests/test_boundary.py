"""The C-ABI library loads and exports every symbol include/flover.h declares (no compute without a GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2305_13484_amd as fl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flover.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flover_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = fl.load_library()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(fl.EXPORTED_SYMBOLS) == names


def test_no_extern_c_torch_types_in_header():
    text = open(os.path.join(ROOT, "include", "flover.h")).read()
    assert "torch" not in text and "at::" not in text and "std::" not in text


def test_host_only_entry_point_and_argument_errors():
    lib = fl.load_library()
    assert fl.k_find_window([0, 1, 1, 0, 1, 1]) == (1, 1, 4)
    assert fl.k_find_window([]) == (0, 0, 0)
    n = ctypes.c_uint64()
    assert lib.flover_k_gemm_tiled_bytes(2, 100, 64, ctypes.byref(n)) == 0 and n.value == 128 * 64 * 2
    assert lib.flover_k_gemm_tiled_bytes(2, 100, 48, ctypes.byref(n)) == -1          # K not a multiple of 32
    assert b"bad argument" in lib.flover_last_error(None)
    assert lib.flover_k_attention_workspace_bytes(4, 8, 96, 100, ctypes.byref(n)) == -1   # head_dim 96 unsupported
    from paper_2305_13484_amd.binding import _Config
    cfg = _Config(1, 2, 2, 512, 4, 128, 1376, 2000, 160, 16, -1, 0, 0, 1e-6, 10000.0, None, None, 0)
    assert lib.flover_query_arena_bytes(ctypes.byref(cfg), ctypes.byref(n)) == 0 and n.value > 0
    cfg.hidden = 500
    assert lib.flover_query_arena_bytes(ctypes.byref(cfg), ctypes.byref(n)) == -1


def test_host_window_search_matches_oracle():
    from oracle import oracle as orc
    import flover_synth as synth
    for arr in synth.occupancy_arrays(11, 400, 80):
        assert fl.k_find_window(arr) == orc.find_window(arr)


def test_gemm_slicing_is_a_function_of_the_matrix_shape_only():
    """Host logic behind batch invariance: the fused iteration's K slicing never looks at the row count, covers K
    exactly; a context pass of up to 128 rows keeps it, a longer one picks its own count (at most 16) from its rows."""
    from paper_2305_13484_amd.binding import k_gemm_plan
    for dtype in (1, 2):
        for (N, K) in [(12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008), (32000, 4096), (6144, 2048),
                       (50257, 2048), (19968, 6656), (35840, 6656), (64, 64), (130, 1024)]:
            S, kbs = k_gemm_plan(dtype, N, K)
            KB = K // 32
            assert 1 <= S <= 16 and (S - 1) * kbs < KB <= S * kbs
            for rows in (1, 17, 129, 200, 512, 777, 1024):
                Sc, kc = k_gemm_plan(dtype, N, K, rows)
                assert 1 <= Sc <= 16 and (Sc - 1) * kc < KB <= Sc * kc
                if rows <= 128:
                    assert (Sc, kc) == (S, kbs)
    assert k_gemm_plan(0, 1000, 256) == (1, 8)          # fp32 models: one slice


def test_gated_mlp_workspace_sizes_host_only():
    """Where the gated MLP input is one launch it needs no workspace: up to 128 rows, up to 64 where F > 16384; above
    that the two K halves (or a context pass's slices) go through it."""
    lib = fl.load_library()
    n = ctypes.c_uint64()
    for M in (1, 64, 128):
        assert lib.flover_k_gated_workspace_bytes(2, M, 11008, 4096, ctypes.byref(n)) == 0 and n.value == 0
    assert lib.flover_k_gated_workspace_bytes(2, 129, 11008, 4096, ctypes.byref(n)) == 0
    assert n.value >= 2 * 129 * 22016 * 4 and n.value % 256 == 0
    assert lib.flover_k_gated_workspace_bytes(2, 64, 17920, 6656, ctypes.byref(n)) == 0 and n.value == 0
    assert lib.flover_k_gated_workspace_bytes(2, 65, 17920, 6656, ctypes.byref(n)) == 0 and n.value >= 2 * 65 * 35840 * 4
    assert lib.flover_k_gated_workspace_bytes(2, 8, 48, 512, ctypes.byref(n)) == -1      # F not a multiple of 32
    assert lib.flover_k_gated_workspace_bytes(0, 8, 64, 512, ctypes.byref(n)) == -1      # fp32


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's throughput; asking for more is refused with a message, before anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_profile_summary_splits_a_trace_into_iterations(tmp_path):
    """Host logic of the per-iteration summary of a kernel trace: iterations run from one embedding launch to the next,
    only those with an argmax launch count, busy time is the sum of kernel durations, gaps are start minus previous end."""
    import sqlite3
    from paper_2305_13484_amd import profile_summary as ps
    db = str(tmp_path / "kt.db")
    c = sqlite3.connect(db)
    c.execute("create table kernels(name text, start int, end int)")
    t = 0
    for it in range(4):
        names = ["void flk::embed_kernel<2>", "void flk::add_norm_kernel<2, 1>", "void flk::gemm16_direct_kernel<2, 1, 4, 8, 8>"]
        if it != 2:                                   # iteration 2 is a context pass: no argmax
            names.append("flk::argmax_kernel")
        for n in names:
            c.execute("insert into kernels values(?,?,?)", (n, t, t + 5000))
            t += 7000                                 # 5 us busy, 2 us gap
    c.execute("insert into kernels values(?,?,?)", ("void at::native::something", 1, 2))     # foreign kernels are ignored
    c.commit()
    c.close()
    out = ps.iterations(db)
    assert "fused iterations 3, launches per iteration (median) 4" in out
    assert "kernels busy per iteration: median 20.0 us; iteration span: median 26.0 us" in out
    assert "gaps between consecutive launches of an iteration: median 2.00 us" in out
