"""CPU checks of the boundary: the library loads, exports every declared symbol, and its
host-only entry points behave as include/moe_sb.h states.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2501_16103_amd import binding as mb
from tests import helpers as H

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "moe_sb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = mb.lib()
    names = _declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/moe_sb.h but not exported"
    assert sorted(mb.EXPORTS) == names


def test_probe_library_exports_every_declared_symbol():
    """include/moe_probe.h: the measurement kernels live in a library of their own."""
    from paper_2501_16103_amd import probe
    text = open(os.path.join(ROOT, "include", "moe_probe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(moe_probe_[a-z0-9_]+)\s*\(", text)))
    assert names == sorted(probe.EXPORTS)
    for n in names:
        assert hasattr(probe.lib(), n)
    for n in names:
        assert not hasattr(mb.lib(), n), "the product library must not export measurement kernels"


def test_host_only_entry_points():
    assert mb.moe_task_map_bytes(-1, 2, 8, 16, 128, 256) == 0
    assert mb.moe_task_map_bytes(4, 9, 8, 16, 128, 256) == 0        # k > E
    assert mb.moe_task_map_bytes(4, 2, 8, 48, 128, 256) == 0        # tile_m not supported
    nbytes = mb.moe_task_map_bytes(4096, 2, 8, 256, 256, 28672)
    o = H.blob_offsets(8)
    assert nbytes % 4 == 0 and nbytes // 4 >= o["sorted_rows"] + 8192
    assert mb.moe_task_map_bytes(8192, 8, 256, 256, 256, 4096) > mb.moe_task_map_bytes(128, 8, 256, 256, 256, 4096)
    # documented field offsets
    for E in (1, 8, 64, 70, 256):
        lo = mb.moe_map_offsets(E)
        o = H.blob_offsets(E)
        assert all(lo[f] == o[f] for f in lo)
    # grid bound = (floor(R/tile_m) + min(E,R)) * ceil(N/tile_n)
    assert mb.moe_grid_upper_bound(4096, 2, 8, 256, 256, 28672) == (32 + 8) * 112
    assert mb.moe_grid_upper_bound(1, 6, 64, 16, 64, 2816) == (0 + 6) * 44
    assert mb.moe_grid_upper_bound(0, 2, 8, 16, 128, 512) == 0
    # two strategies: (floor(R/tile_m) + min(E,R)*ceil(small_max/tile_m_small)) * ceil(N/tile_n)
    assert mb.moe_grid_upper_bound_tiled(4096, 8, 64, 256, 256, 2560, 64, 64) == (128 + 64) * 10
    assert mb.moe_grid_upper_bound_tiled(4096, 8, 64, 256, 256, 2560, 64, 200) == (128 + 64 * 4) * 10
    assert mb.moe_grid_upper_bound_tiled(4096, 8, 64, 256, 256, 2560, 0, 0) == mb.moe_grid_upper_bound(4096, 8, 64, 256, 256, 2560)
    assert mb.moe_grid_upper_bound_tiled(4096, 8, 64, 256, 256, 2560, 64, 0) == 0       # invalid pair
    assert mb.moe_tile_pair_supported(mb.MOE_DTYPE_BF16, 256, 256, 64)
    assert not mb.moe_tile_pair_supported(mb.MOE_DTYPE_BF16, 256, 256, 0)
    assert not mb.moe_tile_pair_supported(mb.MOE_DTYPE_FP8_E4M3, 256, 256, 64)
    assert mb.moe_tile_supported(mb.MOE_DTYPE_BF16, 256, 256)
    assert mb.moe_tile_supported(mb.MOE_DTYPE_FP8_E4M3, 16, 128)
    assert mb.moe_tile_supported(mb.MOE_DTYPE_FP8_E4M3, 256, 256)
    assert not mb.moe_tile_supported(mb.MOE_DTYPE_FP8_E4M3, 128, 128)
    assert mb.strerror(mb.MOE_ERR_ROUTING).startswith("routing id")
    assert mb.strerror(0) == "ok"


def test_grid_bound_covers_any_routing(oracle_mod):
    import numpy as np
    rng = np.random.default_rng(0)
    for _ in range(200):
        E = int(rng.integers(1, 40))
        k = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.integers(0, 80))
        tile_m = int(rng.choice([16, 32, 64]))
        ids = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]) if T else np.zeros((0, k), np.int32)
        tm = oracle_mod.build_task_map(ids, T, k, E, tile_m, 64, 128)
        assert tm.total_tiles <= mb.moe_grid_upper_bound(T, k, E, tile_m, 64, 128)


def test_null_arguments_rejected_on_host():
    lib = mb.lib()
    assert lib.moe_build_task_map(None, 4, 2, 8, 16, 128, 256, None, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_task_map_status(None, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_grouped_gemm(None, None, None, None, None, None, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_task_map_expand(None, 8, None, 0, None) == mb.MOE_ERR_INVALID_ARG


def test_mfma_probe_rejects_bad_arguments_before_any_launch():
    from paper_2501_16103_amd import probe
    lib = probe.lib()
    assert lib.moe_probe_mfma(8, 1, 10, None, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_mfma(16, 1, 10, None, None) == mb.MOE_ERR_INVALID_ARG   # no sink
    assert lib.moe_probe_mfma(32, 0, 0, 1, None) == mb.MOE_ERR_INVALID_ARG        # no iterations


def test_pipeline_probe_rejects_bad_arguments_before_any_launch():
    from paper_2501_16103_amd import probe
    lib = probe.lib()
    big, small = ctypes.c_size_t(513 << 20), ctypes.c_size_t(1 << 20)
    assert lib.moe_probe_pipeline(0, 10, 16, big, 16, None) == mb.MOE_ERR_INVALID_ARG     # no such mode
    assert lib.moe_probe_pipeline(13, 10, 16, big, 16, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_pipeline(1, 11, 16, big, 16, None) == mb.MOE_ERR_INVALID_ARG     # odd k-step count
    assert lib.moe_probe_pipeline(1, 0, 16, big, 16, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_pipeline(1, 10, None, big, 16, None) == mb.MOE_ERR_INVALID_ARG   # no source
    assert lib.moe_probe_pipeline(1, 10, 16, big, None, None) == mb.MOE_ERR_INVALID_ARG   # no sink
    assert lib.moe_probe_pipeline(1, 10, 24, big, 16, None) == mb.MOE_ERR_INVALID_ARG     # misaligned source
    assert lib.moe_probe_pipeline(3, 10, 16, ctypes.c_size_t((1 << 20) - 1), 16, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_pipeline(4, 10, 16, small, 16, None) == mb.MOE_ERR_INVALID_ARG   # modes 4 and 12 need 513 MiB
    assert lib.moe_probe_pipeline(12, 10, 16, small, 16, None) == mb.MOE_ERR_INVALID_ARG


def test_splitk_host_functions():
    assert mb.moe_splitk_workspace_bytes(1024, 1, 4096, 2) == 2 * 1024 * 4096 * 4
    assert mb.moe_splitk_workspace_bytes(1024, 1, 4096, 1) == 0
    # 8 experts, N = 4096, K = 14336: split where 256 x 256 tiles would leave CUs idle and experts are not tiny
    assert mb.moe_default_k_parts(1024, 1, 8, 14336, 4096) == 2
    assert mb.moe_default_k_parts(1536, 1, 8, 14336, 4096) == 2
    assert mb.moe_default_k_parts(2048, 1, 8, 14336, 4096) == 1      # 192 tiles expected: enough
    assert mb.moe_default_k_parts(512, 1, 8, 14336, 4096) == 1       # 64 rows per expert: narrower tiles instead
    assert mb.moe_default_k_parts(768, 1, 8, 14336, 4096) == 1
    assert mb.moe_default_k_parts(4096, 2, 8, 4096, 28672) == 1      # the headline shape is never split
    assert mb.moe_default_k_parts(1024, 1, 8, 1024, 4096) == 1       # too few k-tiles to share
    with pytest.raises(mb.MoeError):
        mb.moe_default_k_parts(8, 20, 16, 256, 128)
    # argument checks happen before any launch
    lib = mb.lib()
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, 512, 1, 2, 1024, 256, 256, 256).c_struct()
    assert lib.moe_grouped_gemm_splitk(None, None, None, None, ctypes.byref(d), 2, None, 0, None) == mb.MOE_ERR_INVALID_ARG
    assert lib.moe_grouped_gemm_splitk(16, 16, 16, 16, ctypes.byref(d), 3, 16, 1 << 30, None) == mb.MOE_ERR_UNSUPPORTED
    assert lib.moe_grouped_gemm_splitk(16, 16, 16, 16, None, 2, 16, 1 << 30, None) == mb.MOE_ERR_INVALID_ARG


def test_default_tiling_is_supported_and_matches_the_benchmark_choices():
    """Host-only: the heuristic returns a tiling a kernel exists for, and reproduces the tilings the benchmark
    points were tuned to (slack rows aside, where the heuristic always enables them for 256-row tiles)."""
    from paper_2501_16103_amd import workloads as wk
    # (mixtral_down_zipf at T=256 is tuned by hand to its skewed routing; the heuristic assumes a balanced one)
    pts = [wk.mixtral_up(T) for T in (16, 256, 4096)] + [wk.mixtral_down_zipf(4096)]
    pts += [wk.fine_grained(T) for T in (128, 2048, 8192)] + [wk.decode_fp8(T) for T in (1, 8, 32)] + [wk.paper_eval("worst")]
    for w in pts:
        dt = mb.MOE_DTYPE_FP8_E4M3 if w.dtype == "fp8" else mb.MOE_DTYPE_BF16
        g = mb.moe_default_tiling(dt, w.T, w.k, w.E, w.K, w.N)
        assert mb.moe_tiling_supported(dt, g)
        assert (g.tile_m, g.tile_n) == (w.tile_m, w.tile_n), (w.name, w.T)
    # short grids (8 experts, N = 4096 or 2048): the largest tile that still covers three quarters of the CUs
    for (R, K, N, want) in ((512, 14336, 4096, (128, 128)), (768, 14336, 4096, (128, 128)), (1024, 14336, 4096, (128, 256)),
                            (1536, 14336, 4096, (128, 256)), (2048, 14336, 4096, (256, 256)), (1024, 2048, 2048, (128, 128)),
                            (512, 2048, 2048, (64, 128)), (32, 14336, 4096, (128, 128))):
        g = mb.moe_default_tiling(mb.MOE_DTYPE_BF16, R, 1, 8, K, N)
        assert (g.tile_m, g.tile_n) == want and mb.moe_tiling_supported(mb.MOE_DTYPE_BF16, g), (R, K, N, g)
    # N that only 64-wide tiles divide, and one nothing divides
    g = mb.moe_default_tiling(mb.MOE_DTYPE_FP8_E4M3, 8, 2, 16, 256, 192)
    assert (g.tile_m, g.tile_n) == (16, 64) and mb.moe_tiling_supported(mb.MOE_DTYPE_FP8_E4M3, g)
    with pytest.raises(mb.MoeError):
        mb.moe_default_tiling(mb.MOE_DTYPE_BF16, 8, 2, 16, 256, 100)
    with pytest.raises(mb.MoeError):
        mb.moe_default_tiling(mb.MOE_DTYPE_BF16, 8, 20, 16, 256, 128)


def test_every_scalar_load_in_inline_asm_waits_in_the_same_statement():
    """Host-only source check.  The compiler takes an asm statement's outputs as available when the statement
    ends; a scalar load left in flight across statements can have its destination registers spilled and
    reused before the data arrives (this produced wild row ids once).  So every asm string that issues a
    scalar load must also contain the wait for it."""
    import os
    import re
    root = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2501_16103_amd", "csrc")
    seen = 0
    for name in sorted(os.listdir(root)):
        text = open(os.path.join(root, name)).read()
        for m in re.finditer(r"asm\s+volatile\s*\((.*?)\)\s*;", text, re.S):
            body = m.group(1)
            if "s_load" in body or "s_buffer_load" in body:
                seen += 1
                assert "s_waitcnt lgkmcnt(0)" in body, f"{name}: scalar load without its wait in the same asm statement"
    assert seen >= 1
