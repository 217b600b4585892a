"""ctypes binding of libmoe_sb: argument marshalling only.

Every function has the name and meaning of the C entry point it forwards to
(see include/moe_sb.h).  Tensors are torch tensors used purely as device
buffers; the current torch stream is passed as the hipStream_t.  If the
compiled library is missing, importing the functions fails: there is no
fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_sb.so")

MOE_OK = 0
MOE_ERR_INVALID_ARG = -1
MOE_ERR_UNSUPPORTED = -2
MOE_ERR_ROUTING = -3
MOE_ERR_HIP = -4
MOE_ERR_TOO_LARGE = -5
MOE_DTYPE_BF16 = 0
MOE_DTYPE_FP8_E4M3 = 1
MOE_W_LAYOUT_KN = 0
MOE_W_LAYOUT_NK = 1
MOE_EPILOGUE_NONE = 0
MOE_EPILOGUE_SWIGLU = 1
MOE_ORDER_ASCENDING = 0
MOE_ORDER_SPREAD = 1
MOE_ORDER_INTERLEAVE = 2
MOE_LAUNCH_AUTO = 0
MOE_LAUNCH_PER_TILE = 1
MOE_LAUNCH_RESIDENT = 2
MOE_MAP_MAGIC = 0x3142534D
MOE_MAP_HDR_WORDS = 32
HDR = dict(MAGIC=0, T=1, K_TOP=2, E=3, N=4, TILE_M=5, TILE_N=6, NT=7, M=8, TOTAL_TILES=9, ORDER=10,
           STATUS=11, R=12, E64=13, SIGMA_ORDER=14, TILE_M_SMALL=15,
           SMALL_MAX_ROWS=16, TILE_M_SLACK=17, HEAVY_TILES=18)

EXPORTS = [
    "moe_map_off_counts", "moe_map_off_offsets", "moe_map_off_sigma", "moe_map_off_tile_prefix",
    "moe_map_off_task_records", "moe_map_off_sorted_rows", "moe_task_map_bytes", "moe_grid_upper_bound", "moe_build_task_map",
    "moe_build_task_map_ordered", "moe_build_task_map_tiled", "moe_grid_upper_bound_tiled", "moe_tile_pair_supported",
    "moe_build_task_map_ex", "moe_tiling_supported", "moe_w_layout_supported", "moe_default_tiling",
    "moe_task_map_status", "moe_task_map_expand", "moe_grouped_gemm", "moe_tile_supported", "moe_combine",
    "moe_grouped_gemm_splitk", "moe_splitk_workspace_bytes", "moe_default_k_parts",
    "moe_grouped_gemm_splitk_static", "moe_splitk_static_scratch_bytes",
    "moe_grouped_gemm_batched", "moe_reduce_task_tiles", "moe_grouped_gemm_tail_split", "moe_tail_split_workspace_bytes",
    "moe_strerror",
]


class MoeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class moe_gemm_desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("T", ctypes.c_int32), ("k", ctypes.c_int32), ("E", ctypes.c_int32),
                ("K", ctypes.c_int32), ("N", ctypes.c_int32), ("tile_m", ctypes.c_int32),
                ("tile_n", ctypes.c_int32), ("x_scale", ctypes.c_void_p), ("w_scale", ctypes.c_void_p),
                ("tile_m_small", ctypes.c_int32), ("small_max_rows", ctypes.c_int32),
                ("tile_m_slack", ctypes.c_int32), ("epilogue", ctypes.c_int32), ("w_layout", ctypes.c_int32),
                ("launch_mode", ctypes.c_int32)]


class moe_reduce_task(ctypes.Structure):
    _fields_ = [("Y", ctypes.c_void_p), ("topk_weights", ctypes.c_void_p), ("T", ctypes.c_int32), ("k", ctypes.c_int32),
                ("N", ctypes.c_int32), ("out", ctypes.c_void_p)]


class moe_tiling(ctypes.Structure):
    _fields_ = [("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32), ("order", ctypes.c_int32),
                ("tile_m_small", ctypes.c_int32), ("small_max_rows", ctypes.c_int32),
                ("tile_m_slack", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2501_16103_amd.build` "
                              "(or __graft_entry__.build()). There is no fallback implementation.")
        L = ctypes.CDLL(LIB_PATH)
        for n in ("moe_map_off_counts", "moe_map_off_offsets", "moe_map_off_sigma", "moe_map_off_tile_prefix",
                  "moe_map_off_task_records", "moe_map_off_sorted_rows"):
            getattr(L, n).restype = ctypes.c_size_t
            getattr(L, n).argtypes = [ctypes.c_int]
        L.moe_task_map_bytes.restype = ctypes.c_size_t
        L.moe_task_map_bytes.argtypes = [ctypes.c_int] * 6
        L.moe_grid_upper_bound.restype = ctypes.c_int64
        L.moe_grid_upper_bound.argtypes = [ctypes.c_int] * 6
        L.moe_build_task_map.restype = ctypes.c_int
        L.moe_build_task_map.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p]
        L.moe_build_task_map_ordered.restype = ctypes.c_int
        L.moe_build_task_map_ordered.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 7 + [ctypes.c_void_p, ctypes.c_void_p]
        L.moe_build_task_map_tiled.restype = ctypes.c_int
        L.moe_build_task_map_tiled.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 9 + [ctypes.c_void_p, ctypes.c_void_p]
        L.moe_grid_upper_bound_tiled.restype = ctypes.c_int64
        L.moe_grid_upper_bound_tiled.argtypes = [ctypes.c_int] * 8
        L.moe_tile_pair_supported.restype = ctypes.c_int
        L.moe_tile_pair_supported.argtypes = [ctypes.c_int] * 4
        L.moe_build_task_map_ex.restype = ctypes.c_int
        L.moe_build_task_map_ex.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.POINTER(moe_tiling),
                                                                                      ctypes.c_void_p, ctypes.c_void_p]
        L.moe_tiling_supported.restype = ctypes.c_int
        L.moe_tiling_supported.argtypes = [ctypes.c_int, ctypes.POINTER(moe_tiling)]
        L.moe_default_tiling.restype = ctypes.c_int
        L.moe_default_tiling.argtypes = [ctypes.c_int] * 6 + [ctypes.POINTER(moe_tiling)]
        L.moe_w_layout_supported.restype = ctypes.c_int
        L.moe_w_layout_supported.argtypes = [ctypes.c_int, ctypes.POINTER(moe_tiling), ctypes.c_int]
        L.moe_task_map_status.restype = ctypes.c_int
        L.moe_task_map_status.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        L.moe_task_map_expand.restype = ctypes.c_int
        L.moe_task_map_expand.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        L.moe_grouped_gemm.restype = ctypes.c_int
        L.moe_grouped_gemm.argtypes = [ctypes.c_void_p] * 5 + [ctypes.POINTER(moe_gemm_desc), ctypes.c_void_p]
        L.moe_tile_supported.restype = ctypes.c_int
        L.moe_tile_supported.argtypes = [ctypes.c_int] * 3
        L.moe_combine.restype = ctypes.c_int
        L.moe_combine.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                  ctypes.c_void_p, ctypes.c_void_p]
        L.moe_grouped_gemm_splitk.restype = ctypes.c_int
        L.moe_grouped_gemm_splitk.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.POINTER(moe_gemm_desc), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                              ctypes.c_void_p]
        L.moe_grouped_gemm_splitk_static.restype = ctypes.c_int
        L.moe_grouped_gemm_splitk_static.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                     ctypes.POINTER(moe_gemm_desc), ctypes.c_int, ctypes.c_void_p]
        L.moe_splitk_static_scratch_bytes.restype = ctypes.c_size_t
        L.moe_splitk_static_scratch_bytes.argtypes = []
        L.moe_grouped_gemm_batched.restype = ctypes.c_int
        L.moe_grouped_gemm_batched.argtypes = [ctypes.c_void_p] * 4 + [ctypes.POINTER(moe_gemm_desc),
                                                                       ctypes.POINTER(moe_reduce_task), ctypes.c_void_p]
        L.moe_reduce_task_tiles.restype = ctypes.c_int64
        L.moe_reduce_task_tiles.argtypes = [ctypes.c_int, ctypes.c_int]
        L.moe_grouped_gemm_tail_split.restype = ctypes.c_int
        L.moe_grouped_gemm_tail_split.argtypes = [ctypes.c_void_p] * 4 + [ctypes.POINTER(moe_gemm_desc), ctypes.c_void_p,
                                                                          ctypes.c_size_t, ctypes.c_void_p]
        L.moe_tail_split_workspace_bytes.restype = ctypes.c_size_t
        L.moe_tail_split_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int]
        L.moe_splitk_workspace_bytes.restype = ctypes.c_size_t
        L.moe_splitk_workspace_bytes.argtypes = [ctypes.c_int] * 4
        L.moe_default_k_parts.restype = ctypes.c_int
        L.moe_default_k_parts.argtypes = [ctypes.c_int] * 5
        L.moe_strerror.restype = ctypes.c_char_p
        L.moe_strerror.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().moe_strerror(code).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def moe_task_map_bytes(T_max: int, k: int, E: int, tile_m: int, tile_n: int, N: int) -> int:
    return int(lib().moe_task_map_bytes(T_max, k, E, tile_m, tile_n, N))


def moe_grid_upper_bound(T: int, k: int, E: int, tile_m: int, tile_n: int, N: int) -> int:
    return int(lib().moe_grid_upper_bound(T, k, E, tile_m, tile_n, N))


def moe_tile_supported(dtype: int, tile_m: int, tile_n: int) -> bool:
    return bool(lib().moe_tile_supported(dtype, tile_m, tile_n))


def moe_map_offsets(E: int) -> dict:
    L = lib()
    return dict(counts=int(L.moe_map_off_counts(E)), offsets=int(L.moe_map_off_offsets(E)),
                sigma=int(L.moe_map_off_sigma(E)), tile_prefix=int(L.moe_map_off_tile_prefix(E)),
                task_records=int(L.moe_map_off_task_records(E)),
                sorted_rows=int(L.moe_map_off_sorted_rows(E)))


def alloc_task_map(T_max: int, k: int, E: int, tile_m: int, tile_n: int, N: int, device="cuda") -> torch.Tensor:
    nbytes = moe_task_map_bytes(T_max, k, E, tile_m, tile_n, N)
    if nbytes == 0:
        raise MoeError(MOE_ERR_INVALID_ARG, "moe_task_map_bytes")
    return torch.empty(nbytes // 4, dtype=torch.int32, device=device)


def moe_build_task_map(topk_ids: torch.Tensor, T: int, k: int, E: int, tile_m: int, tile_n: int, N: int,
                       task_map: torch.Tensor, check: bool = True) -> int:
    rc = lib().moe_build_task_map(_ptr(topk_ids), T, k, E, tile_m, tile_n, N, _ptr(task_map), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_build_task_map")
    return rc


def moe_build_task_map_ordered(topk_ids: torch.Tensor, T: int, k: int, E: int, tile_m: int, tile_n: int, N: int,
                               order: int, task_map: torch.Tensor, check: bool = True) -> int:
    rc = lib().moe_build_task_map_ordered(_ptr(topk_ids), T, k, E, tile_m, tile_n, N, order, _ptr(task_map), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_build_task_map_ordered")
    return rc


def moe_build_task_map_tiled(topk_ids: torch.Tensor, T: int, k: int, E: int, tile_m: int, tile_n: int, N: int,
                             order: int, tile_m_small: int, small_max_rows: int, task_map: torch.Tensor,
                             check: bool = True) -> int:
    rc = lib().moe_build_task_map_tiled(_ptr(topk_ids), T, k, E, tile_m, tile_n, N, order, tile_m_small,
                                        small_max_rows, _ptr(task_map), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_build_task_map_tiled")
    return rc


def moe_grid_upper_bound_tiled(T: int, k: int, E: int, tile_m: int, tile_n: int, N: int, tile_m_small: int,
                               small_max_rows: int) -> int:
    return int(lib().moe_grid_upper_bound_tiled(T, k, E, tile_m, tile_n, N, tile_m_small, small_max_rows))


def moe_tile_pair_supported(dtype: int, tile_m: int, tile_n: int, tile_m_small: int) -> bool:
    return bool(lib().moe_tile_pair_supported(dtype, tile_m, tile_n, tile_m_small))


@dataclass
class Tiling:
    tile_m: int
    tile_n: int
    order: int = 0
    tile_m_small: int = 0
    small_max_rows: int = 0
    tile_m_slack: int = 0

    def c_struct(self) -> moe_tiling:
        return moe_tiling(self.tile_m, self.tile_n, self.order, self.tile_m_small, self.small_max_rows, self.tile_m_slack)


def moe_build_task_map_ex(topk_ids: torch.Tensor, T: int, k: int, E: int, N: int, tiling: Tiling,
                          task_map: torch.Tensor, check: bool = True) -> int:
    g = tiling.c_struct()
    rc = lib().moe_build_task_map_ex(_ptr(topk_ids), T, k, E, N, ctypes.byref(g), _ptr(task_map), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_build_task_map_ex")
    return rc


def moe_tiling_supported(dtype: int, tiling: Tiling) -> bool:
    g = tiling.c_struct()
    return bool(lib().moe_tiling_supported(dtype, ctypes.byref(g)))


def moe_default_tiling(dtype: int, T: int, k: int, E: int, K: int, N: int) -> Tiling:
    g = moe_tiling()
    rc = lib().moe_default_tiling(dtype, T, k, E, K, N, ctypes.byref(g))
    if rc != MOE_OK:
        raise MoeError(rc, "moe_default_tiling")
    return Tiling(g.tile_m, g.tile_n, g.order, g.tile_m_small, g.small_max_rows, g.tile_m_slack)


def moe_w_layout_supported(dtype: int, tiling: Tiling, w_layout: int) -> bool:
    g = tiling.c_struct()
    return bool(lib().moe_w_layout_supported(dtype, ctypes.byref(g), w_layout))


def moe_task_map_status(task_map: torch.Tensor) -> int:
    return int(lib().moe_task_map_status(_ptr(task_map), _stream()))


def moe_task_map_expand(task_map: torch.Tensor, E: int, table: torch.Tensor, grid: int, check: bool = True) -> int:
    rc = lib().moe_task_map_expand(_ptr(task_map), E, _ptr(table), grid, _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_task_map_expand")
    return rc


@dataclass
class GemmDesc:
    dtype: int
    T: int
    k: int
    E: int
    K: int
    N: int
    tile_m: int
    tile_n: int
    x_scale: Optional[torch.Tensor] = None
    w_scale: Optional[torch.Tensor] = None
    tile_m_small: int = 0
    small_max_rows: int = 0
    tile_m_slack: int = 0
    epilogue: int = 0
    w_layout: int = 0
    launch_mode: int = 0

    def c_struct(self) -> moe_gemm_desc:
        return moe_gemm_desc(self.dtype, self.T, self.k, self.E, self.K, self.N, self.tile_m, self.tile_n,
                             None if self.x_scale is None else self.x_scale.data_ptr(),
                             None if self.w_scale is None else self.w_scale.data_ptr(),
                             self.tile_m_small, self.small_max_rows, self.tile_m_slack, self.epilogue, self.w_layout,
                             self.launch_mode)


def moe_grouped_gemm(X: torch.Tensor, W: torch.Tensor, topk_ids: Optional[torch.Tensor], task_map: torch.Tensor,
                     Y: torch.Tensor, desc: GemmDesc, check: bool = True) -> int:
    d = desc.c_struct()
    rc = lib().moe_grouped_gemm(_ptr(X), _ptr(W), _ptr(topk_ids), _ptr(task_map), _ptr(Y), ctypes.byref(d), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_grouped_gemm")
    return rc


def moe_combine(Y: torch.Tensor, topk_weights: Optional[torch.Tensor], T: int, k: int, N: int, out: torch.Tensor,
                check: bool = True) -> int:
    rc = lib().moe_combine(_ptr(Y), _ptr(topk_weights), T, k, N, _ptr(out), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_combine")
    return rc


def moe_splitk_workspace_bytes(T: int, k: int, N: int, k_parts: int) -> int:
    return int(lib().moe_splitk_workspace_bytes(T, k, N, k_parts))


def moe_default_k_parts(T: int, k: int, E: int, K: int, N: int) -> int:
    rc = lib().moe_default_k_parts(T, k, E, K, N)
    if rc < 1:
        raise MoeError(rc, "moe_default_k_parts")
    return rc


def moe_grouped_gemm_splitk(X: torch.Tensor, W: torch.Tensor, task_map: torch.Tensor, Y: torch.Tensor, desc: "GemmDesc",
                            k_parts: int, workspace: Optional[torch.Tensor], check: bool = True) -> int:
    """Split-k form of moe_grouped_gemm; `workspace`: device tensor of >= moe_splitk_workspace_bytes(...) bytes."""
    c = desc.c_struct()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().moe_grouped_gemm_splitk(_ptr(X), _ptr(W), _ptr(task_map), _ptr(Y), ctypes.byref(c), int(k_parts),
                                       _ptr(workspace), ctypes.c_size_t(nbytes), _stream() if X is not None else None)
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_grouped_gemm_splitk")
    return rc


def moe_tail_split_workspace_bytes(tile_m: int = 256, tile_n: int = 256) -> int:
    return int(lib().moe_tail_split_workspace_bytes(tile_m, tile_n))


def moe_grouped_gemm_tail_split(X: torch.Tensor, W: torch.Tensor, task_map: torch.Tensor, Y: torch.Tensor, desc: "GemmDesc",
                                workspace: Optional[torch.Tensor], check: bool = True) -> int:
    """moe_grouped_gemm with the tiles of a partly filled last round split along K; `workspace`: device tensor of
    >= moe_tail_split_workspace_bytes(tile_m, tile_n) bytes."""
    c = desc.c_struct()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().moe_grouped_gemm_tail_split(_ptr(X), _ptr(W), _ptr(task_map), _ptr(Y), ctypes.byref(c), _ptr(workspace),
                                           ctypes.c_size_t(nbytes), _stream() if X is not None else None)
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_grouped_gemm_tail_split")
    return rc


def moe_reduce_task_tiles(T: int, N: int) -> int:
    return int(lib().moe_reduce_task_tiles(T, N))


def moe_grouped_gemm_batched(X: torch.Tensor, W: torch.Tensor, task_map: torch.Tensor, Y: torch.Tensor, desc: "GemmDesc",
                             red_Y: torch.Tensor, red_weights: Optional[torch.Tensor], red_T: int, red_k: int, red_N: int,
                             red_out: torch.Tensor, check: bool = True) -> int:
    """moe_grouped_gemm with a reduction task (moe_combine's sum over red_Y [red_T, red_k, red_N]) in the same launch."""
    d = desc.c_struct()
    r = moe_reduce_task(None if red_Y is None else red_Y.data_ptr(), None if red_weights is None else red_weights.data_ptr(),
                        red_T, red_k, red_N, None if red_out is None else red_out.data_ptr())
    rc = lib().moe_grouped_gemm_batched(_ptr(X), _ptr(W), _ptr(task_map), _ptr(Y), ctypes.byref(d), ctypes.byref(r), _stream())
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_grouped_gemm_batched")
    return rc


def moe_splitk_static_scratch_bytes() -> int:
    return int(lib().moe_splitk_static_scratch_bytes())


def moe_grouped_gemm_splitk_static(X: torch.Tensor, W: torch.Tensor, task_map: torch.Tensor, Y: torch.Tensor,
                                   desc: "GemmDesc", k_parts: int, check: bool = True) -> int:
    """moe_grouped_gemm_splitk without a workspace: the partial sums go to the library's static device array."""
    c = desc.c_struct()
    rc = lib().moe_grouped_gemm_splitk_static(_ptr(X), _ptr(W), _ptr(task_map), _ptr(Y), ctypes.byref(c), int(k_parts),
                                              _stream() if X is not None else None)
    if check and rc != MOE_OK:
        raise MoeError(rc, "moe_grouped_gemm_splitk_static")
    return rc


class MoeLayerPlan:
    """Buffers and tilings for one bf16 MoE feed-forward layer (Sec. 2.2) run with the library's calls only:

        map(T, k) -> gate+up product with the fused gated activation -> map(T*k, 1) -> down product -> weighted sum.

    The second product sees the T*k activated rows as tokens of their own, each routed to exactly one expert
    (the flattened routing with k = 1), so the same two entry points serve both products (the second one in its
    split-k form, with a workspace held here, where moe_default_k_parts says so).  Nothing here computes:
    the plan holds caller-visible device buffers and issues calls on the current stream."""

    def __init__(self, T: int, k: int, E: int, hidden: int, inter: int, device="cuda:0"):
        self.T, self.k, self.E, self.hidden, self.inter = T, k, E, hidden, inter
        R = T * k
        self.g1 = moe_default_tiling(MOE_DTYPE_BF16, T, k, E, hidden, 2 * inter)
        # the down product is the short-grid case (few experts, N = hidden): split along K where that pays
        self.k_parts = moe_default_k_parts(R, 1, E, inter, hidden) if R > 0 else 1
        self.g2 = Tiling(256, 256) if self.k_parts > 1 else moe_default_tiling(MOE_DTYPE_BF16, R, 1, E, inter, hidden)
        self.workspace = (torch.empty(moe_splitk_workspace_bytes(R, 1, hidden, self.k_parts) // 4, dtype=torch.float32, device=device)
                          if self.k_parts > 1 else None)
        self.map1 = alloc_task_map(T, k, E, self.g1.tile_m, self.g1.tile_n, 2 * inter, device)
        self.map2 = alloc_task_map(R, 1, E, self.g2.tile_m, self.g2.tile_n, hidden, device)
        self.act = torch.empty((R, inter), dtype=torch.bfloat16, device=device)       # [T, k, inter]
        self.down = torch.empty((R, hidden), dtype=torch.bfloat16, device=device)     # [T, k, hidden]
        self.out = torch.empty((T, hidden), dtype=torch.bfloat16, device=device)
        self.d1 = GemmDesc(MOE_DTYPE_BF16, T, k, E, hidden, 2 * inter, self.g1.tile_m, self.g1.tile_n,
                           tile_m_small=self.g1.tile_m_small, small_max_rows=self.g1.small_max_rows,
                           tile_m_slack=self.g1.tile_m_slack, epilogue=MOE_EPILOGUE_SWIGLU)
        self.d2 = GemmDesc(MOE_DTYPE_BF16, R, 1, E, inter, hidden, self.g2.tile_m, self.g2.tile_n,
                           tile_m_small=self.g2.tile_m_small, small_max_rows=self.g2.small_max_rows,
                           tile_m_slack=self.g2.tile_m_slack)

    def forward(self, X: torch.Tensor, W_gate_up: torch.Tensor, W_down: torch.Tensor, topk_ids: torch.Tensor,
                topk_weights: Optional[torch.Tensor]) -> torch.Tensor:
        """X [T, hidden]; W_gate_up [E, hidden, 2*inter] (gate columns first); W_down [E, inter, hidden];
        topk_ids int32 [T, k]; topk_weights fp32 [T, k] or None.  Returns out [T, hidden] (the plan's buffer)."""
        T, k, E = self.T, self.k, self.E
        flat = topk_ids.reshape(T * k, 1)
        moe_build_task_map_ex(topk_ids, T, k, E, 2 * self.inter, self.g1, self.map1)
        moe_grouped_gemm(X, W_gate_up, topk_ids, self.map1, self.act, self.d1)
        moe_build_task_map_ex(flat, T * k, 1, E, self.hidden, self.g2, self.map2)
        if self.k_parts > 1:
            moe_grouped_gemm_splitk(self.act, W_down, self.map2, self.down, self.d2, self.k_parts, self.workspace)
        else:
            moe_grouped_gemm(self.act, W_down, flat, self.map2, self.down, self.d2)
        moe_combine(self.down, topk_weights, T, k, self.hidden, self.out)
        return self.out
