"""CPU oracle for the statically batched MoE expert GEMM.  TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front for ``moe_oracle.c`` (plain C, gcc, optional OpenMP
over routed rows).  Nothing here imports or calls the HIP library, and the
product path never imports this package: only tests, the smoke check and the
benchmark's CPU-baseline leg do.

What each call follows in the paper is stated in ``moe_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_bf16_to_f32.restype = ctypes.c_float
        _lib.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.orc_f32_to_bf16_rne.restype = ctypes.c_uint16
        _lib.orc_f32_to_bf16_rne.argtypes = [ctypes.c_float]
        _lib.orc_f64_to_bf16_rne.restype = ctypes.c_uint16
        _lib.orc_f64_to_bf16_rne.argtypes = [ctypes.c_double]
        _lib.orc_e4m3_to_f32.restype = ctypes.c_float
        _lib.orc_e4m3_to_f32.argtypes = [ctypes.c_uint8]
        _lib.orc_build_task_map.restype = ctypes.c_int
        _lib.orc_full_table.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def num_threads() -> int:
    """Threads the OpenMP loops will use (what the CPU baseline reports as cores)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


# ------------------------------------------------------------------ formats
def bf16_to_f32(bits: int) -> float:
    return float(_load().orc_bf16_to_f32(int(bits)))


def f32_to_bf16_rne(x: float) -> int:
    return int(_load().orc_f32_to_bf16_rne(ctypes.c_float(x)))


def f64_to_bf16_rne(x: float) -> int:
    return int(_load().orc_f64_to_bf16_rne(ctypes.c_double(x)))


def e4m3_to_f32(byte: int) -> float:
    return float(_load().orc_e4m3_to_f32(int(byte)))


# ------------------------------------------------------------------ task map
@dataclass
class TaskMap:
    T: int
    k: int
    E: int
    N: int
    tile_m: int
    tile_n: int
    counts: np.ndarray        # [E]
    offsets: np.ndarray       # [E+1]
    sorted_rows: np.ndarray   # [T*k] flat row ids r = t*k+j, grouped by expert
    sigma: np.ndarray         # [M] non-empty -> real expert
    tile_prefix: np.ndarray   # [M] inclusive prefix of tiles per non-empty expert
    M: int
    total_tiles: int
    order: int = 0            # 0: sigma ascending, 1: spread (Sec. 4.2)
    tile_m_small: int = 0     # second tiling strategy: experts with <= small_max_rows rows use this tile_m
    small_max_rows: int = 0
    tile_m_slack: int = 0     # rows the last tile of a tile_m-strategy expert may hold beyond tile_m
    heavy_tiles: int = 0      # order 2: tiles of the heavy experts = block index where the light part begins

    def expert_tile_m(self, e: int) -> int:
        c = int(self.counts[e])
        return self.tile_m_small if (self.small_max_rows > 0 and c <= self.small_max_rows) else self.tile_m

    @property
    def nt(self) -> int:
        return -(-self.N // self.tile_n)


def tile_prefix(nu) -> np.ndarray:
    """Alg. 1 on an explicit list of tile counts."""
    nu = _i32(nu)
    out = np.zeros(len(nu), dtype=np.int32)
    _load().orc_tile_prefix(_p(nu), ctypes.c_int(len(nu)), _p(out))
    return out


def mapping(prefix, B: int):
    """Alg. 2: (h, l) for block index B."""
    prefix = _i32(prefix)
    h = ctypes.c_int32(0)
    l = ctypes.c_int32(0)
    _load().orc_mapping(_p(prefix), ctypes.c_int(len(prefix)), ctypes.c_int(B), ctypes.byref(h), ctypes.byref(l))
    return h.value, l.value


def mapping_two_level(prefix, group: int, B: int):
    """Two-level TilePrefix decode (Sec. 3.1) with groups of `group` tasks: (h, l) for block index B."""
    prefix = _i32(prefix)
    h = ctypes.c_int32(0)
    l = ctypes.c_int32(0)
    _load().orc_mapping_two_level(_p(prefix), ctypes.c_int(len(prefix)), ctypes.c_int(group), ctypes.c_int(B),
                                  ctypes.byref(h), ctypes.byref(l))
    return h.value, l.value


def build_task_map(topk_ids, T: int, k: int, E: int, tile_m: int, tile_n: int, N: int, order: int = 0,
                   tile_m_small: int = 0, small_max_rows: int = 0, tile_m_slack: int = 0) -> TaskMap:
    ids = _i32(topk_ids).reshape(-1)
    assert ids.size == T * k
    counts = np.zeros(E, dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    sorted_rows = np.zeros(max(T * k, 1), dtype=np.int32)
    sigma = np.zeros(max(E, 1), dtype=np.int32)
    prefix = np.zeros(max(E, 1), dtype=np.int32)
    M = ctypes.c_int32(0)
    total = ctypes.c_int32(0)
    heavy = ctypes.c_int32(0)
    rc = _load().orc_build_task_map(_p(ids), ctypes.c_int(T), ctypes.c_int(k), ctypes.c_int(E),
                                    ctypes.c_int(tile_m), ctypes.c_int(tile_n), ctypes.c_int(N), ctypes.c_int(order),
                                    ctypes.c_int(tile_m_small), ctypes.c_int(small_max_rows), ctypes.c_int(tile_m_slack), _p(counts), _p(offsets), _p(sorted_rows), _p(sigma), _p(prefix),
                                    ctypes.byref(M), ctypes.byref(total), ctypes.byref(heavy))
    if rc != 0:
        raise ValueError("routing id outside [0, E)")
    return TaskMap(T, k, E, N, tile_m, tile_n, counts, offsets, sorted_rows[: T * k].copy(),
                   sigma[: M.value].copy(), prefix[: M.value].copy(), M.value, total.value, order,
                   tile_m_small, small_max_rows, tile_m_slack, heavy.value)


def decode_block(tm: TaskMap, B: int):
    """Alg. 4 for block B -> (expert, m_tile, n_tile, rows_in_tile)."""
    out = np.zeros(4, dtype=np.int32)
    _load().orc_decode_block(_p(tm.tile_prefix), _p(tm.sigma), ctypes.c_int(tm.M), _p(tm.counts),
                             ctypes.c_int(tm.tile_m), ctypes.c_int(tm.tile_m_small), ctypes.c_int(tm.small_max_rows), ctypes.c_int(tm.tile_m_slack),
                             ctypes.c_int(B), _p(out))
    return tuple(int(v) for v in out)


def decode_all(tm: TaskMap) -> np.ndarray:
    """Alg. 4 for every block 0..total_tiles-1 -> [total, 4]."""
    out = np.zeros((tm.total_tiles, 4), dtype=np.int32)
    lib = _load()
    row = np.zeros(4, dtype=np.int32)
    for B in range(tm.total_tiles):
        lib.orc_decode_block(_p(tm.tile_prefix), _p(tm.sigma), ctypes.c_int(tm.M), _p(tm.counts),
                             ctypes.c_int(tm.tile_m), ctypes.c_int(tm.tile_m_small), ctypes.c_int(tm.small_max_rows), ctypes.c_int(tm.tile_m_slack),
                             ctypes.c_int(B), _p(row))
        out[B] = row
    return out


def full_table(counts, tile_m: int, tile_n: int, N: int, sigma=None, tile_m_small: int = 0,
               small_max_rows: int = 0, tile_m_slack: int = 0) -> np.ndarray:
    """Prior-art full per-block table by nested loops -> [total, 4].  `sigma` (non-empty experts in
    visiting order) defaults to ascending expert index."""
    counts = _i32(counts)
    order = None
    if sigma is not None:
        sig = [int(e) for e in sigma]
        order = _i32(sig + [e for e in range(len(counts)) if e not in set(sig)])
    nt = -(-N // tile_n)
    def _tm(c):
        return tile_m_small if (small_max_rows > 0 and c <= small_max_rows) else tile_m
    cap = int(sum(-(-int(c) // _tm(int(c))) for c in counts) * nt)   # room for the no-slack tiling, the largest
    table = np.zeros((max(cap, 1), 4), dtype=np.int32)
    n = _load().orc_full_table(_p(counts), ctypes.c_int(len(counts)), _p(order), ctypes.c_int(tile_m),
                               ctypes.c_int(tile_m_small), ctypes.c_int(small_max_rows), ctypes.c_int(tile_m_slack),
                               ctypes.c_int(tile_n), ctypes.c_int(N), _p(table), ctypes.c_int(cap))
    assert 0 <= n <= cap and (tile_m_slack > 0 or n == cap)
    return table[:n]


def heterogeneous_batch_table(tm: TaskMap, reduce_tiles: int) -> np.ndarray:
    """A batch of two task types in one launch (Sec. 3.2, Alg. 3): the GEMM tasks of `tm` followed by ONE reduction
    task of `reduce_tiles` tiles.  The batch's TilePrefix (Alg. 1) runs over nu = [tiles of every non-empty expert in
    sigma order ..., reduce_tiles]; every block is mapped with Alg. 2.  Returns [total + reduce_tiles, 3] rows
    (type, task, l): type 0 = GEMM tile l of expert `task`, type 1 = tile l of the reduction task (task = -1)."""
    nu = [int(tm.tile_prefix[i] - (tm.tile_prefix[i - 1] if i else 0)) for i in range(tm.M)] + [int(reduce_tiles)]
    prefix = tile_prefix(nu)
    out = np.zeros((int(prefix[-1]) if len(prefix) else 0, 3), dtype=np.int32)
    for B in range(len(out)):
        h, l = mapping(prefix, B)
        out[B] = (0, int(tm.sigma[h]), l) if h < tm.M else (1, -1, l)
    return out


def reduce_task_tiles(T: int, N: int, chunks_per_tile: int = 4096) -> int:
    """nu of the reduction task: its output [T, N] in chunks of 8 columns, chunks_per_tile chunks per tile."""
    return -(-(T * (N // 8)) // chunks_per_tile)


# ------------------------------------------------------------------ result
@dataclass
class GemmResult:
    rows: np.ndarray   # flat row ids the outputs are for
    Y32: np.ndarray    # [nrows, N] fp32 sequential accumulation
    Y64: np.ndarray    # [nrows, N] fp64 accumulation
    Ybf: np.ndarray    # [nrows, N] uint16 bf16 bits = rne(Y64)


def _as_u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.int16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _as_u8(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.int8:
        a = a.view(np.uint8)
    assert a.dtype == np.uint8, a.dtype
    return a


def grouped_gemm_bf16(X_bits, W_bits, topk_ids, rows=None) -> GemmResult:
    """X_bits [T,K] uint16 (bf16 bits), W_bits [E,K,N] uint16, topk_ids [T,k]."""
    X = _as_u16(X_bits)
    W = _as_u16(W_bits)
    ids = _i32(topk_ids)
    T, K = X.shape
    E, K2, N = W.shape
    assert K2 == K
    k = ids.shape[1] if ids.ndim == 2 else ids.size // max(T, 1)
    ids = ids.reshape(-1)
    rows_a = np.arange(T * k, dtype=np.int32) if rows is None else _i32(rows)
    n = len(rows_a)
    Y32 = np.zeros((n, N), dtype=np.float32)
    Y64 = np.zeros((n, N), dtype=np.float64)
    Ybf = np.zeros((n, N), dtype=np.uint16)
    _load().orc_grouped_gemm_bf16(_p(X), _p(W), _p(ids), ctypes.c_int(T), ctypes.c_int(k), ctypes.c_int(E),
                                  ctypes.c_int(K), ctypes.c_int(N), _p(rows_a), ctypes.c_int(n),
                                  _p(Y32), _p(Y64), _p(Ybf))
    return GemmResult(rows_a, Y32, Y64, Ybf)


def grouped_gemm_fp8(X_bytes, W_bytes, x_scale, w_scale, topk_ids, rows=None) -> GemmResult:
    """X_bytes [T,K] uint8 (e4m3), W_bytes [E,K,N] uint8, x_scale [T], w_scale [E] fp32."""
    X = _as_u8(X_bytes)
    W = _as_u8(W_bytes)
    xs = np.ascontiguousarray(np.asarray(x_scale, dtype=np.float32))
    ws = np.ascontiguousarray(np.asarray(w_scale, dtype=np.float32))
    ids = _i32(topk_ids)
    T, K = X.shape
    E, K2, N = W.shape
    assert K2 == K and xs.shape == (T,) and ws.shape == (E,)
    k = ids.shape[1] if ids.ndim == 2 else ids.size // max(T, 1)
    ids = ids.reshape(-1)
    rows_a = np.arange(T * k, dtype=np.int32) if rows is None else _i32(rows)
    n = len(rows_a)
    Y32 = np.zeros((n, N), dtype=np.float32)
    Y64 = np.zeros((n, N), dtype=np.float64)
    Ybf = np.zeros((n, N), dtype=np.uint16)
    _load().orc_grouped_gemm_fp8(_p(X), _p(W), _p(xs), _p(ws), _p(ids), ctypes.c_int(T), ctypes.c_int(k),
                                 ctypes.c_int(E), ctypes.c_int(K), ctypes.c_int(N), _p(rows_a),
                                 ctypes.c_int(n), _p(Y32), _p(Y64), _p(Ybf))
    return GemmResult(rows_a, Y32, Y64, Ybf)


def gemm_elements(X, W, topk_ids, k: int, rr, nn, x_scale=None, w_scale=None) -> np.ndarray:
    """fp64 value of single outputs Y[rr[i], nn[i]]; dtype uint16 -> bf16, uint8 -> e4m3."""
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    is_fp8 = X.dtype in (np.uint8, np.int8)
    ids = _i32(topk_ids).reshape(-1)
    rr = _i32(rr)
    nn = _i32(nn)
    K = X.shape[1]
    N = W.shape[2]
    xs = None if x_scale is None else np.ascontiguousarray(np.asarray(x_scale, dtype=np.float32))
    ws = None if w_scale is None else np.ascontiguousarray(np.asarray(w_scale, dtype=np.float32))
    out = np.zeros(len(rr), dtype=np.float64)
    _load().orc_gemm_elements(_p(X), _p(W), _p(xs), _p(ws), _p(ids), ctypes.c_int(k), ctypes.c_int(K),
                              ctypes.c_int(N), ctypes.c_int(int(is_fp8)), _p(rr), _p(nn),
                              ctypes.c_int(len(rr)), _p(out))
    return out


def norm_scale_elements(X, W, topk_ids, k: int, rr, nn, x_scale=None, w_scale=None) -> np.ndarray:
    """||X[t]|| * ||W[e,:,n]|| (scales folded in) for single outputs: the tolerance scale."""
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    is_fp8 = X.dtype in (np.uint8, np.int8)
    ids = _i32(topk_ids).reshape(-1)
    rr = _i32(rr)
    nn = _i32(nn)
    K = X.shape[1]
    N = W.shape[2]
    xs = None if x_scale is None else np.ascontiguousarray(np.asarray(x_scale, dtype=np.float32))
    ws = None if w_scale is None else np.ascontiguousarray(np.asarray(w_scale, dtype=np.float32))
    out = np.zeros(len(rr), dtype=np.float64)
    _load().orc_norm_scale_elements(_p(X), _p(W), _p(xs), _p(ws), _p(ids), ctypes.c_int(k), ctypes.c_int(K),
                                    ctypes.c_int(N), ctypes.c_int(int(is_fp8)), _p(rr), _p(nn),
                                    ctypes.c_int(len(rr)), _p(out))
    return out


def swiglu(Y64):
    """Gated activation of the fp64 sums Y64 [rows, N] (gate columns [0, N/2), up columns [N/2, N)):
    returns (H64 [rows, N/2], Hbf uint16 bf16 bits)."""
    Y64 = np.ascontiguousarray(np.asarray(Y64, dtype=np.float64))
    n, N = Y64.shape
    assert N % 2 == 0
    H64 = np.zeros((n, N // 2), dtype=np.float64)
    Hbf = np.zeros((n, N // 2), dtype=np.uint16)
    _load().orc_swiglu(_p(Y64), ctypes.c_int(n), ctypes.c_int(N), _p(H64), _p(Hbf))
    return H64, Hbf


def combine(Y_bits, weights, T: int, k: int):
    """Sum over a token's k experts of Y_bits [T*k, N] (bf16 bits), weighted by weights [T, k] fp32 or None:
    returns (out64 [T, N], outbf uint16)."""
    Y = _as_u16(Y_bits).reshape(T * k, -1)
    N = Y.shape[1]
    w = None if weights is None else np.ascontiguousarray(np.asarray(weights, dtype=np.float32).reshape(T, k))
    out64 = np.zeros((T, N), dtype=np.float64)
    outbf = np.zeros((T, N), dtype=np.uint16)
    _load().orc_combine(_p(Y), _p(w) if w is not None else None, ctypes.c_int(T), ctypes.c_int(k), ctypes.c_int(N),
                        _p(out64), _p(outbf))
    return out64, outbf
