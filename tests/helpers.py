"""Shared test helpers: expected task-map blob from the oracle, error metrics."""
from __future__ import annotations

import math

import numpy as np
import torch

INT32_MAX = 0x7FFFFFFF
HDR_WORDS = 32
MAGIC = 0x3142534D


def blob_offsets(E: int) -> dict:
    """Word offsets of the blob's fields as documented in include/moe_sb.h."""
    E64 = (E + 63) // 64 * 64
    counts = HDR_WORDS
    offsets = counts + E64
    sigma = offsets + E64 + 64
    prefix = sigma + E64
    records = prefix + E64
    rows = records + 4 * E64
    return dict(E64=E64, counts=counts, offsets=offsets, sigma=sigma, tile_prefix=prefix, task_records=records, sorted_rows=rows)


def expected_blob(tm) -> np.ndarray:
    """The compared part of the blob (header .. sorted_rows[R]) from an oracle TaskMap."""
    o = blob_offsets(tm.E)
    R = tm.T * tm.k
    b = np.zeros(o["sorted_rows"] + R, dtype=np.int32)
    hdr = [MAGIC, tm.T, tm.k, tm.E, tm.N, tm.tile_m, tm.tile_n, tm.nt, tm.M, tm.total_tiles, 0, 0, R, o["E64"],
           getattr(tm, "order", 0), getattr(tm, "tile_m_small", 0), getattr(tm, "small_max_rows", 0),
           getattr(tm, "tile_m_slack", 0), getattr(tm, "heavy_tiles", 0)]
    b[: len(hdr)] = hdr
    b[o["counts"]: o["counts"] + tm.E] = tm.counts
    b[o["offsets"]: o["offsets"] + o["E64"] + 64] = R
    b[o["offsets"]: o["offsets"] + tm.E + 1] = tm.offsets
    b[o["sigma"]: o["sigma"] + o["E64"]] = -1
    b[o["sigma"]: o["sigma"] + tm.M] = tm.sigma
    b[o["tile_prefix"]: o["tile_prefix"] + o["E64"]] = INT32_MAX
    b[o["tile_prefix"]: o["tile_prefix"] + tm.M] = tm.tile_prefix
    rec = np.zeros((o["E64"], 4), dtype=np.int32)
    rec[:, 0], rec[:, 1] = INT32_MAX, -1
    for i in range(tm.M):
        e = int(tm.sigma[i])
        rec[i] = (tm.tile_prefix[i], e, tm.counts[e], tm.offsets[e])
    b[o["task_records"]: o["task_records"] + 4 * o["E64"]] = rec.reshape(-1)
    b[o["sorted_rows"]: o["sorted_rows"] + R] = tm.sorted_rows
    return b


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def tol_bf16(K: int) -> float:
    return 2e-2 * math.sqrt(K / 256.0)


def tol_fp8(K: int) -> float:
    return 6e-2 * math.sqrt(K / 256.0)


def sum_err_coeff(K: int, fp8: bool) -> float:
    """Bound on |fp32 sum - exact sum| / sum|x_k w_k| for K exact products (bf16 x bf16 and e4m3 x e4m3 products are
    exact in fp32).

    bf16: additions in any order, each rounded to nearest: (K - 1) roundings of at most 2^-24 of a partial sum that
    never exceeds sum|x w|: K * 2^-24 (a hair above for the second-order terms).

    fp8: the ISA does not say how the 16x16x32 fp8 MFMA adds its 32 products and the addend.  The model assumed
    here is the usual wide adder: the 33 terms are aligned to the largest exponent among them, each keeps 24
    significant bits counted from that exponent and the rest is CUT OFF (not rounded), the aligned terms are
    added exactly and the result is rounded once to fp32.  With S = |addend| + sum of the 32 |products| <= A
    (A = sum over all K of |x w|): each term loses less than 2^-23 * max term <= 2^-23 * S, 33 terms per
    instruction, plus 2^-24 * S for the final rounding; K / 32 instructions per output:
        (K / 32) * (33 * 2^-23 + 2^-24) * A  =  (2 * 33 / 32 + 1 / 32) * K * 2^-24 * A  =  2.09375 * K * 2^-24 * A.
    Because the lost bits are cut off, the errors are biased instead of averaging out, which is why measured errors
    come close to a worst-case bound at all: up to 1.11 * K * 2^-24 * A over a few hundred seeded random problems
    (a round-to-nearest-per-addition model would allow 1.0 and is violated)."""
    return (2.0 * 33.0 / 32.0 + 1.0 / 32.0 if fp8 else 1.01) * K * 2.0 ** -24


def ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in bf16 units in the last place between two bf16 bit arrays (sign-magnitude aware)."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def y_bits(Y: torch.Tensor) -> np.ndarray:
    return Y.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
