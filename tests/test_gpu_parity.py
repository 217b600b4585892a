"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Task map, counts, offsets and the expanded table must be bit-exact.  Y must agree within
max|err| <= 2e-2*sqrt(K/256)*||x||*||w|| (bf16) or 6e-2*(that scale) (fp8); in addition a much
tighter statistic is asserted (distance to the oracle's bf16 in units in the last place), because
the stated bound alone is loose enough to pass a wrongly routed row at large K.
"""
import numpy as np
import pytest
import torch

from paper_2501_16103_amd import binding as mb
from paper_2501_16103_amd import workloads as wk
from tests import helpers as H

pytestmark = pytest.mark.gpu

POISON = 0x7FC1  # a bf16 NaN with a recognisable payload


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    mb.lib()  # fails loudly when libmoe_sb.so is not built
    return torch.device("cuda:0")


def _build_map(ids_dev, T, k, E, tile_m, tile_n, N, order=0, small=0, thr=0, slack=0):
    tmap = mb.alloc_task_map(max(T, 1), k, E, tile_m, tile_n, N)
    tmap.fill_(0x5A5A5A5A)
    if slack:
        mb.moe_build_task_map_ex(ids_dev, T, k, E, N, mb.Tiling(tile_m, tile_n, order, small, thr, slack), tmap)
    elif small:
        mb.moe_build_task_map_tiled(ids_dev, T, k, E, tile_m, tile_n, N, order, small, thr, tmap)
    elif order == 0:
        mb.moe_build_task_map(ids_dev, T, k, E, tile_m, tile_n, N, tmap)
    else:
        mb.moe_build_task_map_ordered(ids_dev, T, k, E, tile_m, tile_n, N, order, tmap)
    return tmap


MAP_CASES = [
    # T, k, E, tile_m, tile_n, N, routing
    (0, 2, 8, 16, 128, 512, "gauss_topk"),
    (1, 6, 64, 16, 64, 2816, "uniform_topk"),
    (64, 2, 8, 32, 128, 512, "gauss_topk"),
    (512, 2, 8, 64, 128, 4096, "zipf"),            # exactly one chunk of 1024 rows
    (513, 2, 8, 64, 128, 4096, "zipf"),            # one row into the second chunk
    (128, 8, 256, 16, 128, 4096, "gauss_topk"),    # E > 64: several voting rounds, empty experts
    (33, 3, 70, 16, 64, 192, "zipf"),              # E not a multiple of 64
    (4096, 2, 8, 256, 256, 28672, "gauss_topk"),
    (4096, 2, 8, 256, 256, 4096, "zipf"),
    (2048, 8, 256, 64, 128, 4096, "gauss_topk"),
    (8192, 8, 256, 256, 256, 4096, "gauss_topk"),  # 64 chunks
    (4096, 8, 64, 256, 256, 2560, "worst"),
    (4096, 8, 64, 256, 256, 2560, "best"),
    (1000, 1, 1, 128, 128, 128, "best"),
    (3000, 4, 1000, 16, 64, 128, "gauss_topk"),    # 16 groups of 64 tasks: two-level decode
    (700, 2, 640, 16, 64, 128, "zipf"),            # E64 = 640, most experts empty
]


@pytest.mark.parametrize("order", [0, 1, 2], ids=["ascending", "spread", "interleave"])
@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,routing", MAP_CASES)
def test_task_map_bit_exact(dev, oracle_mod, T, k, E, tile_m, tile_n, N, routing, order):
    wl = wk.Workload("mapcase", T, E, k, 64, N, "bf16", routing)
    ids = wk.make_routing(wl)
    tm = oracle_mod.build_task_map(ids.numpy(), T, k, E, tile_m, tile_n, N, order=order)
    want = H.expected_blob(tm)
    ids_dev = ids.to(dev)
    got1 = _build_map(ids_dev, T, k, E, tile_m, tile_n, N, order)
    assert mb.moe_task_map_status(got1) == mb.MOE_OK
    g1 = got1.cpu().numpy()
    np.testing.assert_array_equal(g1[: len(want)], want)
    # determinism: a second build gives the same bytes, scratch included
    got2 = _build_map(ids_dev, T, k, E, tile_m, tile_n, N, order)
    torch.cuda.synchronize()
    assert torch.equal(got1, got2)
    # documented offsets are the library's offsets
    lo = mb.moe_map_offsets(E)
    o = H.blob_offsets(E)
    assert all(lo[f] == o[f] for f in lo)
    # expanded full table == oracle's Alg. 4 decode of every block == brute-force table
    grid = mb.moe_grid_upper_bound(T, k, E, tile_m, tile_n, N)
    assert grid >= tm.total_tiles
    table = torch.full((max(grid, 1), 4), 7, dtype=torch.int32, device=dev)
    mb.moe_task_map_expand(got1, E, table, grid)
    tab = table.cpu().numpy()[:grid]
    np.testing.assert_array_equal(tab[: tm.total_tiles], oracle_mod.full_table(tm.counts, tile_m, tile_n, N, sigma=tm.sigma))
    assert np.all(tab[tm.total_tiles:] == -1)
    if tm.total_tiles <= 6000:
        np.testing.assert_array_equal(tab[: tm.total_tiles], oracle_mod.decode_all(tm))


def test_bad_routing_id_reported_and_gemm_noop(dev):
    T, k, E, K, N = 40, 2, 8, 256, 256
    ids = torch.randint(0, E, (T, k), dtype=torch.int32)
    ids[7, 1] = E
    ids[20, 0] = -3
    tmap = _build_map(ids.to(dev), T, k, E, 16, 128, N)
    assert mb.moe_task_map_status(tmap) == mb.MOE_ERR_ROUTING
    hdr = tmap[:32].cpu().numpy()
    assert hdr[mb.HDR["STATUS"]] == 2 and hdr[mb.HDR["TOTAL_TILES"]] == 0
    X = torch.randn(T, K, device=dev).to(torch.bfloat16)
    W = torch.randn(E, K, N, device=dev).to(torch.bfloat16)
    Y = torch.full((T * k, N), float("nan"), device=dev, dtype=torch.bfloat16)
    mb.moe_grouped_gemm(X, W, None, tmap, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, k, E, K, N, 16, 128))
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y).all())  # nothing gathered, nothing written


def test_argument_errors(dev):
    ids = torch.zeros((4, 2), dtype=torch.int32, device=dev)
    tmap = mb.alloc_task_map(4, 2, 8, 16, 128, 256)
    assert mb.moe_build_task_map(ids, -1, 2, 8, 16, 128, 256, tmap, check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_build_task_map(ids, 4, 9, 8, 16, 128, 256, tmap, check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_build_task_map(ids, 4, 2, 8, 17, 128, 256, tmap, check=False) == mb.MOE_ERR_UNSUPPORTED
    assert mb.moe_build_task_map(None, 4, 2, 8, 16, 128, 256, tmap, check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_build_task_map_ordered(ids, 4, 2, 8, 16, 128, 256, 7, tmap, check=False) == mb.MOE_ERR_INVALID_ARG
    mb.moe_build_task_map(ids, 4, 2, 8, 16, 128, 256, tmap)
    X = torch.zeros(4, 256, device=dev, dtype=torch.bfloat16)
    W = torch.zeros(8, 256, 256, device=dev, dtype=torch.bfloat16)
    Y = torch.zeros(8, 256, device=dev, dtype=torch.bfloat16)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, 4, 2, 8, 256, 256, 16, 128)
    assert mb.moe_grouped_gemm(None, W, None, tmap, Y, d, check=False) == mb.MOE_ERR_INVALID_ARG
    d_bad_k = mb.GemmDesc(mb.MOE_DTYPE_BF16, 4, 2, 8, 200, 256, 16, 128)
    assert mb.moe_grouped_gemm(X, W, None, tmap, Y, d_bad_k, check=False) == mb.MOE_ERR_UNSUPPORTED
    d_fp8 = mb.GemmDesc(mb.MOE_DTYPE_FP8_E4M3, 4, 2, 8, 256, 256, 16, 128)
    assert mb.moe_grouped_gemm(X, W, None, tmap, Y, d_fp8, check=False) == mb.MOE_ERR_INVALID_ARG  # no scales
    # a map built for other tiles makes the kernel a no-op instead of a wild gather
    Y.fill_(float("nan"))
    d_other = mb.GemmDesc(mb.MOE_DTYPE_BF16, 4, 2, 8, 256, 256, 32, 128)
    assert mb.moe_grouped_gemm(X, W, None, tmap, Y, d_other, check=False) == mb.MOE_OK
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y).all())


def _run_gemm(dev, wl, ids, X, W, xs=None, ws=None, order=0, small=0, thr=0, slack=0, launch_mode=0):
    """Run map build + GEMM with Y embedded between poisoned canary rows; returns Y bits [R,N]."""
    R, N = wl.R, wl.N
    pad = 4
    buf = torch.empty((R + 2 * pad, N), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + R]
    tmap = _build_map(ids.to(dev), wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, N, order, small, thr, slack)
    dt = mb.MOE_DTYPE_FP8_E4M3 if wl.dtype == "fp8" else mb.MOE_DTYPE_BF16
    desc = mb.GemmDesc(dt, wl.T, wl.k, wl.E, wl.K, N, wl.tile_m, wl.tile_n,
                       None if xs is None else xs.to(dev), None if ws is None else ws.to(dev), small, thr, slack,
                       launch_mode=launch_mode)
    mb.moe_grouped_gemm(X.to(dev), W.to(dev), ids.to(dev), tmap, Y, desc)
    torch.cuda.synchronize()
    assert mb.moe_task_map_status(tmap) == mb.MOE_OK
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + R:] == POISON), "wrote outside Y"
    return allbits[pad: pad + R]


def _check_y(got_bits, res, Xf, Wf, ids, k, K, tol, xs=None, ws=None):
    """got_bits [R,N] uint16 vs oracle GemmResult; Xf [T,K], Wf [E,K,N] float64 element values."""
    assert not np.any(got_bits == POISON), "a (token, slot) row or column range was never written"
    got = H.bf16_bits_to_f64(got_bits)
    flat = ids.reshape(-1)
    xn = np.sqrt((Xf ** 2).sum(axis=1))              # [T]
    wn = np.sqrt((Wf ** 2).sum(axis=1))              # [E,N]
    scale = xn[np.arange(len(flat)) // k][:, None] * wn[flat]
    if xs is not None:
        scale = scale * (xs[np.arange(len(flat)) // k][:, None] * ws[flat][:, None])
    err = np.abs(got - res.Y64)
    assert np.all(err <= tol * scale), f"max err/scale = {(err / scale).max():.3e} > {tol:.3e}"
    # tight, derived bound: any fp32 summation order errs by at most K*2^-24*sum|x_k w_k|, and the
    # final round-to-nearest bf16 adds at most 2^-8 of the value
    xi = np.arange(len(flat)) // k
    A = np.stack([np.abs(Xf[xi[r]]) @ np.abs(Wf[flat[r]]) for r in range(len(flat))])
    if xs is not None:
        A = A * (xs[xi][:, None] * ws[flat][:, None])
    tight = 2.0 ** -8 * np.abs(res.Y64) * 1.001 + H.sum_err_coeff(K, xs is not None) * A + 1e-30
    assert np.all(err <= tight), f"max err/tight = {(err / tight).max():.3f}"
    # and nearly every stored value is bit-identical to the oracle's single-rounded bf16
    ulp = H.ulp_distance(got_bits, res.Ybf)
    assert (ulp == 0).mean() > 0.97


BF16_CASES = [
    # tile_m, tile_n, T, E, k, K, N, routing
    (16, 128, 64, 8, 2, 256, 512, "gauss_topk"),
    (16, 256, 100, 8, 2, 256, 512, "zipf"),
    (32, 128, 64, 8, 2, 256, 512, "gauss_topk"),      # the tiny benchmark config
    (32, 256, 150, 8, 2, 192, 512, "zipf"),
    (64, 128, 300, 8, 2, 256, 256, "gauss_topk"),
    (64, 256, 300, 8, 2, 128, 512, "zipf"),
    (128, 128, 600, 8, 2, 256, 256, "gauss_topk"),
    (128, 256, 600, 8, 2, 128, 512, "zipf"),
    (256, 256, 1200, 8, 2, 256, 512, "gauss_topk"),
    (256, 256, 700, 16, 2, 128, 256, "zipf"),         # empty experts, one > 2 tiles, ragged tails
    (256, 256, 900, 8, 2, 64, 256, "gauss_topk"),     # one k-tile: prologue and the loop's last iteration only
    (256, 256, 520, 4, 2, 320, 256, "zipf"),          # five k-tiles: three steady iterations and two that fetch nothing
    (16, 128, 40, 256, 8, 128, 256, "gauss_topk"),    # E = 256: four voting rounds
    (64, 128, 257, 3, 1, 64, 128, "worst"),
    (16, 128, 50, 300, 4, 128, 256, "gauss_topk"),    # E = 300: five groups of task records, no streaming launch
    (64, 128, 200, 1000, 2, 64, 128, "zipf"),         # E = 1000: sixteen groups
]


@pytest.mark.parametrize("order", [0, 1, 2], ids=["ascending", "spread", "interleave"])
@pytest.mark.parametrize("tile_m,tile_n,T,E,k,K,N,routing", BF16_CASES)
def test_gemm_bf16_parity(dev, oracle_mod, tile_m, tile_n, T, E, k, K, N, routing, order):
    wl = wk.Workload("parity_bf16", T, E, k, K, N, "bf16", routing, tile_m, tile_n)
    ids, X, W = wk.make_routing(wl), wk.make_x(wl), wk.make_w(wl)
    got = _run_gemm(dev, wl, ids, X, W, order=order)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_y(got, res, X.double().numpy(), W.double().numpy(), ids.numpy(), k, K, H.tol_bf16(K))


TILED_CASES = [
    # T, E, k, K, N, routing, tile_m_small, small_max_rows   (large strategy: 256 x 256)
    (1200, 16, 2, 256, 512, "zipf", 64, 64),
    (700, 16, 2, 128, 256, "zipf", 128, 128),
    (600, 64, 8, 128, 256, "worst", 64, 64),          # 56 one-row experts next to 8 busy ones
    (1200, 8, 2, 256, 512, "gauss_topk", 64, 64),     # nobody is small
    (300, 16, 2, 128, 256, "gauss_topk", 64, 200),    # everybody is small, several small tiles each
]


@pytest.mark.parametrize("order", [0, 1, 2], ids=["ascending", "spread", "interleave"])
@pytest.mark.parametrize("T,E,k,K,N,routing,small,thr", TILED_CASES)
def test_two_tiling_strategies_parity(dev, oracle_mod, T, E, k, K, N, routing, small, thr, order):
    """Alg. 3 with two task types in one launch: map bit-exact, expanded table == nested-loop table, Y == oracle."""
    wl = wk.Workload("parity_tiled", T, E, k, K, N, "bf16", routing, 256, 256)
    assert mb.moe_tile_pair_supported(mb.MOE_DTYPE_BF16, 256, 256, small)
    ids, X, W = wk.make_routing(wl), wk.make_x(wl), wk.make_w(wl)
    tm = oracle_mod.build_task_map(ids.numpy(), T, k, E, 256, 256, N, order=order, tile_m_small=small, small_max_rows=thr)
    tmap = _build_map(ids.to(dev), T, k, E, 256, 256, N, order, small, thr)
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    grid = mb.moe_grid_upper_bound_tiled(T, k, E, 256, 256, N, small, thr)
    assert grid >= tm.total_tiles
    table = torch.full((grid, 4), 7, dtype=torch.int32, device=dev)
    mb.moe_task_map_expand(tmap, E, table, grid)
    tab = table.cpu().numpy()
    np.testing.assert_array_equal(tab[: tm.total_tiles], oracle_mod.full_table(tm.counts, 256, 256, N, sigma=tm.sigma,
                                                                                tile_m_small=small, small_max_rows=thr))
    assert np.all(tab[tm.total_tiles:] == -1)
    got = _run_gemm(dev, wl, ids, X, W, order=order, small=small, thr=thr)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_y(got, res, X.double().numpy(), W.double().numpy(), ids.numpy(), k, K, H.tol_bf16(K))


def test_tiling_pair_mismatch_is_a_noop(dev):
    """A two-strategy map run through the one-strategy kernel (or the other way round) must do nothing."""
    T, E, k, K, N = 300, 16, 2, 128, 256
    wl = wk.Workload("pair_mismatch", T, E, k, K, N, "bf16", "zipf", 256, 256)
    ids = wk.make_routing(wl).to(dev)
    X, W = wk.make_x(wl, dev), wk.make_w(wl, dev)
    Y = torch.full((T * k, N), float("nan"), device=dev, dtype=torch.bfloat16)
    tiled = _build_map(ids, T, k, E, 256, 256, N, 0, 64, 64)
    plain = _build_map(ids, T, k, E, 256, 256, N, 0)
    mb.moe_grouped_gemm(X, W, ids, tiled, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, k, E, K, N, 256, 256))
    mb.moe_grouped_gemm(X, W, ids, plain, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, k, E, K, N, 256, 256, None, None, 64, 64))
    mb.moe_grouped_gemm(X, W, ids, tiled, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, k, E, K, N, 256, 256, None, None, 64, 32))
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y).all())
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, k, E, K, N, 256, 256, None, None, 32, 32)
    assert mb.moe_grouped_gemm(X, W, ids, tiled, Y, d, check=False) == mb.MOE_ERR_UNSUPPORTED


def _ids_from_counts(counts, seed):
    """k = 1 routing with exactly these per-expert row counts, rows shuffled."""
    flat = np.concatenate([np.full(c, e, np.int32) for e, c in enumerate(counts)])
    np.random.default_rng(seed).shuffle(flat)
    return torch.from_numpy(flat.reshape(-1, 1).copy())


SLACK_CASES = [
    # per-expert row counts (k = 1), K, N    (tile 256 x 256, slack 64 and 32)
    ([257, 320, 321, 256, 1, 64, 65, 0, 576, 639, 640, 641], 128, 256),
    ([300, 0, 0, 513, 129, 255, 319], 192, 512),
    ([1025, 1040, 991, 1055], 64, 256),     # the remainders of the Mixtral benchmark point
    ([288, 289, 272, 273, 257, 130, 200, 231, 17, 544, 545], 256, 256),   # every count of live 16-row blocks
]


@pytest.mark.parametrize("slack", [64, 32])
@pytest.mark.parametrize("order", [0, 1, 2], ids=["ascending", "spread", "interleave"])
@pytest.mark.parametrize("counts,K,N", SLACK_CASES)
def test_slack_rows_parity(dev, oracle_mod, counts, K, N, order, slack):
    """Last m-tiles with up to tile_m + slack rows: map bit-exact, expanded table == nested-loop table, Y == oracle."""
    E, T = len(counts), int(sum(counts))
    tiling = mb.Tiling(256, 256, order, 0, 0, slack)
    assert mb.moe_tiling_supported(mb.MOE_DTYPE_BF16, tiling)
    wl = wk.Workload("parity_slack", T, E, 1, K, N, "bf16", "gauss_topk", 256, 256)
    ids = _ids_from_counts(counts, 5 + E + K)
    X, W = wk.make_x(wl), wk.make_w(wl)
    tm = oracle_mod.build_task_map(ids.numpy(), T, 1, E, 256, 256, N, order=order, tile_m_slack=slack)
    tmap = _build_map(ids.to(dev), T, 1, E, 256, 256, N, order, slack=slack)
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    grid = mb.moe_grid_upper_bound(T, 1, E, 256, 256, N)
    assert grid >= tm.total_tiles
    table = torch.full((grid, 4), 7, dtype=torch.int32, device=dev)
    mb.moe_task_map_expand(tmap, E, table, grid)
    tab = table.cpu().numpy()
    np.testing.assert_array_equal(tab[: tm.total_tiles], oracle_mod.full_table(tm.counts, 256, 256, N, sigma=tm.sigma, tile_m_slack=slack))
    assert np.all(tab[tm.total_tiles:] == -1)
    assert tab[: tm.total_tiles, 3].max() > 256, "the case must contain a tile that uses its slack rows"
    got = _run_gemm(dev, wl, ids, X, W, order=order, slack=slack)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_y(got, res, X.double().numpy(), W.double().numpy(), ids.numpy(), 1, K, H.tol_bf16(K))


def test_slack_mismatch_is_a_noop(dev):
    """A map built with slack rows run through the kernel without them (or the other way round) must do nothing."""
    counts, K, N = [300, 20, 600], 64, 256
    T, E = sum(counts), len(counts)
    wl = wk.Workload("slack_mismatch", T, E, 1, K, N, "bf16", "gauss_topk", 256, 256)
    ids = _ids_from_counts(counts, 3).to(dev)
    X, W = wk.make_x(wl, dev), wk.make_w(wl, dev)
    Y = torch.full((T, N), float("nan"), device=dev, dtype=torch.bfloat16)
    with_slack = _build_map(ids, T, 1, E, 256, 256, N, 0, slack=64)
    plain = _build_map(ids, T, 1, E, 256, 256, N, 0)
    mb.moe_grouped_gemm(X, W, ids, with_slack, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256))
    mb.moe_grouped_gemm(X, W, ids, plain, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256, tile_m_slack=64))
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y).all())
    mb.moe_grouped_gemm(X, W, ids, with_slack, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256, tile_m_slack=32))
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y).all())
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256, tile_m_slack=128)
    assert mb.moe_grouped_gemm(X, W, ids, with_slack, Y, d, check=False) == mb.MOE_ERR_UNSUPPORTED
    g = mb.Tiling(256, 256, 0, 0, 0, 256)
    assert mb.moe_build_task_map_ex(ids, T, 1, E, N, g, with_slack, check=False) == mb.MOE_ERR_INVALID_ARG


FP8_CASES = [
    (16, 64, 1, 64, 6, 256, 128, "uniform_topk"),
    (16, 128, 8, 64, 6, 256, 256, "uniform_topk"),
    (16, 256, 32, 64, 6, 384, 512, "uniform_topk"),
    (16, 128, 100, 8, 2, 128, 256, "zipf"),           # several m-tiles per expert
    (32, 128, 100, 8, 2, 256, 256, "zipf"),
    (64, 256, 300, 8, 2, 256, 512, "zipf"),           # fp8 at prefill sizes: 64- and 256-row tiles
    (256, 256, 700, 8, 2, 256, 512, "zipf"),
    (256, 256, 1200, 8, 2, 384, 256, "gauss_topk"),
    (256, 256, 257, 3, 1, 128, 256, "worst"),
]


@pytest.mark.parametrize("tile_m,tile_n,T,E,k,K,N,routing", FP8_CASES)
def test_gemm_fp8_parity(dev, oracle_mod, tile_m, tile_n, T, E, k, K, N, routing):
    wl = wk.Workload("parity_fp8", T, E, k, K, N, "fp8", routing, tile_m, tile_n)
    ids = wk.make_routing(wl)
    Xq, xs = wk.make_x(wl)
    Wq, ws = wk.make_w(wl)
    got = _run_gemm(dev, wl, ids, Xq, Wq, xs, ws)
    res = oracle_mod.grouped_gemm_fp8(Xq.numpy(), Wq.numpy(), xs.numpy(), ws.numpy(), ids.numpy())
    Xf = Xq.view(torch.float8_e4m3fn).double().numpy()
    Wf = Wq.view(torch.float8_e4m3fn).double().numpy()
    _check_y(got, res, Xf, Wf, ids.numpy(), k, K, H.tol_fp8(K), xs.double().numpy(), ws.double().numpy())


def test_identity_weight_returns_tokens_exactly(dev):
    """W = I: every output row is bit-for-bit the gathered token (a property, no oracle needed)."""
    T, E, k, K = 300, 8, 2, 256
    wl = wk.Workload("ident", T, E, k, K, K, "bf16", "zipf", 64, 128)
    ids, X = wk.make_routing(wl), wk.make_x(wl)
    W = torch.eye(K).to(torch.bfloat16).expand(E, K, K).contiguous()
    got = _run_gemm(dev, wl, ids, X, W)
    np.testing.assert_array_equal(got, wk.bits(X)[np.arange(T * k) // k])
