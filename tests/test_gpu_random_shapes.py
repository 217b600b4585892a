"""Seeded random sweep over valid shapes, tilings and options: every case is compared with the oracle.

The hand-picked parity cases fix one thing at a time; this sweep mixes them (tile shape x expert count x ragged
row counts x K and N multiples x sigma order x slack rows x fused activation x weight layout x streaming mode).
"""
import numpy as np
import pytest
import torch

from paper_2501_16103_amd import binding as mb
from paper_2501_16103_amd import workloads as wk
from tests import helpers as H
from tests.test_gpu_neighbours import _check_swiglu
from tests.test_gpu_parity import _check_y

pytestmark = pytest.mark.gpu

POISON = 0x7FC1
BF16_TILES = [(256, 256), (128, 256), (128, 128), (64, 256), (64, 128), (32, 256), (32, 128), (16, 256), (16, 128)]
FP8_TILES = [(16, 256), (16, 128), (16, 64), (32, 128), (64, 256), (256, 256)]


def _case(seed):
    rng = np.random.default_rng(9000 + seed)
    fp8 = bool(rng.random() < 0.3)
    tile_m, tile_n = (FP8_TILES if fp8 else BF16_TILES)[int(rng.integers(0, len(FP8_TILES if fp8 else BF16_TILES)))]
    E = int(rng.choice([1, 2, 3, 8, 17, 64, 70, 256]))
    k = int(rng.integers(1, min(E, 8) + 1))
    # enough rows for a few m-tiles of the busiest expert, few enough for the oracle to finish in a second
    T = int(rng.integers(1, max(2, min(900, (3 * tile_m * E) // k + 2))))
    T = min(T, 1200 // k + 1)
    bk = 128 if fp8 else 64
    K = bk * int(rng.integers(1, 5))
    N = tile_n * int(rng.integers(1, 4))
    routing = str(rng.choice(["gauss_topk", "zipf", "uniform_topk"]))
    opt = dict(order=int(rng.integers(0, 3)), slack=0, swiglu=bool(rng.random() < 0.4), nk=False, stream=0)
    if (tile_m, tile_n) == (256, 256) and not fp8 and rng.random() < 0.5:
        opt["slack"] = 64 if T % 2 == 0 else 32
    if tile_m == 16:
        opt["stream"] = int(rng.choice([0, 1, 8, 16]))
    return fp8, tile_m, tile_n, E, k, T, K, N, routing, opt, rng


@pytest.mark.parametrize("seed", range(48))
def test_random_case(oracle_mod, seed):
    dev = torch.device("cuda:0")
    fp8, tile_m, tile_n, E, k, T, K, N, routing, opt, rng = _case(seed)
    dt = mb.MOE_DTYPE_FP8_E4M3 if fp8 else mb.MOE_DTYPE_BF16
    tiling = mb.Tiling(tile_m, tile_n, opt["order"], 0, 0, opt["slack"])
    if mb.moe_w_layout_supported(dt, tiling, mb.MOE_W_LAYOUT_NK) and rng.random() < 0.5:
        opt["nk"] = True
    print(f"case: fp8={fp8} tile={tile_m}x{tile_n} E={E} k={k} T={T} K={K} N={N} {routing} {opt}", flush=True)
    wl = wk.Workload("random_case", T, E, k, K, N, "fp8" if fp8 else "bf16", routing, tile_m, tile_n)
    ids = wk.make_routing(wl)
    xs = ws = None
    if fp8:
        X, xs = wk.make_x(wl)
        W, ws = wk.make_w(wl)
        if opt["swiglu"]:
            ws = ws * 4.0
    else:
        X, W = wk.make_x(wl), wk.make_w(wl) * (4.0 if opt["swiglu"] else 1.0)
    Wd = (W.transpose(1, 2).contiguous() if opt["nk"] else W).to(dev)
    R, NO = wl.R, (N // 2 if opt["swiglu"] else N)
    pad = 3
    buf = torch.empty((R + 2 * pad, NO), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + R]
    tmap = mb.alloc_task_map(T, k, E, tile_m, tile_n, N)
    mb.moe_build_task_map_ex(ids.to(dev), T, k, E, N, tiling, tmap)
    tm = oracle_mod.build_task_map(ids.numpy(), T, k, E, tile_m, tile_n, N, order=opt["order"], tile_m_slack=opt["slack"])
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    desc = mb.GemmDesc(dt, T, k, E, K, N, tile_m, tile_n, None if xs is None else xs.to(dev), None if ws is None else ws.to(dev),
                       tile_m_slack=opt["slack"], epilogue=mb.MOE_EPILOGUE_SWIGLU if opt["swiglu"] else mb.MOE_EPILOGUE_NONE,
                       w_layout=mb.MOE_W_LAYOUT_NK if opt["nk"] else mb.MOE_W_LAYOUT_KN, launch_mode=opt["stream"])
    mb.moe_grouped_gemm(X.to(dev), Wd, ids.to(dev), tmap, Y, desc)
    torch.cuda.synchronize()
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + R:] == POISON), "wrote outside Y"
    got = allbits[pad: pad + R]
    if fp8:
        res = oracle_mod.grouped_gemm_fp8(wk.bits(X), wk.bits(W), xs.numpy(), ws.numpy(), ids.numpy())
        Xf = X.view(torch.float8_e4m3fn).double().numpy()
        Wf = W.view(torch.float8_e4m3fn).double().numpy()
        sx, sw = xs.double().numpy(), ws.double().numpy()
    else:
        res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
        Xf, Wf, sx, sw = X.double().numpy(), W.double().numpy(), None, None
    if opt["swiglu"]:
        _check_swiglu(oracle_mod, got, res, Xf, Wf, ids.numpy(), k, K, sx, sw)
    else:
        _check_y(got, res, Xf, Wf, ids.numpy(), k, K, H.tol_fp8(K) if fp8 else H.tol_bf16(K), sx, sw)


@pytest.mark.parametrize("seed", range(10))
def test_random_split_k_case(oracle_mod, seed):
    """Seeded random shapes for the split-k launch: expert counts from empty to several tiles, 2 or 4 parts."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(7700 + seed)
    parts = int(rng.choice([2, 4]))
    E = int(rng.choice([1, 2, 3, 8, 17]))
    counts = [int(rng.choice([0, 1, 17, 64, 65, 128, 200, 256, 257, 300, 520])) for _ in range(E)]
    if sum(counts) == 0:
        counts[0] = 33
    while sum(counts) > 1400:
        counts[int(np.argmax(counts))] //= 2
    T = sum(counts)
    K = 64 * parts * int(rng.integers(8, 12))
    N = 256 * int(rng.integers(1, 3))
    order = int(rng.integers(0, 3))
    print(f"case: parts={parts} counts={counts} K={K} N={N} order={order}", flush=True)
    wl = wk.Workload("random_split_k", T, E, 1, K, N, "bf16", "gauss_topk", 256, 256)
    g = torch.Generator().manual_seed(7700 + seed)
    ids = torch.repeat_interleave(torch.arange(E, dtype=torch.int32), torch.tensor(counts))[torch.randperm(T, generator=g)].reshape(T, 1).contiguous()
    X, W = wk.make_x(wl), wk.make_w(wl)
    pad = 3
    buf = torch.empty((T + 2 * pad, N), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + T]
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map_ex(ids.to(dev), T, 1, E, N, mb.Tiling(256, 256, order, 0, 0, 0), tmap)
    work = torch.empty(mb.moe_splitk_workspace_bytes(T, 1, N, parts) // 4, dtype=torch.float32, device=dev)
    mb.moe_grouped_gemm_splitk(X.to(dev), W.to(dev), tmap, Y, mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256), parts, work)
    torch.cuda.synchronize()
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + T:] == POISON), "wrote outside Y"
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_y(allbits[pad: pad + T], res, X.double().numpy(), W.double().numpy(), ids.numpy(), 1, K, H.tol_bf16(K))
