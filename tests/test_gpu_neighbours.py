"""GPU parity of the fused gated activation (epilogue of the grouped GEMM) and of the sum over a token's experts.

Every tile shape is covered, because the gate/up pairing differs between the 32-row and the 16-row MFMA blocks
and the fp8 path applies its scales before the activation.
"""
import numpy as np
import pytest
import torch

from paper_2501_16103_amd import binding as mb
from paper_2501_16103_amd import probe
from paper_2501_16103_amd import workloads as wk
from tests import helpers as H

pytestmark = pytest.mark.gpu

POISON = 0x7FC1


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    mb.lib()
    return torch.device("cuda:0")


def _run_swiglu(dev, wl, ids, X, W, xs=None, ws=None, slack=0, launch_mode=0):
    R, I = wl.R, wl.N // 2
    pad = 4
    buf = torch.empty((R + 2 * pad, I), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + R]
    tmap = mb.alloc_task_map(max(wl.T, 1), wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N)
    mb.moe_build_task_map_ex(ids.to(dev), wl.T, wl.k, wl.E, wl.N, mb.Tiling(wl.tile_m, wl.tile_n, 0, 0, 0, slack), tmap)
    dt = mb.MOE_DTYPE_FP8_E4M3 if wl.dtype == "fp8" else mb.MOE_DTYPE_BF16
    desc = mb.GemmDesc(dt, wl.T, wl.k, wl.E, wl.K, wl.N, wl.tile_m, wl.tile_n,
                       None if xs is None else xs.to(dev), None if ws is None else ws.to(dev),
                       tile_m_slack=slack, epilogue=mb.MOE_EPILOGUE_SWIGLU, launch_mode=launch_mode)
    mb.moe_grouped_gemm(X.to(dev), W.to(dev), ids.to(dev), tmap, Y, desc)
    torch.cuda.synchronize()
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + R:] == POISON), "wrote outside Y"
    return allbits[pad: pad + R]


def _check_swiglu(oracle_mod, got_bits, res, Xf, Wf, ids, k, K, xs=None, ws=None):
    """got_bits [R, N/2]; res: oracle GemmResult of the un-gated product [R, N]."""
    assert not np.any(got_bits == POISON), "an output was never written"
    N = res.Y64.shape[1]
    I = N // 2
    H64, Hbf = oracle_mod.swiglu(res.Y64)
    got = H.bf16_bits_to_f64(got_bits)
    flat = ids.reshape(-1)
    xi = np.arange(len(flat)) // k
    A = np.stack([np.abs(Xf[xi[r]]) @ np.abs(Wf[flat[r]]) for r in range(len(flat))])     # sum |x||w| per (row, n)
    if xs is not None:
        A = A * (xs[xi][:, None] * ws[flat][:, None])
    eps = H.sum_err_coeff(K, xs is not None) * A + 4 * 2.0 ** -24 * np.abs(res.Y64)     # fp32 sums in any order (+ the two scale products)
    g, u = res.Y64[:, :I], res.Y64[:, I:]
    silu = g / (1.0 + np.exp(-g))
    # |d silu / dg| <= 1.1; exp, division and the product in fp32 add a few 2^-24 relative; one bf16 rounding
    tight = 2.0 ** -8 * np.abs(H64) * 1.001 + 1.1 * eps[:, :I] * np.abs(u) + np.abs(silu) * eps[:, I:] + 4e-6 * np.abs(H64) + 1e-30
    err = np.abs(got - H64)
    assert np.all(err <= tight), f"max err/tight = {(err / tight).max():.3f}"
    assert (H.ulp_distance(got_bits, Hbf) == 0).mean() > 0.95


SWIGLU_BF16 = [
    # tile_m, tile_n, slack, T, E, k, K, N, routing
    (256, 256, 0, 700, 8, 2, 128, 512, "zipf"),        # full tiles, 128- and 64-row tail functions
    (256, 256, 64, 1100, 8, 2, 128, 256, "gauss_topk"),  # counts just above 256: slack block in use
    (256, 256, 32, 1100, 8, 2, 128, 256, "gauss_topk"),
    (128, 256, 0, 300, 8, 2, 128, 512, "zipf"),
    (128, 128, 0, 300, 8, 2, 128, 256, "gauss_topk"),
    (64, 256, 0, 150, 8, 2, 192, 512, "zipf"),
    (64, 128, 0, 150, 8, 2, 128, 256, "gauss_topk"),
    (32, 256, 0, 100, 8, 2, 128, 512, "zipf"),
    (32, 128, 0, 64, 8, 2, 256, 512, "gauss_topk"),
    (16, 256, 0, 40, 8, 2, 128, 512, "zipf"),
    (16, 128, 0, 40, 16, 2, 128, 256, "gauss_topk"),
]


@pytest.mark.parametrize("tile_m,tile_n,slack,T,E,k,K,N,routing", SWIGLU_BF16)
def test_swiglu_bf16_parity(dev, oracle_mod, tile_m, tile_n, slack, T, E, k, K, N, routing):
    wl = wk.Workload("parity_swiglu", T, E, k, K, N, "bf16", routing, tile_m, tile_n)
    ids, X = wk.make_routing(wl), wk.make_x(wl)
    W = wk.make_w(wl) * 4.0     # gates of a few units, so that the activation is exercised away from its linear part
    got = _run_swiglu(dev, wl, ids, X, W, slack=slack)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_swiglu(oracle_mod, got, res, X.double().numpy(), W.double().numpy(), ids.numpy(), k, K)


SWIGLU_FP8 = [
    (16, 64, 8, 64, 6, 256, 128, "uniform_topk"),
    (16, 128, 32, 64, 6, 256, 256, "uniform_topk"),
    (16, 256, 32, 16, 2, 384, 512, "zipf"),
    (32, 128, 100, 8, 2, 256, 256, "zipf"),
]


@pytest.mark.parametrize("tile_m,tile_n,T,E,k,K,N,routing", SWIGLU_FP8)
def test_swiglu_fp8_parity(dev, oracle_mod, tile_m, tile_n, T, E, k, K, N, routing):
    wl = wk.Workload("parity_swiglu_fp8", T, E, k, K, N, "fp8", routing, tile_m, tile_n)
    ids = wk.make_routing(wl)
    X, xs = wk.make_x(wl)
    W, ws = wk.make_w(wl)
    ws = ws * 4.0
    got = _run_swiglu(dev, wl, ids, X, W, xs, ws)
    res = oracle_mod.grouped_gemm_fp8(wk.bits(X), wk.bits(W), xs.numpy(), ws.numpy(), ids.numpy())
    Xf = X.view(torch.float8_e4m3fn).double().numpy()
    Wf = W.view(torch.float8_e4m3fn).double().numpy()
    _check_swiglu(oracle_mod, got, res, Xf, Wf, ids.numpy(), k, K, xs.double().numpy(), ws.double().numpy())


def test_swiglu_argument_errors(dev):
    wl = wk.Workload("swiglu_args", 8, 4, 2, 64, 128, "bf16", "gauss_topk", 16, 128)
    ids = wk.make_routing(wl).to(dev)
    X, W = wk.make_x(wl, dev), wk.make_w(wl, dev)
    Y = torch.empty((wl.R, wl.N // 2), dtype=torch.bfloat16, device=dev)
    tmap = mb.alloc_task_map(wl.T, wl.k, wl.E, 16, 128, wl.N)
    mb.moe_build_task_map(ids, wl.T, wl.k, wl.E, 16, 128, wl.N, tmap)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, wl.T, wl.k, wl.E, wl.K, wl.N, 16, 128, epilogue=7)
    assert mb.moe_grouped_gemm(X, W, ids, tmap, Y, d, check=False) == mb.MOE_ERR_INVALID_ARG


COMBINE_CASES = [
    # T, k, N, weighted
    (1, 6, 2816, True),
    (37, 2, 512, True),
    (300, 8, 4096, True),
    (300, 8, 4096, False),
    (4096, 2, 4096, True),
    (5, 1, 8, True),
]


@pytest.mark.parametrize("T,k,N,weighted", COMBINE_CASES)
def test_combine_parity(dev, oracle_mod, T, k, N, weighted):
    g = torch.Generator().manual_seed(1000 + T + k + N)
    Y = torch.randn((T * k, N), generator=g).to(torch.bfloat16)
    w = torch.rand((T, k), generator=g, dtype=torch.float32) if weighted else None
    pad = 2
    buf = torch.empty((T + 2 * pad, N), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    out = buf[pad: pad + T]
    mb.moe_combine(Y.to(dev), None if w is None else w.to(dev), T, k, N, out)
    torch.cuda.synchronize()
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + T:] == POISON), "wrote outside out"
    got_bits = allbits[pad: pad + T]
    bits = Y.view(torch.int16).numpy().view(np.uint16)
    out64, outbf = oracle_mod.combine(bits, None if w is None else w.numpy(), T, k)
    yabs = np.abs(Y.double().numpy()).reshape(T, k, N)
    wabs = np.ones((T, k)) if w is None else np.abs(w.double().numpy())
    A = np.einsum("tj,tjn->tn", wabs, yabs)
    tight = 2.0 ** -8 * np.abs(out64) * 1.001 + (k + 1) * 2.0 ** -24 * A + 1e-30
    err = np.abs(H.bf16_bits_to_f64(got_bits) - out64)
    assert np.all(err <= tight), f"max err/tight = {(err / tight).max():.3f}"
    assert (H.ulp_distance(got_bits, outbf) == 0).mean() > 0.97


def test_combine_argument_errors(dev):
    Y = torch.zeros((4, 8), dtype=torch.bfloat16, device=dev)
    out = torch.zeros((2, 8), dtype=torch.bfloat16, device=dev)
    assert mb.moe_combine(Y, None, 2, 2, 12, out, check=False) == mb.MOE_ERR_UNSUPPORTED
    assert mb.moe_combine(Y, None, 2, 0, 8, out, check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_combine(None, None, 2, 2, 8, out, check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_combine(None, None, 0, 2, 8, None, check=False) == mb.MOE_OK


# ------------------------------------------------------------------ pre-packed weight layout [E][N][K]
NK_CASES = [
    # dtype, tile_m, tile_n, slack, T, E, k, K, N, routing, swiglu
    ("bf16", 256, 256, 0, 700, 8, 2, 128, 512, "zipf", False),
    ("bf16", 256, 256, 64, 1100, 8, 2, 192, 256, "gauss_topk", False),
    ("bf16", 256, 256, 0, 700, 8, 2, 128, 512, "zipf", True),
    ("bf16", 128, 256, 0, 300, 8, 2, 128, 512, "zipf", False),
    ("bf16", 16, 256, 0, 40, 8, 2, 128, 512, "zipf", True),
    ("fp8", 16, 128, 0, 32, 64, 6, 256, 256, "uniform_topk", False),
    ("fp8", 16, 256, 0, 32, 16, 2, 384, 512, "zipf", True),
]


@pytest.mark.parametrize("dtype,tile_m,tile_n,slack,T,E,k,K,N,routing,swiglu", NK_CASES)
def test_nk_weight_layout_parity(dev, oracle_mod, dtype, tile_m, tile_n, slack, T, E, k, K, N, routing, swiglu):
    """The same product with the weights handed over as [E][N][K]; the oracle keeps the [E][K][N] statement."""
    wl = wk.Workload("parity_nk", T, E, k, K, N, dtype, routing, tile_m, tile_n)
    tiling = mb.Tiling(tile_m, tile_n, 0, 0, 0, slack)
    dt = mb.MOE_DTYPE_FP8_E4M3 if dtype == "fp8" else mb.MOE_DTYPE_BF16
    assert mb.moe_w_layout_supported(dt, tiling, mb.MOE_W_LAYOUT_NK)
    ids = wk.make_routing(wl)
    xs = ws = None
    if dtype == "fp8":
        X, xs = wk.make_x(wl)
        W, ws = wk.make_w(wl)
        if swiglu:
            ws = ws * 4.0
    else:
        X, W = wk.make_x(wl), wk.make_w(wl) * (4.0 if swiglu else 1.0)
    W_nk = W.transpose(1, 2).contiguous()
    R, NO = wl.R, (N // 2 if swiglu else N)
    pad = 4
    buf = torch.empty((R + 2 * pad, NO), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + R]
    tmap = mb.alloc_task_map(T, k, E, tile_m, tile_n, N)
    mb.moe_build_task_map_ex(ids.to(dev), T, k, E, N, tiling, tmap)
    desc = mb.GemmDesc(dt, T, k, E, K, N, tile_m, tile_n, None if xs is None else xs.to(dev), None if ws is None else ws.to(dev),
                       tile_m_slack=slack, epilogue=mb.MOE_EPILOGUE_SWIGLU if swiglu else mb.MOE_EPILOGUE_NONE,
                       w_layout=mb.MOE_W_LAYOUT_NK)
    mb.moe_grouped_gemm(X.to(dev), W_nk.to(dev), ids.to(dev), tmap, Y, desc)
    torch.cuda.synchronize()
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + R:] == POISON), "wrote outside Y"
    got = allbits[pad: pad + R]
    if dtype == "fp8":
        res = oracle_mod.grouped_gemm_fp8(wk.bits(X), wk.bits(W), xs.numpy(), ws.numpy(), ids.numpy())
        Xf = X.view(torch.float8_e4m3fn).double().numpy()
        Wf = W.view(torch.float8_e4m3fn).double().numpy()
        sx, sw = xs.double().numpy(), ws.double().numpy()
    else:
        res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
        Xf, Wf, sx, sw = X.double().numpy(), W.double().numpy(), None, None
    if swiglu:
        _check_swiglu(oracle_mod, got, res, Xf, Wf, ids.numpy(), k, K, sx, sw)
    else:
        from tests.test_gpu_parity import _check_y
        _check_y(got, res, Xf, Wf, ids.numpy(), k, K, H.tol_fp8(K) if dtype == "fp8" else H.tol_bf16(K), sx, sw)


def test_nk_layout_unsupported_tiling_is_refused(dev):
    wl = wk.Workload("nk_args", 8, 4, 2, 64, 128, "bf16", "gauss_topk", 32, 128)
    ids = wk.make_routing(wl).to(dev)
    X, W = wk.make_x(wl, dev), wk.make_w(wl, dev)
    Y = torch.empty((wl.R, wl.N), dtype=torch.bfloat16, device=dev)
    tmap = mb.alloc_task_map(wl.T, wl.k, wl.E, 32, 128, wl.N)
    mb.moe_build_task_map(ids, wl.T, wl.k, wl.E, 32, 128, wl.N, tmap)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, wl.T, wl.k, wl.E, wl.K, wl.N, 32, 128, w_layout=mb.MOE_W_LAYOUT_NK)
    assert mb.moe_grouped_gemm(X, W, ids, tmap, Y, d, check=False) == mb.MOE_ERR_UNSUPPORTED
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, wl.T, wl.k, wl.E, wl.K, wl.N, 32, 128, w_layout=5)
    assert mb.moe_grouped_gemm(X, W, ids, tmap, Y, d, check=False) == mb.MOE_ERR_INVALID_ARG


# ------------------------------------------------------------------ resident workgroups streaming tile after tile
STREAM_CASES = [
    # dtype, tile_n, T, E, k, K, N, routing, swiglu, workgroups
    ("bf16", 128, 40, 16, 2, 256, 1024, "gauss_topk", False, 8),     # every workgroup runs a dozen tiles
    ("bf16", 256, 100, 8, 2, 128, 1024, "zipf", False, 16),          # several m-tiles per expert
    ("bf16", 128, 64, 256, 8, 256, 256, "gauss_topk", True, 24),     # four record groups, fused activation
    ("fp8", 128, 32, 64, 6, 512, 512, "uniform_topk", False, 8),
    ("fp8", 64, 8, 64, 6, 512, 256, "uniform_topk", False, 16),
    ("fp8", 256, 32, 16, 2, 512, 1024, "zipf", True, 8),
]


@pytest.mark.parametrize("dtype,tile_n,T,E,k,K,N,routing,swiglu,wgs", STREAM_CASES)
def test_streaming_kernel_parity(dev, oracle_mod, dtype, tile_n, T, E, k, K, N, routing, swiglu, wgs):
    """16-row tiles with a handful of resident workgroups, so that each streams many tiles back to back; the
    result must equal the oracle's and, bit for bit, the one-workgroup-per-tile launch."""
    wl = wk.Workload("parity_stream", T, E, k, K, N, dtype, routing, 16, tile_n)
    ids = wk.make_routing(wl)
    xs = ws = None
    if dtype == "fp8":
        X, xs = wk.make_x(wl)
        W, ws = wk.make_w(wl)
        if swiglu:
            ws = ws * 4.0
    else:
        X, W = wk.make_x(wl), wk.make_w(wl) * (4.0 if swiglu else 1.0)
    outs = []
    for mode in (wgs, mb.MOE_LAUNCH_PER_TILE):
        if swiglu:
            outs.append(_run_swiglu(dev, wl, ids, X, W, xs, ws, launch_mode=mode))
        else:
            from tests.test_gpu_parity import _run_gemm
            outs.append(_run_gemm(dev, wl, ids, X, W, xs, ws, launch_mode=mode))
    np.testing.assert_array_equal(outs[0], outs[1])
    if dtype == "fp8":
        res = oracle_mod.grouped_gemm_fp8(wk.bits(X), wk.bits(W), xs.numpy(), ws.numpy(), ids.numpy())
        Xf = X.view(torch.float8_e4m3fn).double().numpy()
        Wf = W.view(torch.float8_e4m3fn).double().numpy()
        sx, sw = xs.double().numpy(), ws.double().numpy()
    else:
        res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
        Xf, Wf, sx, sw = X.double().numpy(), W.double().numpy(), None, None
    if swiglu:
        _check_swiglu(oracle_mod, outs[0], res, Xf, Wf, ids.numpy(), k, K, sx, sw)
    else:
        from tests.test_gpu_parity import _check_y
        _check_y(outs[0], res, Xf, Wf, ids.numpy(), k, K, H.tol_fp8(K) if dtype == "fp8" else H.tol_bf16(K), sx, sw)


# ------------------------------------------------------------------ the whole step inside a HIP graph
def test_step_captured_in_a_graph_replays_exactly(dev):
    """Map build + grouped GEMM + combine captured once and replayed with new inputs: every replay must equal the
    eager result bit for bit (the library enqueues kernels only: no memset nodes, no host synchronisation)."""
    wl = wk.decode_fp8(32)
    T, k, E, K, N = wl.T, wl.k, wl.E, wl.K, wl.N
    X, xs = wk.make_x(wl, dev)
    W, ws = wk.make_w(wl, dev)
    ids = wk.make_routing(wl).to(dev)
    wts = torch.rand((T, k), device=dev, dtype=torch.float32)
    tmap = mb.alloc_task_map(T, k, E, wl.tile_m, wl.tile_n, N)
    Y = torch.empty((T * k, N), dtype=torch.bfloat16, device=dev)
    out = torch.empty((T, N), dtype=torch.bfloat16, device=dev)
    desc = mb.GemmDesc(mb.MOE_DTYPE_FP8_E4M3, T, k, E, K, N, wl.tile_m, wl.tile_n, xs, ws)

    def step():
        mb.moe_build_task_map(ids, T, k, E, wl.tile_m, wl.tile_n, N, tmap)
        mb.moe_grouped_gemm(X, W, ids, tmap, Y, desc)
        mb.moe_combine(Y, wts, T, k, N, out)

    step()                      # first call sets the kernels' launch attributes: not a thing to capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    g = torch.Generator(device=dev).manual_seed(5)
    for it in range(4):
        # new tokens and a new routing in the same buffers, eager work and synchronisations between the replays
        X.copy_(torch.randint(0, 120, X.shape, generator=g, device=dev, dtype=torch.uint8).view(X.dtype))
        ids.copy_(torch.stack([torch.randperm(E, generator=g, device=dev)[:k] for _ in range(T)]).to(torch.int32))
        step()
        torch.cuda.synchronize()
        want_Y, want_out = Y.clone(), out.clone()
        Y.fill_(float("nan"))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), want_Y.view(torch.int16)), f"replay {it}: Y differs"
        assert torch.equal(out.view(torch.int16), want_out.view(torch.int16)), f"replay {it}: combine differs"


def test_layer_with_split_k_in_a_graph_replays_exactly(dev):
    """The whole layer (two maps, fused gate+up product, split-k down product with its reduction, weighted sum)
    captured once and replayed on new tokens and routings: every replay equals the eager result bit for bit, i.e.
    the split-k parts are added in a fixed order and nothing in the path needs the host."""
    T, k, E, hidden, inter = 600, 2, 8, 256, 2048
    plan = mb.MoeLayerPlan(T, k, E, hidden, inter, dev)
    assert plan.k_parts > 1
    g = torch.Generator(device=dev).manual_seed(9)
    X = torch.randn((T, hidden), generator=g, device=dev).to(torch.bfloat16)
    W1 = (torch.randn((E, hidden, 2 * inter), generator=g, device=dev) * hidden ** -0.5).to(torch.bfloat16)
    W2 = (torch.randn((E, inter, hidden), generator=g, device=dev) * inter ** -0.5).to(torch.bfloat16)
    ids = torch.stack([torch.randperm(E, generator=g, device=dev)[:k] for _ in range(T)]).to(torch.int32)
    wts = torch.rand((T, k), generator=g, device=dev, dtype=torch.float32)
    plan.forward(X, W1, W2, ids, wts)   # first call sets the kernels' launch attributes: not a thing to capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            plan.forward(X, W1, W2, ids, wts)
    torch.cuda.synchronize()
    for it in range(3):
        X.copy_(torch.randn((T, hidden), generator=g, device=dev).to(torch.bfloat16))
        ids.copy_(torch.stack([torch.randperm(E, generator=g, device=dev)[:k] for _ in range(T)]).to(torch.int32))
        plan.forward(X, W1, W2, ids, wts)
        torch.cuda.synchronize()
        want = plan.out.clone()
        assert bool(torch.isfinite(want.float()).all())
        plan.out.fill_(float("nan"))
        plan.down.fill_(float("nan"))
        plan.workspace.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(plan.out.view(torch.int16), want.view(torch.int16)), f"replay {it}: the layer's output differs"


def test_mfma_probe_runs(dev):
    """The measurement probe launches and completes for both block shapes and operand kinds."""
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    for block in (16, 32):
        for rnd in (False, True):
            assert probe.moe_probe_mfma(block, rnd, 50, sink) == mb.MOE_OK
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0


def test_wavefronts_w_and_w_plus_4_share_a_simd(dev):
    """What the alternating schedule of the large bf16 tiles relies on for its speed (not for its results): the
    hardware puts wavefronts w and w + 4 of a 512-thread workgroup on the same SIMD, two per SIMD."""
    n = 3584
    out = torch.full((n * 8,), -1, dtype=torch.int32, device=dev)
    assert probe.moe_probe_wave_placement(n, out) == mb.MOE_OK
    assert probe.moe_probe_wave_placement(0, out) == mb.MOE_ERR_INVALID_ARG
    simd = out.cpu().numpy().reshape(n, 8)
    assert simd.min() >= 0 and simd.max() <= 3
    assert np.array_equal(simd[:, :4], simd[:, 4:])
    assert np.all(np.sort(simd[:, :4], axis=1) == np.arange(4))


def test_pipeline_probe_runs(dev):
    """Every mode of the tile-loop probe launches and completes; the source buffer is left as it was."""
    g = torch.Generator().manual_seed(5)
    src = torch.randn((513 << 20) // 2, generator=g).to(torch.bfloat16).to(dev)
    before = src[: 1 << 20].clone()
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    for mode in range(1, 13):
        assert probe.moe_probe_pipeline(mode, 64, src, sink) == mb.MOE_OK
    for mode in (4, 12):
        assert probe.moe_probe_pipeline(mode, 64, src[: 1 << 20], sink) == mb.MOE_ERR_INVALID_ARG
    assert probe.moe_probe_pipeline(13, 64, src, sink) == mb.MOE_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(src[: 1 << 20], before)


SPLITK_CASES = [
    # per-expert row counts (k = 1), K, N, order, k_parts
    ([300, 256, 288, 31, 0, 513, 257, 700], 1024, 512, 0, 2),     # full, partly filled and empty experts; 8 k-tiles per part
    ([130, 64, 1, 255], 2048, 256, 1, 4),                          # only the narrow task functions; spread order
    ([600, 90], 1536, 768, 0, 2),                                  # 12 k-tiles per part
]


@pytest.mark.parametrize("counts,K,N,order,parts", SPLITK_CASES)
def test_splitk_parity(dev, oracle_mod, counts, K, N, order, parts):
    """The product with every tile split along K over `parts` workgroups and a reduction kernel: same definition,
    same tolerance; rows outside Y untouched; the workspace is the caller's."""
    from tests.test_gpu_parity import _check_y
    E, T = len(counts), sum(counts)
    wl = wk.Workload("parity_splitk", T, E, 1, K, N, "bf16", "gauss_topk", 256, 256)
    g = torch.Generator().manual_seed(777 + T)
    ids = torch.repeat_interleave(torch.arange(E, dtype=torch.int32), torch.tensor(counts))[torch.randperm(T, generator=g)].reshape(T, 1).contiguous()
    X, W = wk.make_x(wl), wk.make_w(wl)
    pad = 3
    buf = torch.empty((T + 2 * pad, N), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + T]
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map_ex(ids.to(dev), T, 1, E, N, mb.Tiling(256, 256, order, 0, 0, 0), tmap)
    nbytes = mb.moe_splitk_workspace_bytes(T, 1, N, parts)
    assert nbytes == parts * T * N * 4
    guard = 64
    ws = torch.full((nbytes // 4 + 2 * guard,), float("nan"), dtype=torch.float32, device=dev)
    desc = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    mb.moe_grouped_gemm_splitk(X.to(dev), W.to(dev), tmap, Y, desc, parts, ws[guard: guard + nbytes // 4])
    torch.cuda.synchronize()
    assert torch.isnan(ws[:guard]).all() and torch.isnan(ws[guard + nbytes // 4:]).all(), "wrote outside the workspace"
    allbits = buf.cpu().numpy().view(np.uint16)
    assert np.all(allbits[:pad] == POISON) and np.all(allbits[pad + T:] == POISON), "wrote outside Y"
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_y(allbits[pad: pad + T], res, X.double().numpy(), W.double().numpy(), ids.numpy(), 1, K, H.tol_bf16(K))


def test_splitk_argument_errors(dev):
    T, E, K, N = 512, 2, 1024, 256
    X = torch.zeros((T, K), dtype=torch.bfloat16, device=dev)
    W = torch.zeros((E, K, N), dtype=torch.bfloat16, device=dev)
    Y = torch.zeros((T, N), dtype=torch.bfloat16, device=dev)
    ids = torch.zeros((T, 1), dtype=torch.int32, device=dev)
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 256, 256, N, tmap)
    ws = torch.zeros(2 * T * N, dtype=torch.float32, device=dev)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 2, ws, check=False) == mb.MOE_OK
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 3, ws, check=False) == mb.MOE_ERR_UNSUPPORTED
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 4, ws, check=False) == mb.MOE_ERR_UNSUPPORTED      # 4 k-tiles per part
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 2, ws[: T * N], check=False) == mb.MOE_ERR_INVALID_ARG   # too small
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 2, None, check=False) == mb.MOE_ERR_INVALID_ARG
    d128 = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 128, 256)
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d128, 2, ws, check=False) == mb.MOE_ERR_UNSUPPORTED
    dsl = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256, tile_m_slack=32)
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, dsl, 2, ws, check=False) == mb.MOE_ERR_UNSUPPORTED
    torch.cuda.synchronize()


def test_splitk_invalid_map_and_empty_input_are_noops(dev):
    """A map whose routing held an id outside [0, E) makes both kernels of the split-k call do nothing (Y and the
    workspace keep their contents), as it does for the plain product; T = 0 returns at once."""
    T, E, K, N = 300, 4, 1024, 256
    X = torch.ones((T, K), dtype=torch.bfloat16, device=dev)
    W = torch.ones((E, K, N), dtype=torch.bfloat16, device=dev)
    Y = torch.full((T, N), POISON, dtype=torch.int16, device=dev)
    ids = torch.zeros((T, 1), dtype=torch.int32, device=dev)
    ids[17, 0] = E      # out of range
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 256, 256, N, tmap, check=False)
    assert mb.moe_task_map_status(tmap) == mb.MOE_ERR_ROUTING
    ws = torch.full((2 * T * N,), 7.0, dtype=torch.float32, device=dev)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 2, ws, check=False) == mb.MOE_OK
    torch.cuda.synchronize()
    assert bool((Y == POISON).all()) and bool((ws == 7.0).all())
    d0 = mb.GemmDesc(mb.MOE_DTYPE_BF16, 0, 1, E, K, N, 256, 256)
    assert mb.moe_grouped_gemm_splitk(None, None, None, None, d0, 2, None, check=False) == mb.MOE_OK


def test_splitk_mismatched_map_is_a_noop(dev):
    """A valid map that was built for another problem (other T, other N, other tiling, slack rows) or a blob that is
    no map at all: neither the product nor the reduction of the split-k call may touch Y, and the reduction must not
    follow row ids it has no reason to trust."""
    T, E, K, N = 300, 4, 1024, 256
    X = torch.ones((T, K), dtype=torch.bfloat16, device=dev)
    W = torch.ones((E, K, N), dtype=torch.bfloat16, device=dev)
    pad = 4
    buf = torch.full((T + 2 * pad, N), POISON, dtype=torch.int16, device=dev)
    Y = buf[pad: pad + T]
    g = torch.Generator().manual_seed(3)
    ids = torch.randint(0, E, (T, 1), generator=g, dtype=torch.int32).to(dev)
    ws = torch.full((2 * T * N,), 7.0, dtype=torch.float32, device=dev)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    maps = []
    # built for more tokens (its row ids reach past this call's Y), for another width, another tiling, with slack rows
    big = mb.alloc_task_map(4 * T, 1, E, 256, 256, N)
    ids_big = torch.randint(0, E, (4 * T, 1), generator=g, dtype=torch.int32).to(dev)
    mb.moe_build_task_map(ids_big, 4 * T, 1, E, 256, 256, N, big)
    maps.append(big)
    m = mb.alloc_task_map(T, 1, E, 256, 256, 2 * N)
    mb.moe_build_task_map(ids, T, 1, E, 256, 256, 2 * N, m)
    maps.append(m)
    m = mb.alloc_task_map(T, 1, E, 128, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 128, 256, N, m)
    maps.append(m)
    m = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map_ex(ids, T, 1, E, N, mb.Tiling(256, 256, 0, 0, 0, 32), m)
    maps.append(m)
    junk = torch.randint(0, 2 ** 20, (big.numel(),), generator=g, dtype=torch.int32).to(dev)   # not a map: no magic word
    maps.append(junk)
    for tmap in maps:
        assert mb.moe_grouped_gemm_splitk(X, W, tmap, Y, d, 2, ws, check=False) == mb.MOE_OK
        torch.cuda.synchronize()
        assert bool((buf == POISON).all()), "a mismatched map made the split-k call write"
        assert bool((ws == 7.0).all())
    # the matching map still works
    m = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 256, 256, N, m)
    mb.moe_grouped_gemm_splitk(X, W, m, Y, d, 2, ws)
    torch.cuda.synchronize()
    assert bool((buf[:pad] == POISON).all()) and bool((buf[pad + T:] == POISON).all())
    assert bool((Y.view(torch.bfloat16) == float(K)).all())


BATCHED_CASES = [
    # per-expert row counts of the GEMM (k = 1), K, N, slack | reduction: T, k, N, weighted
    ([257, 320, 321, 256, 1, 64, 65, 0, 576], 128, 256, 0, 300, 2, 512, True),
    ([1025, 1040, 991, 1055], 192, 512, 32, 1000, 8, 4096, True),      # 125 reduction tiles among 64 GEMM tiles
    ([300, 0, 0, 513, 129], 192, 512, 0, 70, 6, 264, False),            # plain sum, a ragged last reduction tile
    ([512, 512], 128, 1024, 0, 0, 2, 256, True),                        # empty reduction task: the plain product
    ([40], 128, 256, 32, 4096, 2, 1024, True),                          # one GEMM tile, 128 reduction tiles
]


@pytest.mark.parametrize("order", [0, 2], ids=["ascending", "interleave"])
@pytest.mark.parametrize("counts,K,N,slack,rT,rk,rN,weighted", BATCHED_CASES)
def test_heterogeneous_batch_parity(dev, oracle_mod, counts, K, N, slack, rT, rk, rN, weighted, order):
    """Sec. 3.2 / Alg. 3: GEMM tasks and a reduction task in ONE launch.  The GEMM's Y must equal the oracle's and,
    bit for bit, moe_grouped_gemm's; the reduction's output must equal the oracle's sum and, bit for bit,
    moe_combine's; every element of both outputs is written, nothing outside them."""
    from tests.test_gpu_parity import _build_map, _check_y, _ids_from_counts
    E, T = len(counts), int(sum(counts))
    wl = wk.Workload("parity_batched", T, E, 1, K, N, "bf16", "gauss_topk", 256, 256)
    ids = _ids_from_counts(counts, 11 + E + K)
    X, W = wk.make_x(wl), wk.make_w(wl)
    g = torch.Generator().manual_seed(rT + rk)
    Yin = torch.randn((rT * rk, rN), generator=g).to(torch.bfloat16)
    wts = torch.rand((rT, rk), generator=g, dtype=torch.float32) if weighted else None
    pad = 3
    ybuf = torch.full((T + 2 * pad, N), POISON, dtype=torch.int16, device=dev)
    obuf = torch.full((rT + 2 * pad, rN), POISON, dtype=torch.int16, device=dev)
    Y, out = ybuf[pad: pad + T], obuf[pad: pad + rT]
    tmap = _build_map(ids.to(dev), T, 1, E, 256, 256, N, order, slack=slack)
    desc = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256, tile_m_slack=slack)
    Yin_d, wts_d = Yin.to(dev), None if wts is None else wts.to(dev)
    mb.moe_grouped_gemm_batched(X.to(dev), W.to(dev), tmap, Y, desc, Yin_d, wts_d, rT, rk, rN, out)
    torch.cuda.synchronize()
    yb, ob = ybuf.cpu().numpy().view(np.uint16), obuf.cpu().numpy().view(np.uint16)
    assert np.all(yb[:pad] == POISON) and np.all(yb[pad + T:] == POISON), "wrote outside Y"
    assert np.all(ob[:pad] == POISON) and np.all(ob[pad + rT:] == POISON), "wrote outside the reduction's output"
    got_y, got_o = yb[pad: pad + T], ob[pad: pad + rT]
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    _check_y(got_y, res, X.double().numpy(), W.double().numpy(), ids.numpy(), 1, K, H.tol_bf16(K))
    # the same two results from the two separate calls
    Y2 = torch.full((T, N), POISON, dtype=torch.int16, device=dev)
    mb.moe_grouped_gemm(X.to(dev), W.to(dev), None, tmap, Y2, desc)
    np.testing.assert_array_equal(got_y, H.y_bits(Y2))
    if rT > 0:
        assert not np.any(got_o == POISON), "an element of the reduction's output was never written"
        o64, obf = oracle_mod.combine(wk.bits(Yin), None if wts is None else wts.numpy(), rT, rk)
        err = np.abs(H.bf16_bits_to_f64(got_o) - o64)
        A = np.abs(Yin.double().numpy().reshape(rT, rk, rN) * (1.0 if wts is None else wts.double().numpy()[:, :, None])).sum(axis=1)
        assert np.all(err <= 2.0 ** -8 * np.abs(o64) * 1.001 + (rk + 1) * 2.0 ** -24 * A + 1e-30)
        out2 = torch.full((rT, rN), POISON, dtype=torch.int16, device=dev)
        mb.moe_combine(Yin_d, wts_d, rT, rk, rN, out2)
        np.testing.assert_array_equal(got_o, H.y_bits(out2))


def test_heterogeneous_batch_argument_errors(dev):
    T, E, K, N = 300, 4, 128, 256
    X = torch.ones((T, K), dtype=torch.bfloat16, device=dev)
    W = torch.ones((E, K, N), dtype=torch.bfloat16, device=dev)
    Y = torch.zeros((T, N), dtype=torch.bfloat16, device=dev)
    ids = torch.zeros((T, 1), dtype=torch.int32, device=dev)
    Yin = torch.ones((10 * 2, 64), dtype=torch.bfloat16, device=dev)
    out = torch.zeros((10, 64), dtype=torch.bfloat16, device=dev)
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 256, 256, N, tmap)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    assert mb.moe_grouped_gemm_batched(X, W, tmap, Y, d, Yin, None, 10, 2, 64, out, check=False) == mb.MOE_OK
    assert mb.moe_grouped_gemm_batched(X, W, tmap, Y, d, Yin, None, 10, 2, 60, out, check=False) == mb.MOE_ERR_UNSUPPORTED   # N % 8
    assert mb.moe_grouped_gemm_batched(X, W, tmap, Y, d, None, None, 10, 2, 64, out, check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_grouped_gemm_batched(X, W, tmap, Y, d, Yin, None, 10, 0, 64, out, check=False) == mb.MOE_ERR_INVALID_ARG
    m128 = mb.alloc_task_map(T, 1, E, 128, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 128, 256, N, m128)
    d128 = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 128, 256)
    assert mb.moe_grouped_gemm_batched(X, W, m128, Y, d128, Yin, None, 10, 2, 64, out, check=False) == mb.MOE_ERR_UNSUPPORTED   # no batched kernel
    # a map that does not match makes the whole call a no-op, the reduction included
    out.fill_(7.0)
    Y.fill_(7.0)
    assert mb.moe_grouped_gemm_batched(X, W, m128, Y, d, Yin, None, 10, 2, 64, out, check=False) == mb.MOE_OK
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()) and bool((Y == 7.0).all())


def _tail_blocks(total, k_tiles, cus=32):
    """Block indices that a tail-split launch runs in parts, and the number of parts, per the rule in moe_sb.h
    (ascending sigma order: XCD x owns blocks [x * ceil(total / 8), ...))."""
    per_xcd = (total + 7) // 8
    out = {}
    for x in range(8):
        n_x = max(0, min(per_xcd, total - x * per_xcd))
        full = n_x // cus * cus
        t = n_x - full
        parts, best = 1, 4     # length of the last round in quarters of a tile
        for P in (2, 4):
            if t == 0 or k_tiles % P or k_tiles // P < 8:
                break
            length = -(-t * P // cus) * (4 // P)
            if length < best:
                parts, best = P, length
        if parts > 1:
            for B in range(x * per_xcd + full, x * per_xcd + n_x):
                out[B] = parts
    return out


TAIL_CASES = [
    # tile_m, per-expert row counts (k = 1), K, N  (tile_n = 256)                    tiles -> tail of each XCD
    (256, [300, 0, 513, 129, 255, 700], 2048, 1024),        # 40 tiles: 5 per XCD, all of them tail, 4 parts
    (256, [257, 320, 321, 256, 1, 64, 65, 0, 576], 1024, 512),   # 26 tiles, 4 per XCD (the last XCD fewer), K = 1024: 2 parts at most
    (256, [9000, 6000, 4100], 2048, 1024),                  # 77 m-tiles x 4: 308 tiles, 39 per XCD: 32 whole + 7 tail tiles, 4 parts
    (256, [5000, 5200, 3000], 2048, 1024),                  # 212 tiles, 27 per XCD: no split shortens the round
    (256, [4000, 5200, 2000], 2048, 1024),                  # 180 tiles, 23 per XCD: 4 parts in three sub-rounds
    (256, [300, 200], 512, 256),                            # K too short to split: everything runs whole
    (128, [70, 3, 140, 129, 300], 2048, 1024),              # 128-row tiles (and the 64-row task function for the small ones)
    (128, [2000, 2100, 900], 1024, 2048),                   # 41 m-tiles x 8 = 328 tiles: 32 whole + 9 tail per XCD, 2 parts
    (64, [172, 107, 61, 39, 52, 23, 32, 26], 2048, 1024),   # 64-row tiles, the row counts of a skewed routing
    (-256, [1025, 1040, 991, 1055, 280, 300], 2048, 512),   # (negative: 32 slack rows) tail tiles of 257 .. 287 rows
    (-256, [9000, 6000, 4113], 2048, 1024),                 # slack rows, whole rounds and a tail
]


@pytest.mark.parametrize("tile_m,counts,K,N", TAIL_CASES)
def test_tail_split_parity(dev, oracle_mod, tile_m, counts, K, N):
    """The tiles of a partly filled last round run in 2 or 4 parts along K: Y == oracle, nothing outside Y, every
    element written; every tile outside the tails bit for bit what moe_grouped_gemm gives."""
    from tests.test_gpu_parity import _build_map, _check_y, _ids_from_counts
    slack = 32 if tile_m < 0 else 0
    tile_m = abs(tile_m)
    E, T = len(counts), int(sum(counts))
    wl = wk.Workload("parity_tail", T, E, 1, K, N, "bf16", "gauss_topk", tile_m, 256)
    ids = _ids_from_counts(counts, 13 + E + K)
    X, W = wk.make_x(wl), wk.make_w(wl)
    pad = 3
    buf = torch.full((T + 2 * pad, N), POISON, dtype=torch.int16, device=dev)
    Y = buf[pad: pad + T]
    tmap = _build_map(ids.to(dev), T, 1, E, tile_m, 256, N, slack=slack)
    desc = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, tile_m, 256, tile_m_slack=slack)
    guard = 1024
    nws = mb.moe_tail_split_workspace_bytes(tile_m, 256) // 4
    ws = torch.full((nws + 2 * guard,), float("nan"), dtype=torch.float32, device=dev)
    Xd, Wd = X.to(dev), W.to(dev)
    mb.moe_grouped_gemm_tail_split(Xd, Wd, tmap, Y, desc, ws[guard: guard + nws])
    torch.cuda.synchronize()
    assert bool(torch.isnan(ws[:guard]).all()) and bool(torch.isnan(ws[-guard:]).all()), "wrote outside the workspace"
    bits = buf.cpu().numpy().view(np.uint16)
    assert np.all(bits[:pad] == POISON) and np.all(bits[pad + T:] == POISON), "wrote outside Y"
    got = bits[pad: pad + T]
    assert not np.any(got == POISON), "an output was never written"
    tm = oracle_mod.build_task_map(ids.numpy(), T, 1, E, tile_m, 256, N, tile_m_slack=slack)
    table = oracle_mod.full_table(tm.counts, tile_m, 256, N, tile_m_slack=slack)
    tails = _tail_blocks(tm.total_tiles, K // 64)
    if T <= 3000:
        res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
        _check_y(got, res, X.double().numpy(), W.double().numpy(), ids.numpy(), 1, K, H.tol_bf16(K))
    else:
        # the oracle on a sample of complete rows: the first and last row of every tail tile, and 300 others
        rng = np.random.default_rng(5)
        sel = [int(tm.sorted_rows[tm.offsets[e] + m * tile_m + i]) for B, (e, m, n, rows) in enumerate(table) if B in tails for i in (0, rows - 1)]
        sel = np.array(sorted(set(sel) | set(rng.choice(T, size=300, replace=False).tolist())), dtype=np.int32)
        res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy(), rows=sel)
        flat = ids.numpy().reshape(-1)
        Xf, Wf = X.double().numpy(), W.double().numpy()
        err = np.abs(H.bf16_bits_to_f64(got[sel]) - res.Y64)
        A = np.zeros_like(err)
        for e in range(E):
            m = flat[sel] == e
            if m.any():
                A[m] = np.abs(Xf[sel[m]]) @ np.abs(Wf[e])
        assert np.all(err <= 2.0 ** -8 * np.abs(res.Y64) * 1.001 + H.sum_err_coeff(K, False) * A + 1e-30)
        assert (H.ulp_distance(got[sel], res.Ybf) == 0).mean() > 0.97
    Y2 = torch.full((T, N), POISON, dtype=torch.int16, device=dev)
    mb.moe_grouped_gemm(Xd, Wd, None, tmap, Y2, desc)
    plain = H.y_bits(Y2)
    whole = 0
    for B, (e, m_tile, n_tile, rows) in enumerate(table):
        if B in tails:
            continue
        rr = tm.sorted_rows[tm.offsets[e] + m_tile * tile_m: tm.offsets[e] + m_tile * tile_m + rows]
        np.testing.assert_array_equal(got[rr, n_tile * 256:(n_tile + 1) * 256], plain[rr, n_tile * 256:(n_tile + 1) * 256])
        whole += 1
    assert whole + len(tails) == tm.total_tiles
    if K >= 1024 and tm.total_tiles not in (212,):
        assert len(tails) > 0, "the case must exercise the split"
    if not tails:
        np.testing.assert_array_equal(got, plain)


def test_tail_split_argument_errors(dev):
    T, E, K, N = 300, 4, 1024, 256
    X = torch.ones((T, K), dtype=torch.bfloat16, device=dev)
    W = torch.ones((E, K, N), dtype=torch.bfloat16, device=dev)
    Y = torch.full((T, N), 7.0, dtype=torch.bfloat16, device=dev)
    ids = torch.zeros((T, 1), dtype=torch.int32, device=dev)
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map(ids, T, 1, E, 256, 256, N, tmap)
    ws = torch.empty(mb.moe_tail_split_workspace_bytes(256, 256) // 4, dtype=torch.float32, device=dev)
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    assert mb.moe_tail_split_workspace_bytes(256, 256) == 8 * 128 * 288 * 256 * 4
    assert mb.moe_tail_split_workspace_bytes(64, 256) == 8 * 128 * 64 * 256 * 4
    assert mb.moe_tail_split_workspace_bytes(32, 256) == 0 and mb.moe_tail_split_workspace_bytes(256, 128) == 0
    assert mb.moe_grouped_gemm_tail_split(X, W, tmap, Y, d, ws, check=False) == mb.MOE_OK
    assert mb.moe_grouped_gemm_tail_split(X, W, tmap, Y, d, ws[:1000], check=False) == mb.MOE_ERR_INVALID_ARG
    assert mb.moe_grouped_gemm_tail_split(X, W, tmap, Y, d, None, check=False) == mb.MOE_ERR_INVALID_ARG
    d32 = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 32, 256)
    assert mb.moe_grouped_gemm_tail_split(X, W, tmap, Y, d32, ws, check=False) == mb.MOE_ERR_UNSUPPORTED
    dsl = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256, tile_m_slack=64)
    assert mb.moe_grouped_gemm_tail_split(X, W, tmap, Y, dsl, ws, check=False) == mb.MOE_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((Y == float(K)).all())
    # a map built for another problem: none of the three launches may write
    other = mb.alloc_task_map(2 * T, 1, E, 256, 256, N)
    mb.moe_build_task_map(torch.zeros((2 * T, 1), dtype=torch.int32, device=dev), 2 * T, 1, E, 256, 256, N, other)
    Y.fill_(7.0)
    assert mb.moe_grouped_gemm_tail_split(X, W, other, Y, d, ws, check=False) == mb.MOE_OK
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())


LAYER_CASES = [
    # T, k, E, hidden, inter, routing, weighted
    (300, 2, 8, 256, 384, "zipf", True),
    (40, 2, 8, 128, 256, "gauss_topk", True),          # weight-streaming tiles for both products
    (700, 1, 4, 256, 256, "uniform_topk", False),      # k = 1: the second map equals the first one's routing
    (600, 2, 8, 256, 2048, "gauss_topk", True),        # down product split along K (150 rows per expert, one n-tile)
]


@pytest.mark.parametrize("T,k,E,hidden,inter,routing,weighted", LAYER_CASES)
def test_moe_layer_composition(dev, oracle_mod, T, k, E, hidden, inter, routing, weighted):
    """The whole feed-forward layer of Sec. 2.2 from library calls only.  Each stage is checked against the oracle
    applied to the previous stage's device output, so every comparison keeps the single-stage tolerance."""
    from tests.test_gpu_parity import _check_y
    wl1 = wk.Workload("layer_up", T, E, k, hidden, 2 * inter, "bf16", routing, 16, 128)
    wl2 = wk.Workload("layer_down", T * k, E, 1, inter, hidden, "bf16", routing, 16, 128)
    ids = wk.make_routing(wl1)
    X, W1, W2 = wk.make_x(wl1), wk.make_w(wl1) * 4.0, wk.make_w(wl2)
    g = torch.Generator().manual_seed(77 + T)
    wts = torch.rand((T, k), generator=g, dtype=torch.float32) if weighted else None
    plan = mb.MoeLayerPlan(T, k, E, hidden, inter, dev)
    assert (plan.k_parts > 1) == (inter == 2048), "the case meant for the split-k path must take it"
    for buf in (plan.act, plan.down, plan.out):
        buf.view(torch.int16).fill_(POISON)
    out = plan.forward(X.to(dev), W1.to(dev), W2.to(dev), ids.to(dev), None if wts is None else wts.to(dev))
    torch.cuda.synchronize()
    assert out.data_ptr() == plan.out.data_ptr()
    act_bits = plan.act.cpu().view(torch.int16).numpy().view(np.uint16)
    down_bits = plan.down.cpu().view(torch.int16).numpy().view(np.uint16)
    out_bits = plan.out.cpu().view(torch.int16).numpy().view(np.uint16)
    idn = ids.numpy()
    # stage 1: gate+up product with the fused gated activation
    res1 = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W1), idn)
    _check_swiglu(oracle_mod, act_bits, res1, X.double().numpy(), W1.double().numpy(), idn, k, hidden)
    # stage 2: the activated rows as T*k tokens with one expert each
    flat = idn.reshape(T * k, 1)
    res2 = oracle_mod.grouped_gemm_bf16(act_bits, wk.bits(W2), flat)
    _check_y(down_bits, res2, H.bf16_bits_to_f64(act_bits), W2.double().numpy(), flat, 1, inter, H.tol_bf16(inter))
    # stage 3: weighted sum over the k slots of each token
    out64, outbf = oracle_mod.combine(down_bits, None if wts is None else wts.numpy(), T, k)
    yabs = np.abs(H.bf16_bits_to_f64(down_bits)).reshape(T, k, hidden)
    wabs = np.ones((T, k)) if wts is None else np.abs(wts.double().numpy())
    A = np.einsum("tj,tjn->tn", wabs, yabs)
    tight = 2.0 ** -8 * np.abs(out64) * 1.001 + (k + 1) * 2.0 ** -24 * A + 1e-30
    err = np.abs(H.bf16_bits_to_f64(out_bits) - out64)
    assert np.all(err <= tight), f"max err/tight = {(err / tight).max():.3f}"
    assert (H.ulp_distance(out_bits, outbf) == 0).mean() > 0.97
