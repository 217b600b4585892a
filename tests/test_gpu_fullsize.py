"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot compute these problems whole (1-4 TFLOP), so: the task map is compared whole
(bit-exact), and Y is compared on samples the oracle computes one by one -- a few elements in
EVERY tile of the map (its first and last valid row, random columns), plus complete rows that
straddle tile boundaries -- and with properties that hold at any size (every element written,
nothing outside Y touched).
"""
import numpy as np
import pytest
import torch

from paper_2501_16103_amd import binding as mb
from paper_2501_16103_amd import workloads as wk
from tests import helpers as H

pytestmark = pytest.mark.gpu

POISON = 0x7FC1


def _gather_columns(W, experts, cols):
    """W [E,K,N] on the device -> host array [S, K] of the columns W[experts[i], :, cols[i]] (storage bits)."""
    e = torch.as_tensor(experts, dtype=torch.long, device=W.device)
    n = torch.as_tensor(cols, dtype=torch.long, device=W.device)
    out = []
    for lo in range(0, len(e), 4096):
        out.append(W[e[lo:lo + 4096], :, n[lo:lo + 4096]].contiguous().cpu())
    return torch.cat(out)


def _run_full(wl, dev, order=0, k_parts=1, launch_mode=0, inputs=None):
    """`inputs`: (X, W, xs, ws) already on the device, to run one set of weights through several launches."""
    ids = wk.make_routing(wl)
    if inputs is not None:
        X, W, xs, ws = inputs
    elif wl.dtype == "fp8":
        X, xs = wk.make_x(wl, dev)
        W, ws = wk.make_w(wl, dev)
    else:
        X, W, xs, ws = wk.make_x(wl, dev), wk.make_w(wl, dev), None, None
    pad = 2
    buf = torch.empty((wl.R + 2 * pad, wl.N), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + wl.R]
    tmap = mb.alloc_task_map(wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N, dev)
    mb.moe_build_task_map_ex(ids.to(dev), wl.T, wl.k, wl.E, wl.N, mb.Tiling(wl.tile_m, wl.tile_n, order, 0, 0, wl.tile_m_slack), tmap)
    dt = mb.MOE_DTYPE_FP8_E4M3 if wl.dtype == "fp8" else mb.MOE_DTYPE_BF16
    desc = mb.GemmDesc(dt, wl.T, wl.k, wl.E, wl.K, wl.N, wl.tile_m, wl.tile_n, xs, ws, tile_m_slack=wl.tile_m_slack,
                       launch_mode=launch_mode)
    if k_parts > 1:
        work = torch.empty(mb.moe_splitk_workspace_bytes(wl.T, wl.k, wl.N, k_parts) // 4, dtype=torch.float32, device=dev)
        mb.moe_grouped_gemm_splitk(X, W, tmap, Y, desc, k_parts, work)
    else:
        mb.moe_grouped_gemm(X, W, ids.to(dev), tmap, Y, desc)
    torch.cuda.synchronize()
    assert mb.moe_task_map_status(tmap) == mb.MOE_OK
    # properties that hold at any size
    assert bool((buf[:pad] == POISON).all()) and bool((buf[pad + wl.R:] == POISON).all()), "wrote outside Y"
    assert not bool((Y == POISON).any()), "some output was never written"
    return ids, X, W, xs, ws, Y, tmap


def _sample_points(tm, table, rng, per_tile):
    """(r, n) samples: in every tile its first and last valid row at random columns, plus the tile's corners."""
    rr, nn = [], []
    for e, m_tile, n_tile, rows in table:
        base = tm.offsets[e] + m_tile * tm.tile_m
        n0 = n_tile * tm.tile_n
        cand_rows = [0, rows - 1]
        for i in range(per_tile):
            lr = cand_rows[i % 2] if i < 2 else int(rng.integers(0, rows))
            lc = (0 if i == 0 else tm.tile_n - 1) if i < 2 else int(rng.integers(0, tm.tile_n))
            rr.append(int(tm.sorted_rows[base + lr]))
            nn.append(n0 + lc)
    return np.array(rr, np.int32), np.array(nn, np.int32)


def _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn):
    """Compare Y[rr, nn] with the oracle, element by element, through a compact stand-in problem:
    sample i becomes token i with its own one-column expert, so the oracle does the same sums."""
    flat = ids.numpy().reshape(-1)
    toks = rr // wl.k
    exps = flat[rr]
    Xs = X[torch.as_tensor(toks, dtype=torch.long, device=X.device)].cpu()
    Wc = _gather_columns(W, exps, nn)                      # [S, K]
    S = len(rr)
    ids_c = np.arange(S, dtype=np.int32).reshape(S, 1)
    sel = np.arange(S, dtype=np.int32)
    zero = np.zeros(S, dtype=np.int32)
    if wl.dtype == "fp8":
        xsc = xs.cpu().numpy()[toks]
        wsc = ws.cpu().numpy()[exps]
        want = oracle_mod.gemm_elements(Xs.numpy(), Wc.numpy().reshape(S, wl.K, 1), ids_c, 1, sel, zero, x_scale=xsc, w_scale=wsc)
        Xf = Xs.view(torch.float8_e4m3fn).double().numpy()
        Wf = Wc.view(torch.float8_e4m3fn).double().numpy()
        sc = xsc.astype(np.float64) * wsc.astype(np.float64)
        tol = H.tol_fp8(wl.K)
    else:
        want = oracle_mod.gemm_elements(wk.bits(Xs), wk.bits(Wc).reshape(S, wl.K, 1), ids_c, 1, sel, zero)
        Xf, Wf, sc, tol = Xs.double().numpy(), Wc.double().numpy(), 1.0, H.tol_bf16(wl.K)
    got_bits = H.y_bits(Y[torch.as_tensor(rr, dtype=torch.long, device=Y.device), torch.as_tensor(nn, dtype=torch.long, device=Y.device)])
    got = H.bf16_bits_to_f64(got_bits)
    err = np.abs(got - want)
    scale = np.linalg.norm(Xf, axis=1) * np.linalg.norm(Wf, axis=1) * sc
    assert np.all(err <= tol * scale), f"max err/scale {(err / scale).max():.3e} > {tol:.3e}"
    A = (np.abs(Xf) * np.abs(Wf)).sum(axis=1) * sc
    tight = 2.0 ** -8 * np.abs(want) * 1.001 + H.sum_err_coeff(wl.K, wl.dtype == "fp8") * A + 1e-30
    assert np.all(err <= tight), f"max err/tight {(err / tight).max():.3f}"
    want_bits = np.array([oracle_mod.f64_to_bf16_rne(float(v)) for v in want], dtype=np.uint16)
    assert (H.ulp_distance(got_bits, want_bits) == 0).mean() > 0.97


FULL = [
    # workload, samples per tile, complete rows, sigma order
    (wk.mixtral_up(4096), 8, 64, 0),
    (wk.mixtral_up(4096).with_T(4096, tile_m_slack=0), 8, 64, 0),   # the same point with the plain ceil tiling
    (wk.mixtral_up(4096).with_T(4096, tile_m_slack=64), 8, 64, 0),  # and with 64 slack rows (32-row MFMA blocks)
    (wk.mixtral_up(256), 8, 32, 0),
    (wk.decode_fp8(4096), 4, 32, 0),                                # the fp8 layer at a prefill size: 256-row tiles
    (wk.mixtral_up(16), 8, 32, 0),
    (wk.mixtral_down_zipf(4096), 8, 64, 0),
    (wk.mixtral_down_zipf(256), 8, 32, 0),
    (wk.paper_eval("balanced"), 8, 64, 0),                          # Sec. 5: every expert 512 rows
    (wk.paper_eval("best"), 8, 64, 0),                              # Sec. 5: k experts hold everything, E - k are empty
    (wk.paper_eval("worst"), 8, 64, 0),
    (wk.paper_eval("worst"), 8, 64, 1),
    (wk.mixtral_down_zipf(4096), 8, 64, 1),
    (wk.paper_eval("worst"), 8, 64, 2),
    (wk.mixtral_down_zipf(4096), 8, 64, 2),
    (wk.decode_fp8(32), 8, 64, 0),
    (wk.decode_fp8(8), 8, 48, 0),
    (wk.decode_fp8(1), 8, 6, 0),
]


@pytest.mark.parametrize("wl,per_tile,nrows,order", FULL, ids=lambda v: f"{v.name}_T{v.T}" if hasattr(v, "name") else str(v))
def test_full_size_sampled(oracle_mod, wl, per_tile, nrows, order):
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(wl.T * 7 + wl.E)
    ids, X, W, xs, ws, Y, tmap = _run_full(wl, dev, order)
    # task map: whole and bit-exact
    tm = oracle_mod.build_task_map(ids.numpy(), wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N, order=order, tile_m_slack=wl.tile_m_slack)
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    table = oracle_mod.full_table(tm.counts, wl.tile_m, wl.tile_n, wl.N, sigma=tm.sigma, tile_m_slack=wl.tile_m_slack)
    assert len(table) == tm.total_tiles
    # (a) samples in every tile
    rr, nn = _sample_points(tm, table, rng, per_tile)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn)
    # (b) complete rows: first / last row of expert segments and rows next to m-tile boundaries, then random
    rows = []
    for e in range(wl.E):
        c = int(tm.counts[e])
        if c == 0:
            continue
        o = int(tm.offsets[e])
        for pos in (0, c - 1, min(c - 1, wl.tile_m - 1), min(c - 1, wl.tile_m)):
            rows.append(int(tm.sorted_rows[o + pos]))
    rows = list(dict.fromkeys(rows))
    rng.shuffle(rows)
    rows = rows[: nrows // 2] + rng.choice(wl.R, size=min(wl.R, nrows - min(len(rows), nrows // 2)), replace=False).tolist()
    rows = np.array(list(dict.fromkeys(rows)), dtype=np.int32)
    cols = rng.choice(wl.N, size=min(wl.N, 256), replace=False).astype(np.int32)
    cols[:2] = (0, wl.N - 1)
    rr = np.repeat(rows, len(cols))
    nn = np.tile(cols, len(rows))
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn)


def test_split_k_full_size_sampled(oracle_mod):
    """The down projection of a Mixtral-sized layer at 512 tokens (1024 routed rows, 8 experts, K = 14336, N = 4096)
    in the split-k launch the layer plan picks for it: samples in every tile and complete rows."""
    wl = wk.Workload("mixtral_down_layer", 1024, 8, 1, 14336, 4096, "bf16", "gauss_topk", 256, 256)
    k_parts = mb.moe_default_k_parts(wl.T, wl.k, wl.E, wl.K, wl.N)
    assert k_parts == 2
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(512)
    ids, X, W, xs, ws, Y, tmap = _run_full(wl, dev, 0, k_parts)
    tm = oracle_mod.build_task_map(ids.numpy(), wl.T, wl.k, wl.E, 256, 256, wl.N)
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    table = oracle_mod.full_table(tm.counts, 256, 256, wl.N)
    rr, nn = _sample_points(tm, table, rng, 8)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn)
    rows = rng.choice(wl.R, size=24, replace=False).astype(np.int32)
    cols = rng.choice(wl.N, size=128, replace=False).astype(np.int32)
    cols[:2] = (0, wl.N - 1)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, np.repeat(rows, len(cols)), np.tile(cols, len(rows)))


def test_fine_grained_full_size_sampled(oracle_mod):
    """E=256, top-8, 15 GB of weights resident: T=2048 in the benchmark's tiling, 2 samples per tile."""
    wl = wk.fine_grained(2048)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(11)
    ids, X, W, xs, ws, Y, tmap = _run_full(wl, dev)
    tm = oracle_mod.build_task_map(ids.numpy(), wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N)
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    table = oracle_mod.full_table(tm.counts, wl.tile_m, wl.tile_n, wl.N)
    rr, nn = _sample_points(tm, table, rng, 2)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn)


def test_fine_grained_T128_full_size_sampled(oracle_mod):
    """E=256, top-8, T=128 (1024 routed rows over 256 experts: counts of 0 to about 10, several experts empty, Sec. 4.1):
    16-row tiles in the resident launch the benchmark times, and in the one-workgroup-per-tile launch; both must agree
    bit for bit, and with the oracle on 2 samples per tile plus complete rows."""
    wl = wk.fine_grained(128)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(10)
    inputs = (wk.make_x(wl, dev), wk.make_w(wl, dev), None, None)
    ids, X, W, xs, ws, Y, tmap = _run_full(wl, dev, inputs=inputs)
    tm = oracle_mod.build_task_map(ids.numpy(), wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N)
    assert (tm.counts == 0).any(), "the point must have empty experts"
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    table = oracle_mod.full_table(tm.counts, wl.tile_m, wl.tile_n, wl.N, sigma=tm.sigma)
    assert len(table) == tm.total_tiles
    rr, nn = _sample_points(tm, table, rng, 2)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn)
    # complete rows: first and last row of every tenth expert's segment, then random ones
    rows = []
    for e in range(0, wl.E, 10):
        c, o = int(tm.counts[e]), int(tm.offsets[e])
        if c:
            rows += [int(tm.sorted_rows[o]), int(tm.sorted_rows[o + c - 1])]
    rows += rng.choice(wl.R, size=16, replace=False).tolist()
    rows = np.array(list(dict.fromkeys(rows))[:40], dtype=np.int32)
    assert len(rows) >= 32
    cols = rng.choice(wl.N, size=256, replace=False).astype(np.int32)
    cols[:2] = (0, wl.N - 1)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, np.repeat(rows, len(cols)), np.tile(cols, len(rows)))
    y_resident = Y.clone()
    _, _, _, _, _, Y1, _ = _run_full(wl, dev, launch_mode=mb.MOE_LAUNCH_PER_TILE, inputs=inputs)
    assert torch.equal(y_resident, Y1), "resident and per-tile launches differ"


def test_fine_grained_T8192_full_size_sampled(oracle_mod):
    """E=256, top-8, T=8192: 256-row tiles with slack rows (about one tile per expert), 2 samples per tile."""
    wl = wk.fine_grained(8192)
    assert wl.tile_m_slack > 0
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(12)
    ids, X, W, xs, ws, Y, tmap = _run_full(wl, dev)
    tm = oracle_mod.build_task_map(ids.numpy(), wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N, tile_m_slack=wl.tile_m_slack)
    want = H.expected_blob(tm)
    np.testing.assert_array_equal(tmap.cpu().numpy()[: len(want)], want)
    table = oracle_mod.full_table(tm.counts, wl.tile_m, wl.tile_n, wl.N, tile_m_slack=wl.tile_m_slack)
    assert table[:, 3].max() > wl.tile_m, "the point must exercise the slack rows"
    rr, nn = _sample_points(tm, table, rng, 2)
    _check_elements(oracle_mod, wl, ids, X, W, xs, ws, Y, rr, nn)


def test_headline_with_fused_activation_sampled(oracle_mod):
    """The headline shape with the gated activation fused into the epilogue: 4 samples in every tile."""
    wl = wk.mixtral_up(4096)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(13)
    ids = wk.make_routing(wl)
    X = wk.make_x(wl, dev)
    W = wk.make_w(wl, dev)
    W.mul_(4.0)   # gates of a few units
    I = wl.N // 2
    pad = 2
    buf = torch.empty((wl.R + 2 * pad, I), dtype=torch.int16, device=dev)
    buf.fill_(POISON)
    Y = buf[pad: pad + wl.R]
    tmap = mb.alloc_task_map(wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N, dev)
    mb.moe_build_task_map_ex(ids.to(dev), wl.T, wl.k, wl.E, wl.N, mb.Tiling(wl.tile_m, wl.tile_n, 0, 0, 0, wl.tile_m_slack), tmap)
    mb.moe_grouped_gemm(X, W, ids.to(dev), tmap, Y,
                        mb.GemmDesc(mb.MOE_DTYPE_BF16, wl.T, wl.k, wl.E, wl.K, wl.N, wl.tile_m, wl.tile_n,
                                    tile_m_slack=wl.tile_m_slack, epilogue=mb.MOE_EPILOGUE_SWIGLU))
    torch.cuda.synchronize()
    assert bool((buf[:pad] == POISON).all()) and bool((buf[pad + wl.R:] == POISON).all()), "wrote outside Y"
    assert not bool((Y == POISON).any()), "some output was never written"
    tm = oracle_mod.build_task_map(ids.numpy(), wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N, tile_m_slack=wl.tile_m_slack)
    table = oracle_mod.full_table(tm.counts, wl.tile_m, wl.tile_n, wl.N, tile_m_slack=wl.tile_m_slack)
    rr, nn = _sample_points(tm, table, rng, 4)      # nn: weight columns of the tile; the tile's outputs are half as many
    out_col = (nn // wl.tile_n) * (wl.tile_n // 2) + (nn % wl.tile_n) // 2
    flat = ids.numpy().reshape(-1)
    toks, exps = rr // wl.k, flat[rr]
    Xs = X[torch.as_tensor(toks, dtype=torch.long, device=dev)].cpu()
    S = len(rr)
    ids_c = np.arange(S, dtype=np.int32).reshape(S, 1)
    sel, zero = np.arange(S, dtype=np.int32), np.zeros(S, dtype=np.int32)
    vals, absum = [], []
    for cols in (out_col, out_col + I):             # gate column, up column
        Wc = _gather_columns(W, exps, cols)
        vals.append(oracle_mod.gemm_elements(wk.bits(Xs), wk.bits(Wc).reshape(S, wl.K, 1), ids_c, 1, sel, zero))
        absum.append((np.abs(Xs.double().numpy()) * np.abs(Wc.double().numpy())).sum(axis=1))
    H64, Hbf = oracle_mod.swiglu(np.stack(vals, axis=1))
    H64, Hbf = H64[:, 0], Hbf[:, 0]
    got_bits = H.y_bits(Y[torch.as_tensor(rr, dtype=torch.long, device=dev), torch.as_tensor(out_col, dtype=torch.long, device=dev)])
    got = H.bf16_bits_to_f64(got_bits)
    g, u = vals
    eps_g, eps_u = (H.sum_err_coeff(wl.K, False) * a for a in absum)
    silu = g / (1.0 + np.exp(-g))
    tight = 2.0 ** -8 * np.abs(H64) * 1.001 + 1.1 * eps_g * np.abs(u) + np.abs(silu) * eps_u + 4e-6 * np.abs(H64) + 1e-30
    err = np.abs(got - H64)
    assert np.all(err <= tight), f"max err/tight {(err / tight).max():.3f}"
    assert (H.ulp_distance(got_bits, Hbf) == 0).mean() > 0.95
