"""CPU pins of the oracle's result and number formats.

The product has a plain definition (Sec. 2.2: token tensor times each selected
expert's weight), so the oracle is pinned against an independent library
matmul in fp64 on explicitly gathered rows, against hand-worked values, and
against symmetries; bf16 / e4m3 handling is pinned against the tensor library's
own conversions and against values that follow from the format definitions.
"""
import json
import os
import struct

import numpy as np
import pytest
import torch

from paper_2501_16103_amd import workloads as wk

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.bfloat16).contiguous().view(torch.int16).numpy().view(np.uint16)


def _from_bits(b: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)


def _bf16_val(bits_: int) -> float:
    return struct.unpack("<f", struct.pack("<I", (bits_ & 0xFFFF) << 16))[0]


def _nearest_even_bf16(x: float) -> int:
    """Exact single rounding of a double to bf16: pick, among the library's candidate and its two
    neighbours on the bf16 grid, the value nearest to x in exact rational arithmetic (ties: even)."""
    from fractions import Fraction
    c = int(_bf16_bits(torch.tensor([x], dtype=torch.float64))[0])
    best = None
    for cand in (c - 1, c, c + 1):
        if cand < 0 or (cand & 0x7FFF) > 0x7F80:
            continue
        v = _bf16_val(cand)
        if np.isinf(v):
            continue
        d = abs(Fraction(x) - Fraction(v))
        key = (d, cand & 1)
        if best is None or key < best[0]:
            best = (key, cand)
    return best[1]


def _assert_bf16_of_f64(Ybf: np.ndarray, Y64: np.ndarray):
    """Ybf must be the single-rounding RNE of Y64.  The library's double->bf16 cast goes through
    fp32 (two roundings), so where the two differ the exact rational check decides."""
    lib = _bf16_bits(torch.from_numpy(Y64))
    diff = np.argwhere(Ybf != lib)
    assert len(diff) <= max(2, Ybf.size // 500)
    for idx in map(tuple, diff):
        assert int(Ybf[idx]) == _nearest_even_bf16(float(Y64[idx]))
    # and a random sample of agreeing elements is checked exactly too
    flat = np.random.default_rng(0).choice(Ybf.size, size=min(200, Ybf.size), replace=False)
    for f in flat:
        idx = np.unravel_index(f, Ybf.shape)
        assert int(Ybf[idx]) == _nearest_even_bf16(float(Y64[idx]))


# ------------------------------------------------------------------ formats
def test_bf16_decode_matches_definition(oracle_mod):
    for bits_, val in [(0x3F80, 1.0), (0xBF80, -1.0), (0x4000, 2.0), (0x3F00, 0.5), (0x0000, 0.0),
                       (0x3FC0, 1.5), (0x0080, 2.0 ** -126), (0x0001, 2.0 ** -133), (0x7F7F, (2 - 2 ** -7) * 2.0 ** 127)]:
        assert oracle_mod.bf16_to_f32(bits_) == val


def test_bf16_rne_hand_cases(oracle_mod):
    f = oracle_mod.f32_to_bf16_rne
    d = oracle_mod.f64_to_bf16_rne
    # 1 + 2^-8 is exactly halfway between 1.0 (even) and 1+2^-7 -> 1.0
    assert f(1.0 + 2.0 ** -8) == 0x3F80 and d(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even) -> up
    assert f(1.0 + 3 * 2.0 ** -8) == 0x3F82 and d(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # just above the tie rounds up
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -20) == 0x3F81 and d(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    # carry into the exponent: 2 - 2^-9 -> 2.0
    assert f(2.0 - 2.0 ** -9) == 0x4000 and d(2.0 - 2.0 ** -9) == 0x4000
    # sign, zero, infinity, overflow to infinity
    assert f(-1.0) == 0xBF80 and d(-0.0) == 0x8000 and f(float("inf")) == 0x7F80
    assert d(1e39) == 0x7F80 and d(-1e39) == 0xFF80
    # fp64 -> bf16 in one rounding differs from going through fp32 first (double rounding)
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30  # above the tie in fp64, on the tie after fp32 rounding
    assert d(x) == 0x3F81 and f(np.float32(x)) == 0x3F80


def test_bf16_rne_matches_tensor_library(oracle_mod):
    g = torch.Generator().manual_seed(7)
    x = torch.randn(20000, generator=g) * torch.exp(torch.randn(20000, generator=g) * 8)
    # add exact ties
    base = torch.randn(2000, generator=g).to(torch.bfloat16).to(torch.float32)
    ulp = (base.abs() * 2.0 ** -8)
    x = torch.cat([x, base + ulp * 0.5, base - ulp * 0.5])
    want = _bf16_bits(x)
    got = np.array([oracle_mod.f32_to_bf16_rne(float(v)) for v in x.tolist()], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)
    got64 = np.array([oracle_mod.f64_to_bf16_rne(float(v)) for v in x.tolist()], dtype=np.uint16)
    np.testing.assert_array_equal(got64, want)  # an fp32 value converts the same from fp64


def test_e4m3_all_codes(oracle_mod):
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for c in range(256):
        v = oracle_mod.e4m3_to_f32(c)
        s, E, m = c >> 7, (c >> 3) & 15, c & 7
        if E == 15 and m == 7:
            assert np.isnan(v) and np.isnan(lib[c])
            continue
        want = (2.0 ** -6) * (m / 8.0) if E == 0 else (2.0 ** (E - 7)) * (1 + m / 8.0)
        want = -want if s else want
        assert v == want == lib[c]
    assert oracle_mod.e4m3_to_f32(0x7E) == 448.0 and oracle_mod.e4m3_to_f32(0x01) == 2.0 ** -9


# ------------------------------------------------------------------ result
def test_two_expert_values_hand_example(oracle_mod):
    with open(os.path.join(GOLD, "two_expert_values.json")) as f:
        g = json.load(f)
    X = _bf16_bits(torch.tensor(g["X"], dtype=torch.float32))
    W = _bf16_bits(torch.tensor(g["W"], dtype=torch.float32))
    res = oracle_mod.grouped_gemm_bf16(X, W, np.array(g["topk_ids"], np.int32))
    np.testing.assert_array_equal(res.Y64, np.array(g["Y_by_flat_row"], dtype=np.float64))
    np.testing.assert_array_equal(res.Y32, np.array(g["Y_by_flat_row"], dtype=np.float32))
    np.testing.assert_array_equal(_from_bits(res.Ybf).float().numpy(), np.array(g["Y_by_flat_row"], np.float32))


def _problem(T, E, k, K, N, seed, dtype="bf16", routing="gauss_topk"):
    wl = wk.Workload(f"pin{seed}", T, E, k, K, N, dtype, routing)
    return wl, wk.make_routing(wl), wk.make_x(wl), wk.make_w(wl)


@pytest.mark.parametrize("T,E,k,K,N", [(5, 3, 2, 48, 40), (64, 8, 2, 256, 512), (17, 9, 3, 130, 70)])
def test_bf16_against_library_matmul(oracle_mod, T, E, k, K, N):
    """Gather rows explicitly and multiply with the library in fp64: K != N, so a transposed
    operand, a wrong expert, a wrong token or a dropped term cannot pass."""
    wl, ids, X, W = _problem(T, E, k, K, N, seed=T)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    Xd, Wd = X.double(), W.double()
    for r in range(T * k):
        t, e = r // k, int(ids.reshape(-1)[r])
        want = Xd[t] @ Wd[e]
        np.testing.assert_allclose(res.Y64[r], want.numpy(), rtol=1e-12, atol=1e-12)
        # fp32 sequential accumulation stays within its forward error bound K*eps*sum|x||w|
        bound = K * 2.0 ** -24 * (Xd[t].abs() @ Wd[e].abs()).numpy() + 1e-30
        assert np.all(np.abs(res.Y32[r].astype(np.float64) - want.numpy()) <= bound)
    # stored bf16 = one RNE rounding of the fp64 sum
    _assert_bf16_of_f64(res.Ybf, res.Y64)


def test_reduces_to_plain_and_batched_gemm(oracle_mod):
    # E=1, k=1: one plain GEMM
    wl, ids, X, W = _problem(12, 1, 1, 64, 24, seed=1)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    np.testing.assert_allclose(res.Y64, (X.double() @ W[0].double()).numpy(), rtol=1e-12, atol=1e-12)
    # every token to every expert (k=E): a batched GEMM, Y[t,j] = X[t] @ W[ids[t,j]]
    wl, ids, X, W = _problem(6, 4, 4, 32, 16, seed=2)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    bat = torch.einsum("tk,ekn->ten", X.double(), W.double())  # [T,E,N]
    want = torch.stack([bat[t, ids[t].long()] for t in range(6)]).reshape(-1, 16)
    np.testing.assert_allclose(res.Y64, want.numpy(), rtol=1e-12, atol=1e-12)


def test_identity_weight_returns_gathered_tokens(oracle_mod):
    T, E, k, K = 9, 4, 2, 32
    wl, ids, X, _ = _problem(T, E, k, K, K, seed=3)
    W = torch.eye(K).to(torch.bfloat16).expand(E, K, K).contiguous()
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    want = wk.bits(X)[np.arange(T * k) // k]
    np.testing.assert_array_equal(res.Ybf, want)


def test_symmetries(oracle_mod):
    T, E, k, K, N = 10, 5, 2, 64, 48
    wl, ids, X, W = _problem(T, E, k, K, N, seed=4)
    base = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy()).Y64.reshape(T, k, N)
    # permuting tokens permutes Y's token axis
    perm = torch.randperm(T, generator=torch.Generator().manual_seed(0))
    p = oracle_mod.grouped_gemm_bf16(wk.bits(X[perm]), wk.bits(W), ids[perm].numpy()).Y64.reshape(T, k, N)
    np.testing.assert_array_equal(p, base[perm.numpy()])
    # relabelling experts together with W leaves Y unchanged
    ep = torch.randperm(E, generator=torch.Generator().manual_seed(1))
    inv = torch.empty_like(ep)
    inv[ep] = torch.arange(E)
    q = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W[ep]), inv[ids.long()].int().numpy()).Y64.reshape(T, k, N)
    np.testing.assert_array_equal(q, base)


def test_row_subset_and_single_elements(oracle_mod):
    wl, ids, X, W = _problem(20, 6, 3, 96, 80, seed=5)
    full = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    rows = np.array([59, 0, 17, 33], dtype=np.int32)
    sub = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy(), rows=rows)
    np.testing.assert_array_equal(sub.Y64, full.Y64[rows])
    np.testing.assert_array_equal(sub.Ybf, full.Ybf[rows])
    rr = np.array([0, 59, 31, 31], np.int32)
    nn = np.array([0, 79, 5, 40], np.int32)
    el = oracle_mod.gemm_elements(wk.bits(X), wk.bits(W), ids.numpy(), 3, rr, nn)
    np.testing.assert_allclose(el, full.Y64[rr, nn], rtol=1e-13)
    ns = oracle_mod.norm_scale_elements(wk.bits(X), wk.bits(W), ids.numpy(), 3, rr, nn)
    for i in range(4):
        t, e = rr[i] // 3, int(ids.reshape(-1)[rr[i]])
        want = float(X[t].double().norm() * W[e, :, nn[i]].double().norm())
        assert abs(ns[i] - want) <= 1e-12 * want


@pytest.mark.parametrize("T,E,k,K,N", [(8, 16, 6, 128, 64), (3, 5, 2, 256, 48)])
def test_fp8_against_library_dequant_matmul(oracle_mod, T, E, k, K, N):
    wl, ids, (Xq, xs), (Wq, ws) = _problem(T, E, k, K, N, seed=6, dtype="fp8", routing="uniform_topk")
    res = oracle_mod.grouped_gemm_fp8(Xq.numpy(), Wq.numpy(), xs.numpy(), ws.numpy(), ids.numpy())
    Xd = Xq.view(torch.float8_e4m3fn).to(torch.float64)
    Wd = Wq.view(torch.float8_e4m3fn).to(torch.float64)
    for r in range(T * k):
        t, e = r // k, int(ids.reshape(-1)[r])
        want = (Xd[t] @ Wd[e]) * float(xs[t]) * float(ws[e])
        np.testing.assert_allclose(res.Y64[r], want.numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(res.Y32[r], want.numpy(), rtol=1e-4, atol=1e-6)
    _assert_bf16_of_f64(res.Ybf, res.Y64)
    # the quantised problem still approximates the unquantised one (scales used the right way round)
    g = torch.Generator().manual_seed(0)
    assert float(xs.min()) > 0 and float(ws.min()) > 0
    el = oracle_mod.gemm_elements(Xq.numpy(), Wq.numpy(), ids.numpy(), k, [0, T * k - 1], [0, N - 1],
                                  x_scale=xs.numpy(), w_scale=ws.numpy())
    np.testing.assert_allclose(el, res.Y64[[0, T * k - 1], [0, N - 1]], rtol=1e-13)


def test_fp8_quantisation_recipe_roundtrip():
    wl = wk.decode_fp8(8)
    Xq, xs = wk.make_x(wl)
    deq = Xq.view(torch.float8_e4m3fn).float() * xs[:, None]
    # per-token scale maps the row maximum onto the largest finite e4m3 value
    assert torch.all(Xq.view(torch.float8_e4m3fn).float().abs().amax(dim=1) == 448.0)
    g = wk._gen("cpu", wl.name, wl.T, "x")
    x = torch.randn(wl.T, wl.K, generator=g)
    assert float((deq - x).abs().max()) < 0.07 * float(x.abs().max())


def test_statistics_at_config_scale(oracle_mod):
    """X ~ N(0,1), W ~ N(0,1/K)  =>  Y ~ N(0,1): mean square close to 1."""
    wl = wk.tiny()
    ids, X, W = wk.make_routing(wl), wk.make_x(wl), wk.make_w(wl)
    res = oracle_mod.grouped_gemm_bf16(wk.bits(X), wk.bits(W), ids.numpy())
    ms = float((res.Y64 ** 2).mean())
    assert 0.9 < ms < 1.1
