"""CPU pins of the oracle's neighbours of the product: the gated activation and the sum over a token's experts.

Pinned against closed forms, an independent library (torch.nn.functional.silu, numpy einsum in fp64) and
hand values; a swapped gate/up half, a wrong sign in the exponent, a missing weight or a wrong (t, j) stride
fails at least one of them.
"""
import math

import numpy as np
import torch

from tests import helpers as H


def test_swiglu_hand_values(oracle_mod):
    # gate | up, N = 4: silu(0) = 0, silu(ln 3) = ln3 * 3/4, silu(-ln 3) = -ln3 / 4
    l3 = math.log(3.0)
    Y = np.array([[0.0, l3, 5.0, 7.0],
                  [-l3, 2.0, -2.0, 0.5]])
    H64, Hbf = oracle_mod.swiglu(Y)
    want = np.array([[0.0, l3 * 0.75 * 7.0],
                     [(-l3 * 0.25) * -2.0, 2.0 / (1.0 + math.exp(-2.0)) * 0.5]])
    np.testing.assert_allclose(H64, want, rtol=1e-15, atol=0)
    assert [oracle_mod.bf16_to_f32(int(b)) for b in Hbf.reshape(-1)] == \
           [oracle_mod.bf16_to_f32(oracle_mod.f64_to_bf16_rne(float(v))) for v in want.reshape(-1)]


def test_swiglu_against_library_and_identities(oracle_mod):
    rng = np.random.default_rng(3)
    Y = rng.normal(size=(37, 64)) * 4.0
    H64, _ = oracle_mod.swiglu(Y)
    g, u = torch.from_numpy(Y[:, :32]), torch.from_numpy(Y[:, 32:])
    np.testing.assert_allclose(H64, (torch.nn.functional.silu(g) * u).numpy(), rtol=1e-13, atol=1e-300)
    # silu(g) - silu(-g) = g: with up = 1 the two halves of a +/- pair differ by g
    G = rng.normal(size=(5, 8)) * 3
    ones = np.ones_like(G)
    Hp, _ = oracle_mod.swiglu(np.concatenate([G, ones], axis=1))
    Hm, _ = oracle_mod.swiglu(np.concatenate([-G, ones], axis=1))
    np.testing.assert_allclose(Hp - Hm, G, rtol=1e-13, atol=1e-15)
    # large gates pass the up value through scaled by the gate; large negative gates close
    big, _ = oracle_mod.swiglu(np.array([[40.0, -40.0, 3.0, 3.0]]))
    assert abs(big[0, 0] - 120.0) < 1e-12 and abs(big[0, 1]) < 1e-14


def test_combine_hand_and_library(oracle_mod):
    T, k, N = 3, 2, 4
    vals = np.arange(T * k * N, dtype=np.float64).reshape(T * k, N) - 7.0   # small integers: exact in bf16
    bits = np.array([[oracle_mod.f64_to_bf16_rne(float(v)) for v in row] for row in vals], dtype=np.uint16)
    w = np.array([[0.5, 0.25], [1.0, -2.0], [0.0, 3.0]], dtype=np.float32)
    out64, outbf = oracle_mod.combine(bits, w, T, k)
    want = np.einsum("tj,tjn->tn", w.astype(np.float64), vals.reshape(T, k, N))
    np.testing.assert_array_equal(out64, want)        # all terms exact in fp64
    # token 1 by hand: rows 2 and 3 hold [1, 2, 3, 4] and [5, 6, 7, 8]; 1 * row2 - 2 * row3
    assert out64[1].tolist() == [-9.0, -10.0, -11.0, -12.0]
    # token 0: rows [-7, -6, -5, -4] and [-3, -2, -1, 0]; 0.5 * row0 + 0.25 * row1
    assert out64[0].tolist() == [-4.25, -3.5, -2.75, -2.0]
    plain, _ = oracle_mod.combine(bits, None, T, k)
    np.testing.assert_array_equal(plain, vals.reshape(T, k, N).sum(axis=1))
    np.testing.assert_array_equal(H.bf16_bits_to_f64(outbf), want)  # small integers and halves: exact in bf16 too


def test_combine_random_against_einsum(oracle_mod):
    rng = np.random.default_rng(11)
    T, k, N = 17, 6, 40
    y = torch.from_numpy(rng.normal(size=(T * k, N))).to(torch.bfloat16)
    bits = y.view(torch.int16).numpy().view(np.uint16)
    w = rng.random(size=(T, k)).astype(np.float32)
    out64, outbf = oracle_mod.combine(bits, w, T, k)
    want = np.einsum("tj,tjn->tn", w.astype(np.float64), y.double().numpy().reshape(T, k, N))
    np.testing.assert_allclose(out64, want, rtol=1e-14, atol=1e-14)
    got_bf = H.bf16_bits_to_f64(outbf)
    assert np.all(np.abs(got_bf - out64) <= 2.0 ** -8 * np.abs(out64))


# ------------------------------------------------------------------ heterogeneous batch (Sec. 3.2, Alg. 3)
def test_heterogeneous_batch_mapping_against_nested_loops(oracle_mod):
    """GEMM tasks plus one reduction task in one batch: Alg. 1 + 2 over the extended list of tile counts must give, for
    every block, what plain nested loops over (task, tile) give -- the prior-art full table of Sec. 2.1 with one more
    task at its end -- and the GEMM part must be the GEMM map's own decode, untouched by the extra task."""
    rng = np.random.default_rng(77)
    for (T, E, k, N, red) in ((300, 8, 2, 512, 5), (64, 70, 3, 256, 1), (10, 4, 1, 256, 0), (0, 4, 2, 256, 3)):
        ids = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32) if T else np.zeros((0, k), np.int32)
        tm = oracle_mod.build_task_map(ids, T, k, E, 64, 128, N)
        got = oracle_mod.heterogeneous_batch_table(tm, red)
        want = []
        nt = -(-N // 128)
        for e in range(E):                      # GEMM tasks in ascending expert order, empty ones have no tiles
            for l in range(-(-int(tm.counts[e]) // 64) * nt):
                want.append((0, e, l))
        for l in range(red):                    # then the reduction task
            want.append((1, -1, l))
        assert got.tolist() == [list(w) for w in want]
        assert len(got) == tm.total_tiles + red
        for B in range(tm.total_tiles):         # the GEMM blocks decode as without the extra task
            e, m_tile, n_tile, _ = oracle_mod.decode_block(tm, B)
            mt = -(-int(tm.counts[e]) // 64)
            assert got[B].tolist() == [0, e, n_tile * mt + m_tile]


def test_reduce_task_tiles_closed_form(oracle_mod):
    assert oracle_mod.reduce_task_tiles(4096, 4096) == 4096 * 512 // 4096
    assert oracle_mod.reduce_task_tiles(1, 8) == 1
    assert oracle_mod.reduce_task_tiles(0, 4096) == 0
    assert oracle_mod.reduce_task_tiles(33, 1024) == -(-33 * 128 // 4096)
