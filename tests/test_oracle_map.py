"""CPU pins of the oracle's task map (Alg. 1, 2, 4; Sec. 4.1, 4.3; Sec. 5 scenarios).

Each test checks the oracle against something other than itself: hand-worked
fixtures, a brute-force nested-loop table, invariants that any correct map
satisfies, or the closed-form expert loads of the paper's scenarios.
"""
import json
import os

import numpy as np
import pytest
import torch

from paper_2501_16103_amd import workloads as wk

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


def test_alg1_alg2_hand_example(oracle_mod):
    g = _gold("alg2_prefix_example.json")
    prefix = oracle_mod.tile_prefix(g["nu"])
    assert prefix.tolist() == g["tile_prefix"]
    for B, h, l in g["blocks"]:
        assert oracle_mod.mapping(prefix, B) == (h, l)


def test_alg4_empty_expert_hand_example(oracle_mod):
    g = _gold("empty_expert_map.json")
    tm = oracle_mod.build_task_map(g["topk_ids"], g["T"], g["k"], g["E"], g["tile_m"], g["tile_n"], g["N"])
    assert tm.counts.tolist() == g["counts"]
    assert tm.offsets.tolist() == g["offsets"]
    assert tm.sorted_rows.tolist() == g["sorted_rows"]
    assert tm.sigma.tolist() == g["sigma"] and tm.M == g["M"]
    assert tm.tile_prefix.tolist() == g["tile_prefix"] and tm.total_tiles == g["total_tiles"]
    assert oracle_mod.decode_all(tm).tolist() == g["table"]


def test_two_expert_map_hand_example(oracle_mod):
    g = _gold("two_expert_values.json")
    tm = oracle_mod.build_task_map(g["topk_ids"], g["T"], g["k"], g["E"], g["tile_m"], g["tile_n"], g["N"])
    assert tm.counts.tolist() == g["counts"]
    assert tm.offsets.tolist() == g["offsets"]
    assert tm.sorted_rows.tolist() == g["sorted_rows"]
    assert tm.sigma.tolist() == g["sigma"]
    assert tm.tile_prefix.tolist() == g["tile_prefix"]
    assert oracle_mod.decode_all(tm).tolist() == g["table"]


def _random_ids(rng, T, k, E, skew):
    ids = np.zeros((T, k), dtype=np.int32)
    p = np.arange(1, E + 1, dtype=np.float64) ** (-skew)
    p /= p.sum()
    for t in range(T):
        ids[t] = rng.choice(E, size=k, replace=False, p=p)
    return ids


CASES = [
    # T, k, E, tile_m, tile_n, N, skew
    (1, 1, 1, 16, 64, 64, 0.0),
    (7, 2, 5, 16, 128, 300, 0.0),
    (64, 2, 8, 32, 128, 512, 0.0),
    (33, 3, 70, 16, 64, 200, 2.0),       # E > 64: several voting rounds, many empty experts
    (200, 8, 256, 16, 128, 256, 1.0),
    (129, 2, 8, 128, 256, 512, 3.0),     # counts around the tile size
    (50, 6, 64, 64, 128, 2816, 0.5),
]


@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,skew", CASES)
def test_decode_equals_bruteforce_table(oracle_mod, T, k, E, tile_m, tile_n, N, skew):
    """Alg. 2 + Alg. 4 decode of every block == the prior-art full table by nested loops."""
    rng = np.random.default_rng(1234 + T + E)
    ids = _random_ids(rng, T, k, E, skew)
    tm = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N)
    table = oracle_mod.full_table(tm.counts, tile_m, tile_n, N)
    assert table.shape[0] == tm.total_tiles
    np.testing.assert_array_equal(oracle_mod.decode_all(tm), table)


@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,skew", CASES)
def test_map_invariants(oracle_mod, T, k, E, tile_m, tile_n, N, skew):
    rng = np.random.default_rng(99 + T * 7 + E)
    ids = _random_ids(rng, T, k, E, skew)
    tm = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N)
    R = T * k
    flat = ids.reshape(-1)
    # counts against an independent library histogram
    np.testing.assert_array_equal(tm.counts, np.bincount(flat, minlength=E))
    assert tm.counts.sum() == R and tm.offsets[0] == 0 and tm.offsets[E] == R
    np.testing.assert_array_equal(np.diff(tm.offsets), tm.counts)
    # token index arrays: a permutation, right expert, ascending inside a segment
    assert sorted(tm.sorted_rows.tolist()) == list(range(R))
    # equals a library stable sort of the rows by expert
    np.testing.assert_array_equal(tm.sorted_rows, np.argsort(flat, kind="stable"))
    for e in range(E):
        seg = tm.sorted_rows[tm.offsets[e]:tm.offsets[e + 1]]
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)
    # sigma: ascending, exactly the non-empty experts
    assert tm.sigma.tolist() == [e for e in range(E) if tm.counts[e] > 0]
    assert tm.M == len(tm.sigma)
    # prefix: strictly increasing, closed form of the last entry
    nt = -(-N // tile_n)
    mt = -(-tm.counts // tile_m)
    assert np.all(np.diff(np.concatenate([[0], tm.tile_prefix])) > 0)
    assert tm.total_tiles == int(mt.sum()) * nt
    np.testing.assert_array_equal(tm.tile_prefix, np.cumsum(mt[tm.sigma] * nt))
    # decode is a bijection onto {(e, m<mt_e, n<nt)} and rows add up per n-tile
    table = oracle_mod.decode_all(tm)
    seen = set(map(tuple, table[:, :3].tolist()))
    assert len(seen) == tm.total_tiles
    assert seen == {(e, m, n) for e in range(E) for m in range(mt[e]) for n in range(nt)}
    for n in range(nt):
        assert table[table[:, 2] == n][:, 3].sum() == R  # every routed row once per n-tile


def test_decode_with_zero_tile_tasks_matches_compact(oracle_mod):
    """Counting prefix entries <= B over the full-E prefix (zeros for empty experts)
    picks the same expert as the compact prefix followed by sigma."""
    rng = np.random.default_rng(5)
    ids = _random_ids(rng, 40, 2, 24, 2.5)
    tm = oracle_mod.build_task_map(ids, 40, 2, 24, 16, 64, 128)
    assert tm.M < 24  # some experts empty
    nt = 2
    nu_full = (-(-tm.counts // 16)) * nt
    full_prefix = oracle_mod.tile_prefix(nu_full)
    for B in range(tm.total_tiles):
        h_full, l_full = oracle_mod.mapping(full_prefix, B)
        h, l = oracle_mod.mapping(tm.tile_prefix, B)
        assert int(tm.sigma[h]) == h_full and l == l_full


def test_paper_scenarios_closed_form_counts(oracle_mod):
    """Sec. 5: balanced = T*k/E rows each; best = k experts with T rows; worst = E-k
    experts with exactly one row, the k busy experts share the rest."""
    T, E, k = 4096, 64, 8
    for scen in ("balanced", "best", "worst"):
        wl = wk.paper_eval(scen, T)
        ids = wk.make_routing(wl).numpy()
        assert all(len(set(row)) == k for row in ids.tolist())  # distinct experts per token
        tm = oracle_mod.build_task_map(ids, T, k, E, 256, 256, wl.N)
        c = tm.counts
        if scen == "balanced":
            assert np.all(c == T * k // E) and tm.M == E
            assert tm.total_tiles == E * 2 * 10
        elif scen == "best":
            assert np.all(c[:k] == T) and np.all(c[k:] == 0) and tm.M == k
            assert tm.total_tiles == k * 16 * 10
        else:
            assert np.all(c[k:] == 1) and c[:k].sum() == T * k - (E - k) and tm.M == E
            assert np.all(c[: k - 1] == T) and c[k - 1] == T - (E - k)


def test_T0_and_bad_id(oracle_mod):
    tm = oracle_mod.build_task_map(np.zeros((0, 2), np.int32), 0, 2, 8, 16, 64, 128)
    assert tm.total_tiles == 0 and tm.M == 0 and tm.counts.sum() == 0
    with pytest.raises(ValueError):
        oracle_mod.build_task_map([[0, 8]], 1, 2, 8, 16, 64, 128)
    with pytest.raises(ValueError):
        oracle_mod.build_task_map([[-1, 2]], 1, 2, 8, 16, 64, 128)


def test_workload_routing_recipes():
    for wl in (wk.tiny(), wk.mixtral_up(256), wk.mixtral_down_zipf(256), wk.fine_grained(128), wk.decode_fp8(32)):
        ids = wk.make_routing(wl)
        assert ids.dtype == torch.int32 and tuple(ids.shape) == (wl.T, wl.k)
        assert int(ids.min()) >= 0 and int(ids.max()) < wl.E
        s = torch.sort(ids, dim=1).values
        assert bool((s[:, 1:] != s[:, :-1]).all())  # without replacement
        assert torch.equal(ids, wk.make_routing(wl))  # seeded
    # zipf is skewed, gauss_topk roughly balanced
    z = np.bincount(wk.make_routing(wk.mixtral_down_zipf(4096)).numpy().ravel(), minlength=8)
    assert z.max() > 3 * z.min()
    b = np.bincount(wk.make_routing(wk.mixtral_up(4096)).numpy().ravel(), minlength=8)
    assert b.max() < 1.2 * b.min()


# ------------------------------------------------------------------ expert ordering (Sec. 4.2)
def test_spread_order_hand_example(oracle_mod):
    g = _gold("spread_order_example.json")
    ids = np.concatenate([np.full(c, e, np.int32) for e, c in enumerate(g["counts"])]).reshape(-1, 1)
    T = len(ids)
    tm = oracle_mod.build_task_map(ids, T, 1, g["E"], g["tile_m"], g["tile_n"], g["N"], order=1)
    assert tm.counts.tolist() == g["counts"]
    assert tm.sigma.tolist() == g["sigma"]
    assert tm.tile_prefix.tolist() == g["tile_prefix"]
    # the fixture is self-consistent with its own stated rule
    rev3 = lambda r: int(f"{r:03b}"[::-1], 2)
    assert [rev3(r) for r in g["rank"]] == g["key_bitrev3"]
    assert [g["key_bitrev3"].index(kk) for kk in range(8)] == g["sigma"]


@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,skew", CASES)
def test_spread_order_properties(oracle_mod, T, k, E, tile_m, tile_n, N, skew):
    rng = np.random.default_rng(4321 + T + E)
    ids = _random_ids(rng, T, k, E, skew)
    asc = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N, order=0)
    spr = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N, order=1)
    # only sigma and the prefix may differ
    np.testing.assert_array_equal(asc.counts, spr.counts)
    np.testing.assert_array_equal(asc.offsets, spr.offsets)
    np.testing.assert_array_equal(asc.sorted_rows, spr.sorted_rows)
    assert sorted(spr.sigma.tolist()) == asc.sigma.tolist() and spr.total_tiles == asc.total_tiles
    nt = -(-N // tile_n)
    tiles = (-(-spr.counts // tile_m)) * nt
    np.testing.assert_array_equal(spr.tile_prefix, np.cumsum(tiles[spr.sigma]))
    # the busiest expert comes first; the second busiest sits at the half point of the key space
    M = spr.M
    by_load = sorted(range(E), key=lambda e: (-tiles[e], e))
    by_load = [e for e in by_load if spr.counts[e] > 0]
    assert spr.sigma[0] == by_load[0]
    if M >= 2:
        P = 1 << (M - 1).bit_length()
        n_before_half = sum(1 for r in range(M) if int(f"{r:0{max(P.bit_length() - 1, 1)}b}"[::-1], 2) < P // 2) if P > 1 else 0
        assert spr.sigma[n_before_half] == by_load[1]
    # decode of every block == nested-loop table visiting experts in sigma order
    np.testing.assert_array_equal(oracle_mod.decode_all(spr), oracle_mod.full_table(spr.counts, tile_m, tile_n, N, sigma=spr.sigma))


def test_spread_order_on_paper_worst_case(oracle_mod):
    """Sec. 5 worst case: the k busy experts end up evenly spaced among the 56 one-token experts."""
    wl = wk.paper_eval("worst")
    ids = wk.make_routing(wl).numpy()
    tm = oracle_mod.build_task_map(ids, wl.T, wl.k, wl.E, 256, 256, wl.N, order=1)
    pos = sorted(int(np.where(tm.sigma == e)[0][0]) for e in range(wl.k))
    assert pos == [0, 8, 16, 24, 32, 40, 48, 56]


# ------------------------------------------------------------------ two tiling strategies (Alg. 3)
def test_two_tilings_hand_example(oracle_mod):
    g = _gold("two_tilings_example.json")
    ids = np.concatenate([np.full(c, e, np.int32) for e, c in enumerate(g["counts"])]).reshape(-1, 1)
    tm = oracle_mod.build_task_map(ids, len(ids), 1, g["E"], g["tile_m"], g["tile_n"], g["N"],
                                   tile_m_small=g["tile_m_small"], small_max_rows=g["small_max_rows"])
    assert [tm.expert_tile_m(e) for e in range(g["E"])] == g["expert_tile_m"]
    assert tm.sigma.tolist() == g["sigma"]
    assert tm.tile_prefix.tolist() == g["tile_prefix"]
    assert oracle_mod.decode_all(tm).tolist() == g["table"]
    assert oracle_mod.full_table(tm.counts, g["tile_m"], g["tile_n"], g["N"], tile_m_small=g["tile_m_small"],
                                 small_max_rows=g["small_max_rows"]).tolist() == g["table"]


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,skew", CASES)
def test_two_tilings_properties(oracle_mod, T, k, E, tile_m, tile_n, N, skew, order):
    rng = np.random.default_rng(777 + T + E)
    ids = _random_ids(rng, T, k, E, skew)
    small, thr = 16, 24
    tm = oracle_mod.build_task_map(ids, T, k, E, max(tile_m, 32), tile_n, N, order=order, tile_m_small=small, small_max_rows=thr)
    big = max(tile_m, 32)
    nt = -(-N // tile_n)
    etm = np.array([small if 0 < c <= thr else big for c in tm.counts])
    mt = np.where(tm.counts > 0, -(-tm.counts // etm), 0)
    np.testing.assert_array_equal(tm.tile_prefix, np.cumsum(mt[tm.sigma] * nt))
    table = oracle_mod.decode_all(tm)
    np.testing.assert_array_equal(table, oracle_mod.full_table(tm.counts, big, tile_n, N, sigma=tm.sigma,
                                                                tile_m_small=small, small_max_rows=thr))
    # every routed row is covered exactly once per n-tile, with the tile height of its expert's strategy
    for n in range(nt):
        sub = table[table[:, 2] == n]
        assert sub[:, 3].sum() == T * k
    for e, m_tile, n_tile, rows in table.tolist():
        assert rows == min(etm[e], tm.counts[e] - m_tile * etm[e]) and rows >= 1


# ------------------------------------------------------------------ slack rows in the last m-tile
def test_slack_tiling_hand_example(oracle_mod):
    g = _gold("slack_tiling_example.json")
    ids = np.concatenate([np.full(c, e, np.int32) for e, c in enumerate(g["counts"])]).reshape(-1, 1)
    tm = oracle_mod.build_task_map(ids, len(ids), 1, g["E"], g["tile_m"], g["tile_n"], g["N"], tile_m_slack=g["tile_m_slack"])
    assert tm.sigma.tolist() == g["sigma"]
    assert tm.tile_prefix.tolist() == g["tile_prefix"]
    assert oracle_mod.decode_all(tm).tolist() == g["table"]
    assert oracle_mod.full_table(tm.counts, g["tile_m"], g["tile_n"], g["N"], tile_m_slack=g["tile_m_slack"]).tolist() == g["table"]


@pytest.mark.parametrize("tile_m,slack", [(4, 1), (4, 3), (16, 4), (32, 8), (256, 64)])
def test_slack_tiling_closed_form_and_shape(oracle_mod, tile_m, slack):
    """For every row count: the number of tiles is max(1, ceil((c - slack) / tile_m)); all tiles but the last are
    full; the last holds more than `slack` rows unless it is the only one; slack 0 is the plain ceil."""
    for c in list(range(1, 6 * tile_m + 3)):
        counts = np.array([c], np.int32)
        t = oracle_mod.full_table(counts, tile_m, 8, 8, tile_m_slack=slack)
        mt = len(t)
        assert mt == max(1, -(-(c - slack) // tile_m))
        assert t[:, 1].tolist() == list(range(mt))
        assert (t[:-1, 3] == tile_m).all() and t[:, 3].sum() == c
        assert 1 <= t[-1, 3] <= tile_m + slack
        assert mt == 1 or t[-1, 3] > slack
        t0 = oracle_mod.full_table(counts, tile_m, 8, 8, tile_m_slack=0)
        assert len(t0) == -(-c // tile_m) and len(t0) - mt in (0, 1)


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,skew", CASES)
def test_slack_tiling_properties(oracle_mod, T, k, E, tile_m, tile_n, N, skew, order):
    rng = np.random.default_rng(4242 + T + E)
    ids = _random_ids(rng, T, k, E, skew)
    slack = max(1, tile_m // 4)
    tm = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N, order=order, tile_m_slack=slack)
    nt = -(-N // tile_n)
    mt = np.where(tm.counts > 0, np.maximum(1, -(-(tm.counts - slack) // tile_m)), 0)
    np.testing.assert_array_equal(tm.tile_prefix, np.cumsum(mt[tm.sigma] * nt))
    table = oracle_mod.decode_all(tm)
    np.testing.assert_array_equal(table, oracle_mod.full_table(tm.counts, tile_m, tile_n, N, sigma=tm.sigma, tile_m_slack=slack))
    # every routed row is covered exactly once per n-tile: tile m of an expert starts at row m * tile_m of its segment
    for n in range(nt):
        sub = table[table[:, 2] == n]
        covered = np.zeros(T * k, dtype=np.int32)
        for e, m_tile, _, rows in sub.tolist():
            lo = tm.offsets[e] + m_tile * tile_m
            covered[tm.sorted_rows[lo: lo + rows]] += 1
            assert lo + rows <= tm.offsets[e + 1]
        assert (covered == 1).all()
    # a small second strategy keeps its own plain tiling
    tm2 = oracle_mod.build_task_map(ids, T, k, E, max(tile_m, 32), tile_n, N, order=order, tile_m_small=16, small_max_rows=24,
                                    tile_m_slack=8)
    t2 = oracle_mod.decode_all(tm2)
    np.testing.assert_array_equal(t2, oracle_mod.full_table(tm2.counts, max(tile_m, 32), tile_n, N, sigma=tm2.sigma, tile_m_small=16,
                                                             small_max_rows=24, tile_m_slack=8))
    for e, m_tile, _, rows in t2.tolist():
        if tm2.counts[e] <= 24:
            assert rows == min(16, tm2.counts[e] - 16 * m_tile)


# ------------------------------------------------------------------ two-level TilePrefix (Sec. 3.1)
@pytest.mark.parametrize("n,group", [(1, 64), (5, 2), (64, 64), (65, 64), (130, 64), (200, 8), (1000, 64)])
def test_two_level_mapping_equals_brute_force(oracle_mod, n, group):
    """Against the definition itself: block B belongs to the task whose half-open tile range contains it."""
    rng = np.random.default_rng(n * 131 + group)
    nu = rng.integers(0, 5, size=n)          # zero-tile tasks included: equal neighbours in the prefix
    nu[rng.integers(0, n)] += 1              # at least one tile
    prefix = np.cumsum(nu).astype(np.int32)
    owner = np.repeat(np.arange(n), nu)      # brute force: the task of every block, written out
    first = np.concatenate([[0], prefix[:-1]])
    for B in range(int(prefix[-1])):
        h, l = oracle_mod.mapping_two_level(prefix, group, B)
        assert h == owner[B] and l == B - first[h]
        assert (h, l) == oracle_mod.mapping(prefix, B)


# ------------------------------------------------------------------ heavy-first order (order 2, Sec. 4.2)
def test_heavy_first_order_hand_example(oracle_mod):
    g = _gold("heavy_first_order_example.json")
    ids = np.concatenate([np.full(c, e, np.int32) for e, c in enumerate(g["counts"])]).reshape(-1, 1)
    tm = oracle_mod.build_task_map(ids, len(ids), 1, g["E"], g["tile_m"], g["tile_n"], g["N"], order=2)
    assert tm.sigma.tolist() == g["sigma"]
    assert tm.tile_prefix.tolist() == g["tile_prefix"]
    assert tm.heavy_tiles == g["heavy_tiles"]


@pytest.mark.parametrize("T,k,E,tile_m,tile_n,N,skew", CASES)
def test_heavy_first_order_properties(oracle_mod, T, k, E, tile_m, tile_n, N, skew):
    rng = np.random.default_rng(31337 + T + E)
    ids = _random_ids(rng, T, k, E, skew)
    tm = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N, order=2)
    base = oracle_mod.build_task_map(ids, T, k, E, tile_m, tile_n, N, order=0)
    # same experts, same per-expert data; only sigma and the prefix move
    assert sorted(tm.sigma.tolist()) == base.sigma.tolist() and tm.total_tiles == base.total_tiles
    np.testing.assert_array_equal(tm.counts, base.counts)
    np.testing.assert_array_equal(tm.sorted_rows, base.sorted_rows)
    nt = -(-N // tile_n)
    c = tm.counts[tm.sigma]
    tiles = -(-c // tile_m) * nt
    light = 4 * c <= tile_m
    # heavy block first, light block last, the boundary is heavy_tiles
    nh = int((~light).sum())
    assert not light[:nh].any() and light[nh:].all()
    assert tm.heavy_tiles == int(tiles[:nh].sum())
    assert all(tiles[i] > tiles[i + 1] or (tiles[i] == tiles[i + 1] and tm.sigma[i] < tm.sigma[i + 1]) for i in range(nh - 1))
    assert all(tm.sigma[i] < tm.sigma[i + 1] for i in range(nh, tm.M - 1))
    np.testing.assert_array_equal(tm.tile_prefix, np.cumsum(tiles))
    # the decode still equals the nested-loop table in that expert order
    np.testing.assert_array_equal(oracle_mod.decode_all(tm), oracle_mod.full_table(tm.counts, tile_m, tile_n, N, sigma=tm.sigma))
