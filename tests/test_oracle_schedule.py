"""Pins for the scheduler oracle: invariants the paper and arithmetic fix, hand-derived spot
values, a second transcription of Algorithm 1, and execution of schedules on tiny GEMMs."""
import os
from collections import Counter

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import schedule as S
from oracle import simulate
from oracle import gemm as G
from paper_2408_11417_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

shape_st = st.tuples(st.integers(1, 300), st.integers(1, 300), st.integers(1, 400))
blk_st = st.tuples(st.sampled_from([16, 32, 64, 128]), st.sampled_from([16, 32, 64, 128]),
                   st.sampled_from([8, 16, 32, 64]))
grid_st = st.sampled_from([1, 2, 3, 4, 7, 8, 16, 24, 64, 104, 256])
policy_st = st.integers(0, 7)


def test_spot_values_from_golden_file():
    n = 0
    for line in open(os.path.join(GOLDEN, "schedule_spot_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        left, right = line.split("|")
        M, N, K, bm, bn, bk, g, pol = left.split()
        want = [int(v) for v in right.split()]
        p = S.plan(int(M), int(N), int(K), S.POLICY_NAMES.index(pol), int(bm), int(bn), int(bk), int(g))
        h = p.header
        got = [h["tiles"], h["iters_per_tile"], h["total_iters"], h["sk_tiles"], h["sk_iters"],
               h["iters_per_wg"], h["dp_tiles"]]
        assert got == want, line
        n += 1
    assert n == 15


def test_last_workgroup_of_all_sk_on_wave_quantisation_case():
    # 63360 iterations over 256 workgroups of 248: the last one is short (hand value 120)
    p = S.plan(3840, 4224, 4096, S.POLICY_ALL_SK, 256, 128, 32, 256)
    r = p.ranges[255]
    assert r.sk_iter_end - r.sk_iter_begin == 120
    assert all(p.ranges[x].sk_iter_end - p.ranges[x].sk_iter_begin == 248 for x in range(255))


@settings(max_examples=300, deadline=None)
@given(shape_st, blk_st, grid_st, policy_st)
def test_every_mac_iteration_covered_exactly_once(shape, blk, g, policy):
    p = S.plan(*shape, policy, *blk, g)
    h = p.header
    seen = Counter()
    for s in p.segments:
        assert 0 <= s.k_begin < s.k_end <= h["iters_per_tile"]
        assert 0 <= s.tile < h["tiles"] and 0 <= s.wg < g
        for k in range(s.k_begin, s.k_end):
            seen[(s.tile, k)] += 1
    assert len(seen) == h["total_iters"]
    assert set(seen.values()) <= {1}


@settings(max_examples=300, deadline=None)
@given(shape_st, blk_st, grid_st, policy_st)
def test_ranges_and_roles(shape, blk, g, policy):
    p = S.plan(*shape, policy, *blk, g)
    h = p.header
    ipt, ipw = h["iters_per_tile"], h["iters_per_wg"]
    # Stream-K ranges: contiguous, ordered, disjoint, union = [0, sk_iters), none longer than ipw
    pos = 0
    for x, r in enumerate(p.ranges):
        assert r.sk_iter_begin == pos and r.sk_iter_end >= r.sk_iter_begin
        assert r.sk_iter_end - r.sk_iter_begin <= ipw
        pos = r.sk_iter_end
    assert pos == h["sk_iters"] == h["sk_tiles"] * ipt
    # hybrids leave whole waves to the data-parallel part
    if 0 < h["sk_tiles"] < h["tiles"]:
        assert h["dp_tiles"] % g == 0
    per_tile_first = Counter()
    contrib_by_tile = {}
    by_wg = {}
    for s in p.segments:
        by_wg.setdefault(s.wg, []).append(s)
        if s.role in (S.ROLE_FULL, S.ROLE_OWNER):
            per_tile_first[s.tile] += 1
            assert s.k_begin == 0
            assert (s.k_end == ipt) == (s.role == S.ROLE_FULL)
        else:
            assert s.k_begin > 0
            contrib_by_tile.setdefault(s.tile, []).append(s)
    assert all(per_tile_first[t] == 1 for t in range(h["tiles"]))
    for wg, segs in by_wg.items():
        contribs = [i for i, s in enumerate(segs) if s.role == S.ROLE_CONTRIB]
        assert contribs in ([], [0])               # at most one partial per workgroup, and it comes first
        sk = [s for s in segs if s.tile < h["sk_tiles"]]
        dp = [s for s in segs if s.tile >= h["sk_tiles"]]
        assert segs == sk + dp                      # Stream-K work first, then data-parallel tiles
        assert [s.tile for s in dp] == [h["sk_tiles"] + wg + j * g for j in range(len(dp))]
        assert all(s.role == S.ROLE_FULL for s in dp)
    for s in p.segments:
        if s.role == S.ROLE_OWNER:
            cs = S.contributors(p, s)
            got = sorted(c.wg for c in contrib_by_tile[s.tile])
            assert cs == got
            k = s.k_end                             # contributors tile [k_end, ipt) with no gap, ascending wg
            for c in sorted(contrib_by_tile[s.tile], key=lambda c: c.wg):
                assert c.k_begin == k
                k = c.k_end
            assert k == ipt
        if s.role == S.ROLE_FULL:
            assert s.tile not in contrib_by_tile


@settings(max_examples=200, deadline=None)
@given(shape_st, blk_st, grid_st)
def test_pure_data_parallel_is_one_tile_per_workgroup_per_wave(shape, blk, g):
    p = S.plan(*shape, S.POLICY_DP, *blk, g)
    h = p.header
    assert h["sk_tiles"] == 0 and h["iters_per_wg"] == 0
    assert all(s.role == S.ROLE_FULL for s in p.segments)
    owner = {s.tile: s.wg for s in p.segments}
    assert owner == {t: t % g for t in range(h["tiles"])}
    if h["tiles"] <= g:
        assert Counter(s.wg for s in p.segments) == Counter(range(h["tiles"]))
    assert S.makespan_iters(p) == S.cdiv(h["tiles"], g) * h["iters_per_tile"]


def _algorithm1_by_iteration(M, N, K, bm, bn, bk, g):
    """Second, independent reading of Algorithm 1: label every global iteration with the
    workgroup that the equal split gives it and with its tile, then group runs."""
    ipt = -(-K // bk)
    total = -(-M // bm) * -(-N // bn) * ipt
    ipw = -(-total // g)
    out = []
    for i in range(total):
        wg, tile, k = i // ipw, i // ipt, i % ipt
        if out and out[-1][0] == wg and out[-1][1] == tile and out[-1][3] == k:
            out[-1][3] = k + 1
        else:
            out.append([wg, tile, k, k + 1])
    return [tuple(s) for s in out]


@settings(max_examples=200, deadline=None)
@given(shape_st, blk_st, grid_st)
def test_all_stream_k_equals_second_transcription_of_algorithm_1(shape, blk, g):
    p = S.plan(*shape, S.POLICY_ALL_SK, *blk, g)
    assert p.header["dp_tiles"] == 0
    got = [(s.wg, s.tile, s.k_begin, s.k_end) for s in p.segments]
    assert got == _algorithm1_by_iteration(*shape, *blk, g)


@settings(max_examples=200, deadline=None)
@given(shape_st, blk_st, grid_st)
def test_policy_family_structure(shape, blk, g):
    plans = [S.plan(*shape, pol, *blk, g) for pol in range(8)]
    T = plans[0].header["tiles"]
    ipt = plans[0].header["iters_per_tile"]
    order = [0, 1, 2, 3, 4, 5, 7, 6]                # b = 0..6, then all-Stream-K
    sk = [plans[i].header["sk_tiles"] for i in order]
    assert sk == sorted(sk) and sk[-1] == T
    rem = T % g
    assert plans[1].header["sk_tiles"] == min(T, rem)
    if rem == 0:
        assert plans[1].segments == plans[0].segments          # nothing left over: one batch == DP
        for b in range(2, 6):                                   # whole waves: every segment is a full tile
            assert all(s.role == S.ROLE_FULL for s in plans[b].segments)
    for b in range(1, 6):
        if rem + (b - 1) * g >= T:                              # batches cover everything == all-Stream-K
            assert plans[b].segments == plans[6].segments
    for p in plans:                                             # never worse than data-parallel waves
        h = p.header
        assert S.makespan_iters(p) == h["iters_per_wg"] + h["dp_waves"] * ipt   # workgroup 0 is busiest
        assert S.makespan_iters(p) <= S.cdiv(T, g) * ipt


@settings(max_examples=200, deadline=None)
@given(shape_st, blk_st, grid_st, policy_st)
def test_data_parallel_first_only_swaps_the_two_phases(shape, blk, g, policy):
    # Sec. 3.2's earlier hybrid: same ranges, same segments per workgroup, data-parallel tiles in front
    a = S.plan(*shape, policy, *blk, g)
    b = S.plan(*shape, policy, *blk, g, dp_first=True)
    assert b.header["dp_first"] and not a.header["dp_first"]
    assert {k: v for k, v in a.header.items() if k != "dp_first"} == {k: v for k, v in b.header.items() if k != "dp_first"}
    assert a.ranges == b.ranges
    assert sorted(a.segments) == sorted(b.segments)
    for x in range(g):
        sa = [s for s in a.segments if s.wg == x]
        sb = [s for s in b.segments if s.wg == x]
        n_dp = a.ranges[x].dp_tile_count
        n_sk = len(sa) - n_dp
        assert sb == sa[n_sk:] + sa[:n_sk]
        # under either order the data-parallel segments are whole tiles beyond the Stream-K region
        assert all(s.role == S.ROLE_FULL and s.tile >= a.header["sk_tiles"] for s in sb[:n_dp])


@settings(max_examples=300, deadline=None)
@given(shape_st, blk_st, grid_st, policy_st, st.booleans())
def test_k_aligned_order_keeps_the_work_and_moves_head_and_owner(shape, blk, g, policy, dp_first):
    # same iterations per workgroup as Algorithm 1; only the order inside a workgroup and the owner change
    a = S.plan(*shape, policy, *blk, g, dp_first=dp_first)
    b = S.plan(*shape, policy, *blk, g, dp_first=dp_first, k_aligned=True)
    ipt = a.header["iters_per_tile"]
    assert a.ranges == b.ranges
    strip = lambda segs: sorted(s[:4] for s in segs)                      # noqa: E731
    assert strip(a.segments) == strip(b.segments)
    pieces = {}
    for s in b.segments:
        pieces.setdefault(s.tile, []).append(s)
    for tile, ps in pieces.items():
        ps.sort(key=lambda s: s.k_begin)
        assert ps[0].k_begin == 0 and ps[-1].k_end == ipt
        assert all(x.k_end == y.k_begin for x, y in zip(ps, ps[1:]))     # the tile's k-range, cut without gaps
        if len(ps) == 1:
            assert ps[0].role == S.ROLE_FULL
            continue
        assert [s.role for s in ps] == [S.ROLE_CONTRIB] * (len(ps) - 1) + [S.ROLE_OWNER]   # the last piece owns
        assert S.contributors(b, ps[-1]) == [s.wg for s in ps[-2::-1]]   # the others, nearest first
        assert [s.wg for s in ps] == list(range(ps[0].wg, ps[0].wg + len(ps)))
    for x in range(g):
        sa = [s[:4] for s in a.segments if s.wg == x and s.tile < a.header["sk_tiles"]]
        sb = [s[:4] for s in b.segments if s.wg == x and s.tile < a.header["sk_tiles"]]
        if len(sa) > 1:
            whole = [s for s in sa if s[2] == 0 and s[3] == ipt]
            head = [sa[-1]] if sa[-1][3] < ipt else []                     # the range's last piece, from k = 0
            tail = [sa[0]] if sa[0][2] > 0 else []                         # the range's first piece, up to k = ipt
            assert sb == whole + head + tail and len(sb) == len(sa)
            # pace: every piece but the tail starts at k = 0 after a whole number of tiles
            t = 0
            for s in sb[:len(sb) - len(tail)]:
                assert s[2] == 0 and t % ipt == 0
                t += s[3] - s[2]
        else:
            assert sb == sa


def test_k_aligned_worked_example():
    # 5 tiles of 8 iterations over 4 workgroups, all Stream-K: 10 iterations each.
    #   wg0: tile0 [0,8) whole, tile1 [0,2)        -> whole tile first: tile0 FULL, tile1 [0,2) CONTRIB
    #   wg1: tile1 [2,8), tile2 [0,4)              -> head first: tile2 [0,4) CONTRIB, tile1 [2,8) OWNER
    #   wg2: tile2 [4,8), tile3 [0,6)              -> tile3 [0,6) CONTRIB, tile2 [4,8) OWNER
    #   wg3: tile3 [6,8), tile4 [0,8) whole        -> tile4 FULL, tile3 [6,8) OWNER
    p = S.plan(40, 8, 64, S.POLICY_ALL_SK, 8, 8, 8, 4, k_aligned=True)
    C, O, F = S.ROLE_CONTRIB, S.ROLE_OWNER, S.ROLE_FULL
    assert [tuple(s) for s in p.segments] == [
        (0, 0, 0, 8, F), (0, 1, 0, 2, C),
        (1, 2, 0, 4, C), (1, 1, 2, 8, O),
        (2, 3, 0, 6, C), (2, 2, 4, 8, O),
        (3, 4, 0, 8, F), (3, 3, 6, 8, O)]
    q = S.plan(40, 8, 64, S.POLICY_ALL_SK, 8, 8, 8, 4)
    assert [tuple(s) for s in q.segments] == [
        (0, 0, 0, 8, F), (0, 1, 0, 2, O),
        (1, 1, 2, 8, C), (1, 2, 0, 4, O),
        (2, 2, 4, 8, C), (2, 3, 0, 6, O),
        (3, 3, 6, 8, C), (3, 4, 0, 8, F)]


@settings(max_examples=200, deadline=None)
@given(st.integers(1, 70), st.integers(1, 70))
def test_tile_orders_are_bijections_onto_the_tile_grid(tiles_m, tiles_n):
    T = tiles_m * tiles_n
    rm = [S.tile_coords(t, tiles_m, tiles_n, S.ORDER_ROW_MAJOR) for t in range(T)]
    assert rm == [(m, n) for m in range(tiles_m) for n in range(tiles_n)]
    gr = [S.tile_coords(t, tiles_m, tiles_n, S.ORDER_GROUPED) for t in range(T)]
    assert sorted(gr) == rm
    # bands of 8 tile rows, walked column by column: hand construction
    want = []
    for band in range(0, tiles_m, 8):
        rows = min(8, tiles_m - band)
        want += [(band + r, n) for n in range(tiles_n) for r in range(rows)]
    assert gr == want


def test_grouped_order_makes_compact_blocks():
    # 32 x 32 tiles (8192^2 at 256 x 256): 32 consecutive indices = 8 rows x 4 columns
    blk = [S.tile_coords(t, 32, 32, S.ORDER_GROUPED) for t in range(64, 96)]
    assert {m for m, _ in blk} == set(range(8)) and {n for _, n in blk} == {8, 9, 10, 11}
    with pytest.raises(ValueError):
        S.tile_coords(0, 4, 4, 2)


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        S.plan(0, 16, 16, 0, 16, 16, 16, 4)
    with pytest.raises(ValueError):
        S.plan(16, 16, 16, 9, 16, 16, 16, 4)


# ---- executing schedules: integer-valued inputs make every schedule exact ------------------------

@pytest.mark.parametrize("policy", range(8))
def test_executed_schedule_equals_bruteforce_16cubed(policy):
    A, B = inputs.small_int_pair(16, 16, 16, inputs.F16, 11)
    a, b = G.decode_numpy(A, G.F16), G.decode_numpy(B, G.F16)
    ref = [[sum(a[i][k] * b[k][j] for k in range(16)) for j in range(16)] for i in range(16)]
    for k_aligned in (False, True):
        p = S.plan(16, 16, 16, policy, 8, 8, 4, 6, k_aligned=k_aligned)
        assert np.array_equal(simulate.run_plan(p, a, b).astype(np.float64), np.array(ref))


@settings(max_examples=60, deadline=None)
@given(st.tuples(st.integers(1, 70), st.integers(1, 70), st.integers(1, 90)),
       st.tuples(st.sampled_from([8, 16, 32]), st.sampled_from([8, 16, 32]), st.sampled_from([4, 8, 16])),
       st.sampled_from([1, 3, 4, 7, 16, 40]), policy_st, st.integers(0, 2 ** 31))
def test_executed_schedule_is_exact_on_integer_inputs(shape, blk, g, policy, seed):
    M, N, K = shape
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, seed)
    a, b = G.decode_numpy(A, G.BF16), G.decode_numpy(B, G.BF16)
    p = S.plan(M, N, K, policy, *blk, g, order=seed % 2, dp_first=seed % 3 == 0, k_aligned=seed % 5 < 2)
    assert np.array_equal(simulate.run_plan(p, a, b).astype(np.float64), a @ b)


def test_executed_schedule_within_fp32_tolerance_on_random_inputs():
    A, B = inputs.uniform_pair(96, 80, 200, inputs.F16, 5)
    ref = G.gemm_fp64(A, B, G.F16)
    a, b = G.decode_numpy(A, G.F16), G.decode_numpy(B, G.F16)
    for policy in range(8):
        p = S.plan(96, 80, 200, policy, 32, 32, 16, 7)
        assert G.rel_error(simulate.run_plan(p, a, b), ref) < 1e-4
