"""Policy selection on synthetic sweep records (CPU only): the Bloom properties the paper relies on
(Sec. 4.2: no false negatives) and the selection rules built on them."""
import random
import time

import paper_2408_11417_amd as sk
from paper_2408_11417_amd import selector
from oracle import bloom as Bm
from oracle import schedule as S


def _fake_records(n, seed):
    """Times that depend on the schedule the way the hardware roughly does: work per workgroup plus
    a fixed cost per split tile, with multiplicative noise."""
    rng = random.Random(seed)
    recs = []
    for _ in range(n):
        M, N, K = (16 * rng.randint(4, 512) for _ in range(3))
        tile = list(sk.sk_default_tile(M, N, K))
        times, sk_tiles = [], []
        for p in range(7):
            o = S.plan(M, N, K, p, *tile, 256)
            split = sum(1 for s in o.segments if s.role == S.ROLE_OWNER)
            times.append(int((S.makespan_iters(o) * 1000 + 4000 * (split > 0) + 20000) * (1 + 0.02 * rng.random())))
            sk_tiles.append(o.header["sk_tiles"])
        recs.append({"M": M, "N": N, "K": K, "tile": tile, "tiles": o.header["tiles"],
                     "iters_per_tile": o.header["iters_per_tile"], "time_ns": times, "sk_tiles": sk_tiles})
    return recs


def test_winner_mask_matches_oracle():
    rng = random.Random(1)
    for _ in range(500):
        t = [rng.randint(1000, 3000) for _ in range(7)]
        for tol in (0.0, 0.05, 0.2):
            assert selector.winner_mask(t, tol) == Bm.winner_mask(t, tol)


def test_no_false_negatives_and_selection_rules():
    recs = _fake_records(160, 3)
    for mode in ("exact", "shape"):
        for tol in (0.0, 0.2):
            rep = selector.evaluate(recs, 120, tol, mode)
            assert rep["false_negatives"] == 0
            assert 0.0 <= rep["held_pruning_rate"] < 1.0
            assert 0.0 < rep["held_mean_ratio"] <= 1.0
    sel = selector.PolicySelector(recs[:120], 0.2, "shape")
    for r in recs[:120]:
        p, mask, fb = sel.select(r, r["time_ns"])
        assert not fb and (mask >> p) & 1
        assert mask & selector.winner_mask(r["time_ns"], 0.2) == selector.winner_mask(r["time_ns"], 0.2)
        # a build-set size always gets a policy within the tolerance of its best
        assert r["time_ns"][p] <= min(r["time_ns"]) * 1.2 + 1
        ps, _, _ = sel.select(r)
        assert (mask >> ps) & 1
    sel.close()


def test_fallback_follows_the_cost_model():
    # whole waves of tiles: nothing to gain from splitting -> data-parallel
    assert selector.fallback_policy(4096, 4096, 4096, (256, 256, 64)) == sk.SK_POLICY_DP
    # four tiles with 128 iterations each on 256 workgroups -> split them
    assert selector.fallback_policy(64, 512, 8192, (32, 128, 64)) == sk.SK_POLICY_SK1_DP
    # 265 tiles of 11 iterations: splitting 9 leftover tiles 28 ways costs more than it saves
    assert selector.fallback_policy(13520, 560, 688, (256, 128, 64)) in (sk.SK_POLICY_DP, sk.SK_POLICY_SK2_DP)
    # 289 tiles (1.13 waves) with 128 iterations: one or two Stream-K batches, not a second mostly empty wave
    assert selector.fallback_policy(4352, 4352, 8192, (256, 256, 64)) in (sk.SK_POLICY_SK1_DP, sk.SK_POLICY_SK2_DP)


def test_exact_filters_equal_oracle_filters_and_batch_query():
    recs = _fake_records(60, 5)
    sel = selector.PolicySelector(recs, 0.05, "exact")
    o = Bm.build([(r["M"], r["N"], r["K"], Bm.winner_mask(r["time_ns"], 0.05)) for r in recs])
    for f in range(7):
        assert sk.bloom_bits(sel.bloom, f) == o.words[f]
    sizes = [(r["M"], r["N"], r["K"]) for r in recs] + [(17, 19, 23), (1, 2, 3)]
    assert sk.bloom_query_many(sel.bloom, sizes) == [o.query(*s) for s in sizes]
    n = 20000
    t0 = time.perf_counter()
    sk.bloom_query_many(sel.bloom, sizes[:1] * n)
    per_query_us = (time.perf_counter() - t0) / n * 1e6
    assert per_query_us < 50          # paper reports 0.4 us per lookup on one CPU thread; marshalling dominates here
    sel.close()


def test_statistics_shape():
    st = selector.sweep_statistics(_fake_records(40, 9))
    assert abs(sum(st["winner_share"].values()) - 1.0) < 1e-9
    assert st["share_stream_k_within_0_of_dp"] <= st["share_stream_k_within_0.2_of_dp"] <= 1.0
    g = st["gain_over_runner_up"]
    assert sum(v["sizes"] for v in g.values()) <= 40
    for v in g.values():
        assert 0.0 <= v["median"] <= v["p90"] <= v["max"]


def test_runner_up_margin_by_hand():
    # two schedules (policies 1..6 share sk_tiles): DP 100, the Stream-K schedule 80 -> winner SK1_DP, margin 100/80 - 1
    rec = {"M": 64, "N": 64, "K": 64, "tiles": 4, "sk_tiles": [0, 4, 4, 4, 4, 4, 4], "time_ns": [100, 80, 80, 80, 80, 80, 80]}
    st = selector.sweep_statistics([rec])
    assert st["gain_over_runner_up"] == {"SK1_DP": {"sizes": 1, "median": 0.25, "p90": 0.25, "max": 0.25}}


def test_tile_filters_no_false_negatives_and_fallback():
    rng = random.Random(7)
    tiles = [(256, 256, 64), (128, 128, 64), (32, 128, 64)]
    recs = []
    for _ in range(90):
        size = tuple(16 * rng.randint(4, 512) for _ in range(3))
        small = size[0] * size[1] < 512 * 512
        recs.append((size, {tiles[0]: 9000 if small else 5000, tiles[1]: 7000 + rng.randint(0, 50),
                            tiles[2]: 5000 if small else 9000}))
    for mode in ("exact", "class"):
        sel = selector.TileSelector(recs[:60], tiles, 0.1, mode)
        for size, best in recs[:60]:
            want = selector.winner_mask([best[t] for t in tiles], 0.1)
            assert sel.candidates(size) & want == want                    # every inserted winner comes back
            tile, mask, fb = sel.select(size)
            assert not fb and tile in tiles and (mask >> tiles.index(tile)) & 1
        sel.close()
        rep = selector.evaluate_tiles(recs, 60, 0.1, mode)
        assert rep["false_negatives"] == 0 and 0 < rep["held_mean_ratio"] <= 1
        assert rep["held_fallbacks"] == (30 if mode == "exact" else rep["held_fallbacks"])
    assert selector.size_class_key(64, 65, 4096) == (6, 7, 6) and selector.size_class_key(1, 2, 3, (1, 1, 1)) == (0, 1, 2)
    # a size no filter knows falls back to the dispatcher's own tile
    sel = selector.TileSelector(recs[:5], tiles, 0.0, "exact")
    assert sel.select((4096, 4096, 4096)) == ((256, 256, 64), 0, True)     # 256 tiles of 256 x 256: one full wave
    sel.close()


def test_fit_tool_formula_is_the_library_cost_model():
    # the fitting tool restates the dispatcher's formula; with the library's constants it must pick the
    # tile that sk_default_tile picks, on all 500 sweep sizes and the skinny family
    from paper_2408_11417_amd import fit_tile_model as F, inputs
    shapes = inputs.sweep_shapes(500, 4) + [(M, N, K) for M in (16, 32, 64, 128) for N, K in ((8192, 8192), (4096, 4096), (16384, 4096))]
    for M, N, K in shapes:
        pick = min(F.LIBRARY["tflops"], key=lambda t: (F.predict(F.LIBRARY, t, M, N, K), -t[0] * t[1]))
        blk = sk.sk_default_tile(M, N, K, sk.SK_BF16)
        est = {t: F.predict(F.LIBRARY, t, M, N, K) for t in F.LIBRARY["tflops"]}
        assert tuple(blk[:2]) == pick or abs(est[tuple(blk[:2])] - est[pick]) <= 1e-9 * est[pick], (M, N, K, blk, pick)
    # fp8: a modelled pick between the two 8-bit shapes, and an estimate for every policy
    for M, N, K in [(8192, 8192, 8192), (300, 700, 4096), (2048, 1024, 512)]:
        blk = sk.sk_default_tile(M, N, K, sk.SK_FP8_E4M3)
        assert tuple(blk) in ((256, 256, 128), (128, 256, 128))
        plan = sk.sk_plan(M, N, K, sk.SK_POLICY_ALL_SK, None, 256, sk.SK_FP8_E4M3)
        try:
            assert sk.sk_plan_estimate_us(plan) > 0
        finally:
            sk.sk_plan_destroy(plan)
    assert tuple(sk.sk_default_tile(8192, 8192, 8192, sk.SK_FP8_E4M3)) == (256, 256, 128)


def test_winner_mask_error_paths_and_hand_values():
    import ctypes
    lib = sk.binding._lib
    out = ctypes.c_uint32(77)
    arr = (ctypes.c_int64 * 3)(100, 120, 121)
    assert lib.bloom_winner_mask(arr, 3, 200, ctypes.byref(out)) == sk.SK_OK and out.value == 0b011      # 120 <= 100 * 1.2 < 121
    assert lib.bloom_winner_mask(arr, 3, 0, ctypes.byref(out)) == sk.SK_OK and out.value == 0b001
    out.value = 77
    assert lib.bloom_winner_mask(arr, 0, 0, ctypes.byref(out)) == sk.SK_ERR_INVALID_ARG and out.value == 77
    assert lib.bloom_winner_mask(None, 3, 0, ctypes.byref(out)) == sk.SK_ERR_INVALID_ARG
    neg = (ctypes.c_int64 * 2)(-1, 5)
    assert lib.bloom_winner_mask(neg, 2, 0, ctypes.byref(out)) == sk.SK_ERR_INVALID_ARG and out.value == 77
