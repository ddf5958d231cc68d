"""Bloom-filter policy selection on top of a tuning sweep (Sec. 4.2 of the paper).

Records from `sweep.py` say how long each of the seven policies took for a problem size.  The
policies within a tolerance of the best are that size's winners; the size (or, for sizes that
were never profiled, its shape key, see bloom_shape_key) is inserted into the filter of each
winner.  A query returns the candidate policies; the profiler then times only those, or - when no
timing is wanted - the candidate that won most often in the build set is taken.

    python -m paper_2408_11417_amd.selector --sweep sweep_bf16.json --split 400
    python -m paper_2408_11417_amd.selector --tile-sweeps sweep_tile_*.json --split 400     (tile shape as a second parameter)

The first prints, for tolerances 0 / 5 % / 20 %: false negatives on the build split, pruning rate, and on
the held-out split the ratio selected / best and the share of shapes at >= 90 % of the best.
All filter work goes through the C library; nothing here needs a GPU.
"""
import argparse
import json
import sys
import time

from . import binding as sk

N_POL = sk.SK_NUM_POLICIES


def winner_mask(times_ns, tol):
    """Bit p set iff policy p is within (1 + tol) of the fastest (the library's integer rule, bloom_winner_mask)."""
    return sk.bloom_winner_mask(times_ns, int(round(tol * 1000)))


def shape_key(M, N, K, tile=None, grid=256, in_dtype=sk.SK_BF16):
    plan = sk.sk_plan(M, N, K, sk.SK_POLICY_DP, tuple(tile) if tile else None, grid, in_dtype)
    try:
        return sk.bloom_shape_key(plan)
    finally:
        sk.sk_plan_destroy(plan)


def model_estimates(M, N, K, tile, grid=256, dtype=sk.SK_BF16):
    """The library's cost model (sk_plan_estimate_us, the tile dispatcher's model) for the seven policies."""
    est = []
    for p in range(N_POL):
        plan = sk.sk_plan(M, N, K, p, tuple(tile), grid, dtype)
        try:
            est.append(sk.sk_plan_estimate_us(plan))
        finally:
            sk.sk_plan_destroy(plan)
    return est


def fallback_policy(M, N, K, tile, grid=256, dtype=sk.SK_BF16):
    """Used when no filter knows the key: the policy the cost model ranks first; ties go to the
    lower policy number.  Scoring every size of the sweep's build split as if it had fallen through,
    the pick reaches 90 % of the best of seven on 98 % of them (mean 0.987); the earlier rule -
    data-parallel if its waves keep 60 % of the grid busy, else one Stream-K batch - 89 % (mean 0.972)."""
    est = model_estimates(M, N, K, tile, grid, dtype)
    return est.index(min(est))


class PolicySelector:
    """Filters built from sweep records.  mode 'exact' keys by (M, N, K) as the paper does;
    mode 'shape' keys by bloom_shape_key so that unseen sizes can be answered."""

    def __init__(self, records, tol=0.2, mode="shape", grid=256):
        self.tol, self.mode, self.grid = tol, mode, grid
        self.wins = [0] * N_POL
        merged = {}
        for r in records:
            t = r["time_ns"]
            self.wins[t.index(min(t))] += 1
            key = self.key_of(r)
            merged[key] = merged.get(key, 0) | winner_mask(t, tol)
        self.inserted = merged
        self.bloom = sk.bloom_build([(k[0], k[1], k[2], m) for k, m in merged.items()])

    def key_of(self, r):
        if self.mode == "exact":
            return (r["M"], r["N"], r["K"])
        return shape_key(r["M"], r["N"], r["K"], r.get("tile"), self.grid)

    def candidates(self, r):
        return sk.bloom_query(self.bloom, *self.key_of(r))

    def select(self, r, times_ns=None):
        """(policy, candidate mask, used_fallback).  With times: the fastest candidate (the profiler
        ran only the candidates); without: the candidate the cost model ranks first (ties: the one
        with most wins in the build set)."""
        mask = self.candidates(r)
        cands = [p for p in range(N_POL) if (mask >> p) & 1]
        fell_back = not cands
        if fell_back:
            cands = [fallback_policy(r["M"], r["N"], r["K"], r["tile"], self.grid)]
        if times_ns is not None:
            return min(cands, key=lambda p: times_ns[p]), mask, fell_back
        if len(cands) == 1:
            return cands[0], mask, fell_back
        est = model_estimates(r["M"], r["N"], r["K"], r["tile"], self.grid)
        return min(cands, key=lambda p: (est[p], -self.wins[p], p)), mask, fell_back

    def close(self):
        sk.bloom_destroy(self.bloom)


def evaluate(records, split, tol, mode):
    build, held = records[:split], records[split:]
    sel = PolicySelector(build, tol, mode)
    out = {"tol": tol, "mode": mode, "build_sizes": len(build), "held_out_sizes": len(held),
           "distinct_keys": len(sel.inserted)}
    # build split: every inserted (key, policy) must come back; count what the filters prune
    fn = kept = kept_non_dp = 0
    for r in build:
        want = winner_mask(r["time_ns"], tol)
        got = sel.candidates(r)
        fn += bin(want & ~got).count("1")
        kept += bin(got).count("1")
        kept_non_dp += bin(got >> 1).count("1")
    out["false_negatives"] = fn
    out["pruning_rate_build"] = 1 - kept / (N_POL * len(build))
    out["pruning_rate_build_non_dp"] = 1 - kept_non_dp / ((N_POL - 1) * len(build))
    # held-out split
    ratios, ratios_static, kept, miss, fallbacks, dist_kept, dist_all = [], [], 0, 0, 0, 0, 0
    t0 = time.perf_counter()
    for r in held:
        sel.candidates(r)
    out["query_us_incl_key"] = (time.perf_counter() - t0) / max(len(held), 1) * 1e6
    for r in held:
        t = r["time_ns"]
        p, mask, fb = sel.select(r, t)
        ps, _, _ = sel.select(r)
        cands = [q for q in range(N_POL) if (mask >> q) & 1] or [p]
        kept += len(cands)
        fallbacks += fb
        miss += t.index(min(t)) not in cands and min(t) < min(t[q] for q in cands)
        ratios.append(min(t) / t[p])
        ratios_static.append(min(t) / t[ps])
        dist_kept += len({r["sk_tiles"][q] for q in cands})
        dist_all += len(set(r["sk_tiles"]))
    n = max(len(held), 1)
    out.update({
        "held_pruning_rate": 1 - kept / (N_POL * n),
        "held_pruning_rate_distinct_schedules": 1 - dist_kept / max(dist_all, 1),
        "held_fallbacks": fallbacks, "held_best_not_among_candidates": miss,
        "held_share_ge_0.9_of_best": sum(x >= 0.9 for x in ratios) / n,
        "held_mean_ratio": sum(ratios) / n, "held_min_ratio": min(ratios) if ratios else None,
        "held_share_ge_0.9_no_timing": sum(x >= 0.9 for x in ratios_static) / n,
    })
    sel.close()
    return out


def sweep_statistics(records):
    """Winner shares and tolerance curve in the style of Sec. 5.2."""
    n = len(records)
    wins = [0] * N_POL
    gains = []
    for r in records:
        t = r["time_ns"]
        w = t.index(min(t))
        wins[w] += 1
        if w != 0:
            gains.append(t[0] / min(t) - 1)
    out = {"sizes": n, "winner_share": {sk.POLICY_NAMES[p]: wins[p] / n for p in range(N_POL)},
           "stream_k_winner_mean_gain_over_dp": sum(gains) / len(gains) if gains else 0.0,
           "stream_k_winner_max_gain_over_dp": max(gains) if gains else 0.0}
    for tol in (0.0, 0.05, 0.1, 0.2):
        out["share_stream_k_within_%g_of_dp" % tol] = sum(
            min(r["time_ns"][1:]) * 1000 <= r["time_ns"][0] * (1000 + int(tol * 1000)) for r in records) / n
    # per winning policy: by how much it beats the runner-up, the best *different* schedule
    # (policies with the same number of Stream-K tiles are one schedule), in the style of Sec. 5.2
    margins = [[] for _ in range(N_POL)]
    for r in records:
        t = r["time_ns"]
        w = t.index(min(t))
        others = [t[q] for q in range(N_POL) if r["sk_tiles"][q] != r["sk_tiles"][w]]
        if others:
            margins[w].append(min(others) / t[w] - 1)
    out["gain_over_runner_up"] = {}
    for p in range(N_POL):
        m = sorted(margins[p])
        if m:
            out["gain_over_runner_up"][sk.POLICY_NAMES[p]] = {
                "sizes": len(m), "median": m[len(m) // 2], "p90": m[min(len(m) - 1, (9 * len(m)) // 10)], "max": m[-1]}
    return out


# ---- tile shape as a second Bloom-filtered tuning parameter -----------------------------------
# Sec. 4.2 closes with the remark that further tuning parameters can get filters of their own.  Here:
# one filter per tile shape the dispatcher picks from; a size is inserted into the filters of the
# tile shapes whose best policy is within a tolerance of the best (tile, policy) pair of that size.

def size_class_key(M, N, K, octaves=(1, 1, 2)):
    """Key for sizes that were never profiled: the size class ceil(log2 dim) of each dimension, in
    units of `octaves` octaves (tile choice depends mostly on how many tiles M and N make, less on K)."""
    return tuple(((int(d) - 1).bit_length() + o - 1) // o for d, o in zip((M, N, K), octaves))


def tile_records(sweeps):
    """sweeps: {tile: records of a sweep run with --tile}.  Returns per size (M, N, K) a dict
    tile -> best time over the policies, in the order of the first sweep."""
    tiles = list(sweeps)
    out = []
    for i, r in enumerate(sweeps[tiles[0]]):
        size = (r["M"], r["N"], r["K"])
        best = {}
        for t in tiles:
            q = sweeps[t][i]
            assert (q["M"], q["N"], q["K"]) == size
            best[t] = min(q["time_ns"])
        out.append((size, best))
    return out


class TileSelector:
    """One Bloom filter per tile shape.  mode 'exact' keys by (M, N, K); mode 'class' by size_class_key."""

    def __init__(self, recs, tiles, tol=0.1, mode="class", octaves=(1, 1, 2)):
        self.tiles, self.tol, self.mode, self.octaves = list(tiles), tol, mode, octaves
        merged = {}
        for size, best in recs:
            key = self.key_of(size)
            merged[key] = merged.get(key, 0) | winner_mask([best[t] for t in self.tiles], tol)
        self.inserted = merged
        self.bloom = sk.bloom_build([(k[0], k[1], k[2], m) for k, m in merged.items()], n_filters=len(self.tiles))

    def key_of(self, size):
        return tuple(size) if self.mode == "exact" else size_class_key(*size, self.octaves)

    def candidates(self, size):
        return sk.bloom_query(self.bloom, *self.key_of(size))

    def select(self, size):
        """(tile, candidate mask, used_fallback): among the candidate tile shapes the one the library's
        cost model ranks first (under its best policy); among all tile shapes when no filter knows the key."""
        mask = self.candidates(size)
        cands = [t for i, t in enumerate(self.tiles) if (mask >> i) & 1]
        if len(cands) == 1:
            return cands[0], mask, False
        return self.model_pick(size, cands or self.tiles), mask, not cands

    @staticmethod
    def model_pick(size, tiles):
        return min(tiles, key=lambda t: min(model_estimates(*size, t)))

    def close(self):
        sk.bloom_destroy(self.bloom)


def evaluate_tiles(recs, split, tol, mode, octaves=(1, 1, 2)):
    build, held = recs[:split], recs[split:]
    tiles = list(build[0][1])
    sel = TileSelector(build, tiles, tol, mode, octaves)
    out = {"tol": tol, "mode": mode, "octaves": list(octaves), "tiles": [list(t) for t in tiles],
           "build_sizes": len(build), "held_out_sizes": len(held), "distinct_keys": len(sel.inserted)}
    fn = kept = 0
    for size, best in build:
        want = winner_mask([best[t] for t in tiles], tol)
        got = sel.candidates(size)
        fn += bin(want & ~got).count("1")
        kept += bin(got).count("1")
    out["false_negatives"] = fn
    out["pruning_rate_build"] = 1 - kept / (len(tiles) * len(build))
    ratios, ratios_model, fallbacks, kept = [], [], 0, 0
    for size, best in held:
        tile, mask, fb = sel.select(size)
        fallbacks += fb
        kept += bin(mask).count("1") or 1
        ratios.append(min(best.values()) / best[tuple(tile)])
        ratios_model.append(min(best.values()) / best[sel.model_pick(size, tiles)])
    n = max(len(held), 1)
    out.update({"held_fallbacks": fallbacks, "held_pruning_rate": 1 - kept / (len(tiles) * n),
                "held_mean_ratio": sum(ratios) / n, "held_min_ratio": min(ratios) if ratios else None,
                "held_share_ge_0.9_of_best": sum(x >= 0.9 for x in ratios) / n,
                "cost_model_alone_mean_ratio": sum(ratios_model) / n,
                "cost_model_alone_share_ge_0.9": sum(x >= 0.9 for x in ratios_model) / n})
    sel.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sweep", default="")
    ap.add_argument("--tile-sweeps", nargs="*", default=[],
                    help="sweep files made with --tile, one per tile shape: evaluate tile-shape filters instead of policy filters")
    ap.add_argument("--split", type=int, default=400)
    ap.add_argument("--held-sweeps", nargs="*", default=[],
                    help="other sweep files: build from the first --split sizes of --sweep, hold out every size of these")
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    if args.tile_sweeps:
        sweeps = {}
        for f in args.tile_sweeps:
            recs = json.load(open(f))["records"]
            sweeps[tuple(recs[0]["tile"])] = recs
        recs = tile_records(sweeps)
        report = {"tile_evaluations": [evaluate_tiles(recs, args.split, tol, mode)
                                       for mode in ("exact", "class") for tol in (0.0, 0.05, 0.1, 0.2)]}
        text = json.dumps(report, indent=1)
        print(text)
        if args.out:
            open(args.out, "w").write(text)
        return 0
    records = json.load(open(args.sweep))["records"]
    if args.held_sweeps:
        seen = {(r["M"], r["N"], r["K"]) for r in records[:args.split]}
        records = records[:args.split]
        for f in args.held_sweeps:
            for r in json.load(open(f))["records"]:
                if (r["M"], r["N"], r["K"]) not in seen:
                    seen.add((r["M"], r["N"], r["K"]))
                    records.append(r)
    report = {"statistics": sweep_statistics(records), "evaluations": []}
    for mode in ("exact", "shape"):
        for tol in (0.0, 0.05, 0.2):
            report["evaluations"].append(evaluate(records, args.split, tol, mode))
    text = json.dumps(report, indent=1)
    print(text)
    if args.out:
        open(args.out, "w").write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
