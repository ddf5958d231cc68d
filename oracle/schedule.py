"""Scheduler oracle: which workgroup runs which MAC-loop iterations.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Integer arithmetic in plain
Python, one step per passage of the paper, no blocking or shortcuts.

What it follows
---------------
* Algorithm 1 (Sec. 3.1): iterations per tile, total iterations, the equal
  split of the iteration space over g workgroups, and the outer loop that cuts a
  workgroup's range at output-tile boundaries.
* Sec. 3.2: the all-Stream-K schedule (everything is split, no data-parallel
  work) and the hybrids, where a "batch" is one trip of Algorithm 1's outer loop
  for every workgroup, i.e. at most one tile's worth of iterations each.
* Sec. 4.1: a persistent grid of g workgroups; Stream-K batches (zero to six) are
  issued first and data-parallel batches after them, so the fix-up latency of
  the split tiles hides under data-parallel work.
* Sec. 5.3: the fix-up by partial results plus inter-workgroup synchronisation
  (instead of atomic adds); that is where OWNER / CONTRIB roles come from.

Readings taken where the paper is silent or ambiguous
-----------------------------------------------------
R1  The seven policies are b = 0 (pure data-parallel), b = 1..5 Stream-K batches
    followed by data-parallel batches, and all-Stream-K.  b = 6 is kept as an
    eighth, extension id.
R2  With W = T div g full waves and rem = T mod g leftover tiles, b Stream-K
    batches cover sk_tiles = min(T, rem + (b-1)*g) tiles ("one batch" = the
    remainder wave, "two batches" = remainder plus one full wave, Sec. 3.2).
    If rem = 0 and b = 1 nothing is left over, so the schedule equals pure DP.
R3  The Stream-K tiles are the lowest tile indices [0, sk_tiles); the
    data-parallel tiles follow and workgroup x takes sk_tiles + x + j*g.
R4  Algorithm 1 does not clamp a workgroup's range to the iteration total; both
    ends are clamped here (trailing workgroups may be empty).  The split is the
    paper's ceil split, not a balanced one.
R5  Tile index -> coordinates: row-major over the tile grid (order 0), or - because
    Sec. 5.3 asks for cache locality when work is handed to compute units - grouped
    (order 1): the grid is cut into bands of 8 tile rows, and inside a band the
    index walks down the band's rows first and then moves one column to the right,
    so that consecutive tile indices form compact blocks that share A row-blocks
    and B column-blocks.  Either order is a bijection; the schedule (which
    workgroup runs which tile index) is the same for both.
R6  The workgroup whose segment holds a tile's k-iteration 0 owns the tile; the
    others store an fp32 partial in workspace slot = their workgroup id and the
    owner adds them in ascending workgroup order (= ascending k).
    (R7 - R9 of the design notes concern the garbled statement of Algorithm 1, the
    grid and the tile sizes; nothing in this file depends on them.)
R10 k_aligned=True is an execution order the paper does not have; it answers the
    loss of cache locality that Sec. 5.3 remarks on.  Which workgroup runs which
    iterations is Algorithm 1's, unchanged.  A workgroup whose range contains a
    tile boundary runs its whole tiles first, then the piece at the end of its
    range (k-iterations from 0 of its last tile), then the piece at the start of
    its range (the last k-iterations of its first tile); whole tiles and pieces
    from k = 0 then start together in all workgroups.  The owner of a split tile
    is the workgroup holding the tile's last k-iteration - its final piece of work,
    so it waits for nobody - and it adds the partials of the others in descending
    workgroup order.
"""
from collections import namedtuple

POLICY_NAMES = ("DP", "SK1_DP", "SK2_DP", "SK3_DP", "SK4_DP", "SK5_DP", "ALL_SK", "SK6_DP_EXT")
POLICY_DP, POLICY_SK1_DP, POLICY_SK2_DP, POLICY_SK3_DP = 0, 1, 2, 3
POLICY_SK4_DP, POLICY_SK5_DP, POLICY_ALL_SK, POLICY_SK6_DP_EXT = 4, 5, 6, 7
SEVEN_POLICIES = (0, 1, 2, 3, 4, 5, 6)

ROLE_FULL, ROLE_OWNER, ROLE_CONTRIB = 0, 1, 2
ORDER_ROW_MAJOR, ORDER_GROUPED = 0, 1
GROUP_ROWS = 8

Segment = namedtuple("Segment", "wg tile k_begin k_end role")
WgRange = namedtuple("WgRange", "sk_iter_begin sk_iter_end dp_tile_first dp_tile_count")
Plan = namedtuple("Plan", "header ranges segments")


def cdiv(a, b):
    return -(-a // b)


def decompose(M, N, K, blk_m, blk_n, blk_k):
    """Algorithm 1, problem decomposition: tile grid, iterations per tile, total iterations."""
    tiles_m = cdiv(M, blk_m)
    tiles_n = cdiv(N, blk_n)
    iters_per_tile = cdiv(K, blk_k)
    tiles = tiles_m * tiles_n
    return tiles_m, tiles_n, tiles, iters_per_tile, tiles * iters_per_tile


def sk_batches(policy):
    """Number of Stream-K batches b of a policy; None means all-Stream-K (Sec. 3.2, 4.1)."""
    if policy == POLICY_ALL_SK:
        return None
    if policy == POLICY_SK6_DP_EXT:
        return 6
    if 0 <= policy <= 5:
        return policy
    raise ValueError("unknown policy %r" % (policy,))


def sk_tile_count(tiles, g, policy):
    """How many output tiles are handed to the Stream-K region (reading R2)."""
    b = sk_batches(policy)
    if b is None:
        return tiles
    if b == 0:
        return 0
    rem = tiles % g
    return min(tiles, rem + (b - 1) * g)


def tile_coords(tile, tiles_m, tiles_n, order=ORDER_ROW_MAJOR):
    """Tile index -> (tile_m, tile_n) (reading R5)."""
    if order == ORDER_ROW_MAJOR:
        return tile // tiles_n, tile % tiles_n
    if order != ORDER_GROUPED:
        raise ValueError("unknown tile order %r" % (order,))
    per_band = GROUP_ROWS * tiles_n
    first_row = (tile // per_band) * GROUP_ROWS
    rows = min(GROUP_ROWS, tiles_m - first_row)       # the last band may be shorter
    within = tile % per_band
    return first_row + within % rows, within // rows


def wg_sk_range(x, sk_iters, iters_per_wg):
    """Algorithm 1, a workgroup's iteration range, clamped to the Stream-K iteration total (reading R4)."""
    begin = min(x * iters_per_wg, sk_iters)
    end = min((x + 1) * iters_per_wg, sk_iters)
    return begin, end


def wg_sk_segments(x, begin, end, iters_per_tile, k_aligned=False):
    """Algorithm 1, the outer loop over a workgroup's range: cut [begin, end) at tile boundaries.

    k_aligned (reading R10) reorders a range that contains a tile boundary into
    whole tiles, piece from k-iteration 0, piece up to the last k-iteration, and
    hands the OWNER role to the piece that reaches the tile's last iteration
    instead of the one that holds its first."""
    segs = []
    if begin < end:
        # the range touches the tiles first_tile .. last_tile; of each of them it holds the k-iterations
        # where the range and the tile's own interval of the iteration space overlap
        first_tile, last_tile = begin // iters_per_tile, (end - 1) // iters_per_tile
        for tile in range(first_tile, last_tile + 1):
            origin = tile * iters_per_tile
            k_begin = max(begin, origin) - origin
            k_end = min(end, origin + iters_per_tile) - origin
            if k_begin == 0 and k_end == iters_per_tile:
                role = ROLE_FULL
            elif k_aligned:
                role = ROLE_OWNER if k_end == iters_per_tile else ROLE_CONTRIB
            else:
                role = ROLE_OWNER if k_begin == 0 else ROLE_CONTRIB
            segs.append(Segment(x, tile, k_begin, k_end, role))
    if k_aligned and len(segs) > 1:
        whole = [s for s in segs if s.role == ROLE_FULL]
        from_zero = [s for s in segs if s.role != ROLE_FULL and s.k_begin == 0]     # at most the last one
        to_end = [s for s in segs if s.role != ROLE_FULL and s.k_begin > 0]         # at most the first one
        segs = whole + from_zero + to_end
    return segs


def plan(M, N, K, policy, blk_m, blk_n, blk_k, g, order=ORDER_ROW_MAJOR, dp_first=False, k_aligned=False):
    """Full schedule for one problem: header, per-workgroup ranges, canonical segment list.

    The segment list is ordered by workgroup, and inside a workgroup in execution
    order: Stream-K segments ascending, then data-parallel tiles ascending
    (Sec. 3.2 / 4.1: Stream-K batches come first).  dp_first=True swaps the two
    phases - the earlier hybrid that Sec. 3.2 describes, data-parallel batches
    followed by the Stream-K work; which tiles are split and which workgroup gets
    which work does not change.  k_aligned=True: reading R10.
    """
    if min(M, N, K, blk_m, blk_n, blk_k, g) < 1:
        raise ValueError("sizes must be positive")
    if order not in (ORDER_ROW_MAJOR, ORDER_GROUPED):
        raise ValueError("unknown tile order %r" % (order,))
    tiles_m, tiles_n, tiles, ipt, total = decompose(M, N, K, blk_m, blk_n, blk_k)
    sk_tiles = sk_tile_count(tiles, g, policy)
    dp_tiles = tiles - sk_tiles
    sk_iters = sk_tiles * ipt
    ipw = cdiv(sk_iters, g)                       # Algorithm 1, iterations per workgroup, on the SK region
    ranges, segments = [], []
    for x in range(g):
        begin, end = wg_sk_range(x, sk_iters, ipw)
        sk_segs = wg_sk_segments(x, begin, end, ipt, k_aligned)
        first = sk_tiles + x
        count = cdiv(tiles - first, g) if first < tiles else 0
        dp_segs = [Segment(x, first + j * g, 0, ipt, ROLE_FULL) for j in range(count)]
        ranges.append(WgRange(begin, end, first if count else tiles, count))
        segments.extend(dp_segs + sk_segs if dp_first else sk_segs + dp_segs)
    header = dict(M=M, N=N, K=K, policy=policy, blk_m=blk_m, blk_n=blk_n, blk_k=blk_k, grid=g,
                  tiles_m=tiles_m, tiles_n=tiles_n, tiles=tiles, iters_per_tile=ipt,
                  total_iters=total, sk_tiles=sk_tiles, dp_tiles=dp_tiles, sk_iters=sk_iters,
                  iters_per_wg=ipw, dp_waves=cdiv(dp_tiles, g), tile_order=order, dp_first=bool(dp_first),
                  k_aligned=bool(k_aligned))
    return Plan(header, ranges, segments)


def contributors(p, owner_segment):
    """Workgroups whose partials the owner of a split tile adds, in reduction order (R6, R10)."""
    ipt, ipw = p.header["iters_per_tile"], p.header["iters_per_wg"]
    assert owner_segment.role == ROLE_OWNER
    first = (owner_segment.tile * ipt) // ipw
    last = (owner_segment.tile * ipt + ipt - 1) // ipw
    if p.header["k_aligned"]:
        assert owner_segment.wg == last
        return list(range(last - 1, first - 1, -1))
    assert owner_segment.wg == first
    return list(range(first + 1, last + 1))


def makespan_iters(p):
    """MAC-loop iterations executed by the busiest workgroup."""
    load = [0] * p.header["grid"]
    for s in p.segments:
        load[s.wg] += s.k_end - s.k_begin
    return max(load)
