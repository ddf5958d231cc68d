// Host-side scheduler: turns (M, N, K, policy, tile, grid) into the numbers the
// persistent kernel walks, and expands them into the canonical segment list.
// Integer arithmetic only; no device contact.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <vector>
#include "streamk_internal.h"

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Stream-K batches of a policy: 0..6, or -1 for "every tile is split" (Sec. 3.2).
int batches_of(int policy) {
    switch (policy) {
    case SK_POLICY_ALL_SK: return -1;
    case SK_POLICY_SK6_DP_EXT: return 6;
    default: return policy;   // DP .. SK5_DP carry their batch count as enum value
    }
}

bool dtype_in_ok(int d) { return d == SK_F16 || d == SK_BF16 || d == SK_FP8_E4M3; }
bool dtype_out_ok(int d) { return d == SK_F16 || d == SK_BF16 || d == SK_F32; }

// Segments of workgroup x, appended in execution order.
void expand_wg(const sk_plan_header& h, int x, std::vector<sk_segment>* out, sk_wg_range* range, bool dp_first = false,
               bool k_aligned = false) {
    const int64_t ipt = h.iters_per_tile;
    int64_t it = x * (int64_t)h.iters_per_wg;
    int64_t end = it + h.iters_per_wg;
    if (it > h.sk_iters) it = h.sk_iters;
    if (end > h.sk_iters) end = h.sk_iters;
    if (range) { range->sk_iter_begin = it; range->sk_iter_end = end; }
    const size_t at = out ? out->size() : 0;     // where this workgroup's segments start
    auto role_of = [&](const sk_segment& s) {
        if (s.k_begin == 0 && s.k_end == ipt) return SK_ROLE_FULL;
        const bool contributor = k_aligned ? s.k_end < ipt : s.k_begin > 0;
        return contributor ? SK_ROLE_CONTRIB : SK_ROLE_OWNER;
    };
    // a range that contains a tile boundary runs, in the k-aligned order, its whole tiles, then the
    // head piece of its last tile, then the tail piece of its first tile
    int64_t sub[3][2] = {{it, end}, {end, end}, {end, end}};
    if (k_aligned && it < end) {
        const int64_t first_full = ceil_div(it, ipt) * ipt, last_full = end / ipt * ipt;
        if (first_full <= last_full) {
            sub[0][0] = first_full; sub[0][1] = last_full;
            sub[1][0] = last_full;  sub[1][1] = end;
            sub[2][0] = it;         sub[2][1] = first_full;
        }
    }
    for (const auto& r : sub) {
        // Algorithm 1, outer loop: one segment per tile the range touches
        for (int64_t i = r[0]; i < r[1];) {
            const int64_t tile = i / ipt;
            const int64_t tile_first = tile * ipt;
            const int64_t stop = (r[1] < tile_first + ipt) ? r[1] : tile_first + ipt;
            sk_segment s;
            s.wg = x;
            s.tile = (int32_t)tile;
            s.k_begin = (int32_t)(i - tile_first);
            s.k_end = (int32_t)(stop - tile_first);
            s.role = role_of(s);
            if (out) out->push_back(s);
            i = stop;
        }
    }
    // data-parallel tiles follow the Stream-K work (Sec. 4.1) - or precede it (Sec. 3.2's earlier hybrid)
    int32_t count = 0;
    for (int64_t t = (int64_t)h.sk_tiles + x; t < h.tiles; t += h.grid) {
        if (out) {
            const sk_segment s{x, (int32_t)t, 0, (int32_t)ipt, SK_ROLE_FULL};
            if (dp_first) out->insert(out->begin() + (std::ptrdiff_t)(at + count), s);
            else out->push_back(s);
        }
        ++count;
    }
    if (range) {
        range->dp_tile_count = count;
        range->dp_tile_first = count ? h.sk_tiles + x : h.tiles;
    }
}

// Cost model shared by the tile dispatcher and sk_plan_estimate_us.  The constants (sustained
// TFLOP/s of each 16-bit kernel with the grid full, microseconds to drain / store a tile and to
// park or fetch a partial) were fitted to timings of every tile shape on the first 400 of 500 seeded
// problem sizes plus 12 large skinny ones on MI355X - sizes 400 .. 499 are the selector's held-out split
// and stay out of the fit (fit_tile_model.py; the fit optimises the dispatcher's pick, not the
// predicted times, so the constants need not be physical).
struct TileCost { int bm, bn; double tflops; };
const TileCost tile_costs[] = {{256, 256, 1170.}, {256, 128, 1027.}, {128, 128, 826.}, {64, 128, 624.}, {32, 128, 297.}, {16, 128, 47.}};
constexpr int MODEL_GRID = 256;
double model_iter_us(const TileCost& c, int bk) {          // one k-iteration of every workgroup of a full grid
    return 2.0 * c.bm * c.bn * bk * MODEL_GRID / (c.tflops * 1e12) * 1e6;
}
double model_tile_us(const TileCost& c) { return 0.69 + c.bm * c.bn * 2 / 8.86e3; }
// exchange of partial tiles when about `split` workgroups share a tile: the partials an owner (or a
// group leader) fetches one after the other - all of them up to 16 workgroups per tile, beyond that
// the two-level reduction with groups of 8
double model_exchange_us(const TileCost& c, double split) {
    const bool tree = split >= 16;
    const double serial = tree ? 8 + split / 8 : split;
    return 5.77 * (tree ? 2 : 1) + serial * c.bm * c.bn * 4 / 35.9e3;
}

// The constants of a tile shape.  The 8-bit kernels were not fitted: they move the same bytes per
// k-iteration as the 16-bit kernel of the same footprint with twice the k at twice the matrix-core
// rate, so an 8-bit tile is modelled as that 16-bit shape (128 x 256 as 256 x 128) with half its blk_k.
const TileCost* model_constants(int bm, int bn, int in_dtype) {
    if (in_dtype == SK_FP8_E4M3 && bm < bn) std::swap(bm, bn);
    for (const TileCost& t : tile_costs)
        if (t.bm == bm && t.bn == bn) return &t;
    return nullptr;
}
int model_bk(int blk_k, int in_dtype) { return in_dtype == SK_FP8_E4M3 ? blk_k / 2 : blk_k; }

}  // namespace

extern "C" int sk_plan_estimate_us(const sk_plan_t* plan, double* microseconds) {
    if (!plan || !microseconds) return SK_ERR_INVALID_ARG;
    const sk_plan_header& h = plan->h;
    const TileCost* c = model_constants(h.blk_m, h.blk_n, h.in_dtype);
    if (!c) return SK_ERR_UNSUPPORTED;
    // per-iteration time of a workgroup does not depend on how many workgroups the grid has
    const double t_iter = model_iter_us(*c, model_bk(h.blk_k, h.in_dtype)), c_tile = model_tile_us(*c);
    double t = h.dp_waves * (h.iters_per_tile * t_iter + c_tile);
    if (h.sk_tiles > 0) {
        const double sk_waves = (double)h.sk_tiles / h.grid;
        t += h.iters_per_wg * t_iter + c_tile * (sk_waves > 1 ? sk_waves : 1.0);
        if (plan->needs_fixup) {
            double split = (double)h.iters_per_tile / h.iters_per_wg;     // workgroups per tile beyond the owner, about
            if (split < 1) split = 1;
            t += model_exchange_us(*c, split);
            // every workgroup that holds a contributor piece parks one fp32 tile and somebody fetches it, all at
            // about the same time: that traffic shares the memory system (fitted: 6 TB/s for write plus read;
            // with 256 x 256 tiles and a full grid it is 128 MB, the largest term of a short problem)
            int64_t contributors = 0;
            for (int64_t x = 0; x < h.grid; x++) {
                const int64_t b = std::min<int64_t>(x * h.iters_per_wg, h.sk_iters), e = std::min<int64_t>((x + 1) * h.iters_per_wg, h.sk_iters);
                if (e > b && (plan->k_aligned ? e : b) % h.iters_per_tile != 0) contributors++;
            }
            t += (double)contributors * c->bm * c->bn * 8 / 6.0e6;
        }
    }
    *microseconds = t;
    return SK_OK;
}

extern "C" int sk_default_tile(int64_t M, int64_t N, int64_t K, int in_dtype, int32_t* out_blk) {
    if (!out_blk || M < 1 || N < 1 || K < 1 || !dtype_in_ok(in_dtype)) return SK_ERR_INVALID_ARG;
    // Dispatcher: a small cost model over the tile shapes that have a kernel.  For each shape it
    // estimates the time of the better of (a) whole tiles in waves over the grid and (b) the
    // iterations split evenly over the grid plus the cost of exchanging partial tiles, and keeps
    // the cheapest; the model's choice is within 10 % of the fastest tile shape on 95 % of the
    // sizes it was fitted on.
    // candidates: the six 16-bit shapes, or the two 8-bit shapes (modelled through model_constants)
    struct Cand { int bm, bn, bk; };
    static const Cand cands16[] = {{256, 256, 64}, {256, 128, 64}, {128, 128, 64}, {64, 128, 64}, {32, 128, 64}, {16, 128, 64}};
    static const Cand cands8[] = {{256, 256, 128}, {128, 256, 128}};
    const bool fp8 = in_dtype == SK_FP8_E4M3;
    const Cand* cands = fp8 ? cands8 : cands16;
    const int n_cands = fp8 ? 2 : 6, grid = MODEL_GRID;
    double best_t = 0;
    int best = -1;
    for (int i = 0; i < n_cands; i++) {
        const TileCost& c = *model_constants(cands[i].bm, cands[i].bn, in_dtype);
        const double ipt = (double)ceil_div(K, cands[i].bk);
        const double tiles = (double)ceil_div(M, cands[i].bm) * (double)ceil_div(N, cands[i].bn);
        const double t_iter = model_iter_us(c, model_bk(cands[i].bk, in_dtype)), c_tile = model_tile_us(c);
        const double waves = (double)((int64_t)((tiles + grid - 1) / grid));
        const double t_dp = waves * (ipt * t_iter + c_tile);
        const double ipw = (double)((int64_t)((tiles * ipt + grid - 1) / grid));
        double split = grid / tiles;
        if (split > ipt) split = ipt;
        if (split < 1) split = 1;
        double t_sk = ipw * t_iter + c_tile * (tiles > grid ? tiles / grid : 1.0);
        if (((int64_t)tiles % grid) != 0) t_sk += model_exchange_us(c, split);
        const double t = t_dp < t_sk ? t_dp : t_sk;
        if (best < 0 || t < best_t) { best = i; best_t = t; }
    }
    out_blk[0] = cands[best].bm; out_blk[1] = cands[best].bn; out_blk[2] = cands[best].bk;
    return SK_OK;
}

extern "C" int sk_plan(int64_t M, int64_t N, int64_t K, int policy, const sk_config* cfg, sk_plan_t** out) {
    if (!out || M < 1 || N < 1 || K < 1) return SK_ERR_INVALID_ARG;
    if (policy < 0 || policy > SK_POLICY_SK6_DP_EXT) return SK_ERR_INVALID_ARG;
    sk_config c{};
    if (cfg) c = *cfg;
    if (c.blk_m < 0 || c.blk_n < 0 || c.blk_k < 0 || c.grid < 0 || c.tile_order < 0) return SK_ERR_INVALID_ARG;
    const int in_dtype = c.in_dtype ? c.in_dtype - 1 : SK_BF16;
    if (!dtype_in_ok(in_dtype)) return SK_ERR_INVALID_ARG;
    const int out_dtype = c.out_dtype ? c.out_dtype - 1 : (in_dtype == SK_FP8_E4M3 ? SK_BF16 : in_dtype);
    if (!dtype_out_ok(out_dtype)) return SK_ERR_INVALID_ARG;
    int order = c.tile_order ? c.tile_order - 1 : -1;   // -1: decided below, once the split is known
    if (order != -1 && order != SK_ORDER_ROW_MAJOR && order != SK_ORDER_GROUPED) return SK_ERR_INVALID_ARG;
    int32_t blk[3] = {c.blk_m, c.blk_n, c.blk_k};
    if (!blk[0] || !blk[1] || !blk[2]) {
        int32_t def[3];
        sk_default_tile(M, N, K, in_dtype, def);
        for (int i = 0; i < 3; i++) if (!blk[i]) blk[i] = def[i];
    }
    const int grid = c.grid ? c.grid : 256;

    sk_plan_header h{};
    h.M = M; h.N = N; h.K = K; h.policy = policy;
    h.blk_m = blk[0]; h.blk_n = blk[1]; h.blk_k = blk[2]; h.grid = grid;
    h.in_dtype = in_dtype; h.out_dtype = out_dtype;
    // Algorithm 1: iterations per tile, total iterations
    const int64_t tiles_m = ceil_div(M, blk[0]), tiles_n = ceil_div(N, blk[1]);
    const int64_t ipt = ceil_div(K, blk[2]);
    const int64_t tiles = tiles_m * tiles_n;
    const int64_t imax = std::numeric_limits<int32_t>::max();
    if (tiles_m > imax || tiles_n > imax || tiles > imax - grid || ipt > imax) return SK_ERR_INVALID_ARG;
    if (tiles > std::numeric_limits<int64_t>::max() / ipt) return SK_ERR_INVALID_ARG;
    h.tiles_m = (int32_t)tiles_m; h.tiles_n = (int32_t)tiles_n; h.tiles = (int32_t)tiles;
    h.iters_per_tile = (int32_t)ipt;
    h.total_iters = tiles * ipt;
    // Stream-K / data-parallel split (Sec. 3.2, Sec. 4.1)
    const int b = batches_of(policy);
    int64_t sk_tiles;
    if (b < 0) sk_tiles = tiles;
    else if (b == 0) sk_tiles = 0;
    else {
        sk_tiles = tiles % grid + (int64_t)(b - 1) * grid;
        if (sk_tiles > tiles) sk_tiles = tiles;
    }
    // Default tile order: the one under which the tiles that an XCD's workgroups hold at the same
    // time touch fewer operand rows and columns (A row-blocks x blk_m + B column-blocks x blk_n,
    // averaged over the XCDs): that is what the XCD's L2 has to keep per k-iteration.  The
    // workgroups of the grid hold the first min(tiles, grid) tile indices at once, an eighth of
    // them (consecutive indices) per XCD.  Picking by this figure loses 0.4 - 0.7 % against the
    // faster order of each size on a 500-size sweep (either order alone: 0.5 - 3 %, up to 1.5x).
    if (order < 0) {
        auto footprint = [&](int ord) {
            const int64_t active = tiles < grid ? tiles : grid;
            const int64_t per_xcd = active / 8 > 0 ? active / 8 : 1;
            double total = 0;
            int chunks = 0;
            for (int64_t c = 0; c < active; c += per_xcd, ++chunks) {
                std::vector<int64_t> row, col;
                for (int64_t t = c; t < c + per_xcd && t < active; t++) {
                    int64_t tm, tn;
                    if (ord == SK_ORDER_ROW_MAJOR) {
                        tm = t / tiles_n; tn = t % tiles_n;
                    } else {
                        const int64_t per_band = SK_GROUP_ROWS * tiles_n, first = t / per_band * SK_GROUP_ROWS;
                        const int64_t band_rows = tiles_m - first < SK_GROUP_ROWS ? tiles_m - first : SK_GROUP_ROWS;
                        tm = first + t % per_band % band_rows; tn = t % per_band / band_rows;
                    }
                    row.push_back(tm);
                    col.push_back(tn);
                }
                std::sort(row.begin(), row.end());
                std::sort(col.begin(), col.end());
                const auto rows = std::unique(row.begin(), row.end()) - row.begin();
                const auto cols = std::unique(col.begin(), col.end()) - col.begin();
                total += (double)rows * blk[0] + (double)cols * blk[1];
            }
            return total / chunks;
        };
        try {
            order = footprint(SK_ORDER_GROUPED) < footprint(SK_ORDER_ROW_MAJOR) ? SK_ORDER_GROUPED : SK_ORDER_ROW_MAJOR;
        } catch (const std::bad_alloc&) {
            return SK_ERR_NOMEM;
        }
    }
    h.tile_order = order;
    h.fixup = SK_FIXUP_FLAGS;
    h.batch_order = SK_STREAMK_FIRST;
    h.segment_order = SK_SEGMENTS_K_ALIGNED;
    // A single row of low tiles streams B once, in column blocks that are narrow stripes of the same
    // memory rows, and shares only the small A: there the hardware order (neighbouring column
    // blocks on different XCDs) measured 8 - 10 % faster (M <= 64, N = K = 8192: 28.5 against
    // 31.5 us).  Everything else measured faster renumbered - a single column of tiles, two rows
    // of tiles, and also a single row of 128-row tiles (M = 128: 42 against 48 us).
    h.xcd_remap = (tiles_m == 1 && blk[0] <= 64) ? 0 : 1;
    h.sk_tiles = (int32_t)sk_tiles;
    h.dp_tiles = (int32_t)(tiles - sk_tiles);
    h.sk_iters = sk_tiles * ipt;
    const int64_t ipw = ceil_div(h.sk_iters, grid);   // Algorithm 1: iterations per workgroup, on the split region
    if (ipw > imax) return SK_ERR_INVALID_ARG;
    h.iters_per_wg = (int32_t)ipw;
    h.dp_waves = (int32_t)ceil_div(h.dp_tiles, grid);
    h.has_kernel = sk_kernel_available(in_dtype, blk[0], blk[1], blk[2]) ? 1 : 0;

    sk_plan_t* p = new (std::nothrow) sk_plan_t;
    if (!p) return SK_ERR_NOMEM;
    p->h = h;
    // a tile is split iff some workgroup range ends strictly inside it
    p->needs_fixup = (h.sk_iters > ipw && ipw % ipt != 0) ? 1 : 0;
    *out = p;
    return SK_OK;
}

extern "C" int sk_plan_info(const sk_plan_t* plan, sk_plan_header* out) {
    if (!plan || !out) return SK_ERR_INVALID_ARG;
    *out = plan->h;
    return SK_OK;
}

extern "C" int sk_plan_ranges(const sk_plan_t* plan, sk_wg_range* out) {
    if (!plan || !out) return SK_ERR_INVALID_ARG;
    for (int x = 0; x < plan->h.grid; x++) expand_wg(plan->h, x, nullptr, &out[x]);
    return SK_OK;
}

extern "C" int sk_plan_segments(const sk_plan_t* plan, sk_segment* out, size_t cap, size_t* n) {
    if (!plan || !n || (!out && cap)) return SK_ERR_INVALID_ARG;
    std::vector<sk_segment> segs;
    try {
        for (int x = 0; x < plan->h.grid; x++) expand_wg(plan->h, x, &segs, nullptr, plan->dp_first != 0, plan->k_aligned != 0);
    } catch (const std::bad_alloc&) {
        return SK_ERR_NOMEM;
    }
    *n = segs.size();
    if (segs.size() > cap) return SK_ERR_INVALID_ARG;
    if (!segs.empty()) std::memcpy(out, segs.data(), segs.size() * sizeof(sk_segment));
    return SK_OK;
}

extern "C" int sk_plan_tile_coords(const sk_plan_t* plan, int32_t tile, int32_t* tile_m, int32_t* tile_n) {
    if (!plan || !tile_m || !tile_n || tile < 0 || tile >= plan->h.tiles) return SK_ERR_INVALID_ARG;
    const sk_plan_header& h = plan->h;
    if (h.tile_order == SK_ORDER_ROW_MAJOR) {
        *tile_m = tile / h.tiles_n;
        *tile_n = tile % h.tiles_n;
    } else {
        // bands of SK_GROUP_ROWS tile rows, walked column by column
        const int per_band = SK_GROUP_ROWS * h.tiles_n;
        const int band_row = (tile / per_band) * SK_GROUP_ROWS;
        const int rows = h.tiles_m - band_row < SK_GROUP_ROWS ? h.tiles_m - band_row : SK_GROUP_ROWS;
        const int within = tile % per_band;
        *tile_m = band_row + within % rows;
        *tile_n = within / rows;
    }
    return SK_OK;
}

extern "C" int bloom_shape_key(const sk_plan_t* plan, uint32_t* key) {
    if (!plan || !key) return SK_ERR_INVALID_ARG;
    const sk_plan_header& h = plan->h;
    uint32_t waves = (uint32_t)(h.tiles / h.grid);
    if (waves > 3) waves = 3;
    const uint32_t rem = (uint32_t)(h.tiles % h.grid);
    const uint32_t fill = (4 * rem + (uint32_t)h.grid - 1) / (uint32_t)h.grid;   // 0 = no remainder wave, 1..4 quarters
    uint32_t lg = 0;
    for (uint32_t v = (uint32_t)h.iters_per_tile; v > 1; v >>= 1) lg++;
    if (lg > 12) lg = 12;
    key[0] = (uint32_t)h.blk_m << 16 | ((uint32_t)h.blk_n & 0xFFFFu);
    key[1] = waves << 8 | fill;
    key[2] = lg << 16 | ((uint32_t)h.blk_k & 0xFFFFu);
    return SK_OK;
}

extern "C" size_t sk_workspace_bytes(const sk_plan_t* plan) {
    if (!plan) return 0;
    const sk_plan_header& h = plan->h;
    if (plan->fixup == SK_FIXUP_ATOMIC) return sk_ws_partials_offset(h.grid) + sk_ws_image_bytes(plan);
    return sk_ws_partials_offset(h.grid) + (size_t)h.grid * h.blk_m * h.blk_n * sizeof(float);
}

extern "C" int sk_plan_set_fixup(sk_plan_t* plan, int fixup) {
    if (!plan || (fixup != SK_FIXUP_FLAGS && fixup != SK_FIXUP_ATOMIC) || plan->workspace) return SK_ERR_INVALID_ARG;
    plan->fixup = fixup;
    plan->h.fixup = fixup;
    return SK_OK;
}

extern "C" int sk_plan_set_batch_order(sk_plan_t* plan, int batch_order) {
    if (!plan || (batch_order != SK_STREAMK_FIRST && batch_order != SK_DATA_PARALLEL_FIRST)) return SK_ERR_INVALID_ARG;
    plan->dp_first = batch_order == SK_DATA_PARALLEL_FIRST;
    plan->h.batch_order = batch_order;
    return SK_OK;
}

extern "C" int sk_plan_set_segment_order(sk_plan_t* plan, int segment_order) {
    if (!plan || (segment_order != SK_SEGMENTS_ASCENDING && segment_order != SK_SEGMENTS_K_ALIGNED)) return SK_ERR_INVALID_ARG;
    plan->k_aligned = segment_order == SK_SEGMENTS_K_ALIGNED;
    plan->h.segment_order = segment_order;
    return SK_OK;
}

extern "C" int sk_plan_set_spin_limit(sk_plan_t* plan, uint32_t polls) {
    if (!plan) return SK_ERR_INVALID_ARG;
    plan->spin_limit = polls;
    return SK_OK;
}

extern "C" int sk_plan_set_kernel_variant(sk_plan_t* plan, int variant) {
    if (!plan || variant < 0) return SK_ERR_INVALID_ARG;
    plan->kernel_variant = variant;
    return SK_OK;
}

extern "C" void sk_plan_destroy(sk_plan_t* plan) { delete plan; }

extern "C" const char* sk_status_str(int status) {
    switch (status) {
    case SK_OK: return "ok";
    case SK_ERR_INVALID_ARG: return "invalid argument";
    case SK_ERR_UNSUPPORTED: return "unsupported configuration";
    case SK_ERR_WORKSPACE: return "workspace missing or too small";
    case SK_ERR_HIP: return "HIP runtime error";
    case SK_ERR_NOMEM: return "out of host memory";
    case SK_ERR_TIMEOUT: return "tile owner timed out waiting for a partial tile";
    default: return "unknown status";
    }
}
