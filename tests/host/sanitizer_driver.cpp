// Host-only check of the planner and the Bloom selector under AddressSanitizer / UBSan: reads cases
// written by the CPU oracle (tests/test_host_sanitizers.py), runs them through the C ABI of
// streamk_plan.cpp + streamk_bloom.cpp (compiled with g++, no GPU code) and compares every number.
// Exit status 0 = all cases equal; any sanitizer report aborts the run.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "streamk.h"
#include "streamk_internal.h"

// the planner asks the GEMM launcher whether a kernel exists; this build has no launcher
bool sk_kernel_available(int, int, int, int) { return false; }

#define FAIL(...) do { fprintf(stderr, __VA_ARGS__); fprintf(stderr, "\n"); return 1; } while (0)

static int plan_case(FILE* f) {
    long long M, N, K;
    int policy, bm, bn, bk, grid, order, dp_first, k_aligned;
    long long n_seg;
    if (fscanf(f, "%lld %lld %lld %d %d %d %d %d %d %d %d %lld", &M, &N, &K, &policy, &bm, &bn, &bk, &grid, &order, &dp_first, &k_aligned, &n_seg) != 12)
        FAIL("bad plan line");
    sk_config cfg{};
    cfg.blk_m = bm; cfg.blk_n = bn; cfg.blk_k = bk; cfg.grid = grid; cfg.tile_order = order + 1;
    sk_plan_t* plan = nullptr;
    if (sk_plan(M, N, K, policy, &cfg, &plan) != SK_OK) FAIL("sk_plan failed");
    if (sk_plan_set_batch_order(plan, dp_first) != SK_OK || sk_plan_set_segment_order(plan, k_aligned) != SK_OK) FAIL("setters failed");
    size_t n = 0;
    sk_plan_segments(plan, nullptr, 0, &n);
    if ((long long)n != n_seg) FAIL("segment count %zu != %lld (M=%lld N=%lld K=%lld policy=%d)", n, n_seg, M, N, K, policy);
    std::vector<sk_segment> segs(n ? n : 1);
    if (sk_plan_segments(plan, segs.data(), n, &n) != SK_OK) FAIL("sk_plan_segments failed");
    for (size_t i = 0; i < n; i++) {
        int wg, tile, kb, ke, role;
        if (fscanf(f, "%d %d %d %d %d", &wg, &tile, &kb, &ke, &role) != 5) FAIL("bad segment");
        const sk_segment& s = segs[i];
        if (s.wg != wg || s.tile != tile || s.k_begin != kb || s.k_end != ke || s.role != role)
            FAIL("segment %zu differs (M=%lld N=%lld K=%lld policy=%d)", i, M, N, K, policy);
    }
    std::vector<sk_wg_range> ranges(grid);
    if (sk_plan_ranges(plan, ranges.data()) != SK_OK) FAIL("sk_plan_ranges failed");
    for (int x = 0; x < grid; x++) {
        long long b, e;
        int first, count;
        if (fscanf(f, "%lld %lld %d %d", &b, &e, &first, &count) != 4) FAIL("bad range");
        if (ranges[x].sk_iter_begin != b || ranges[x].sk_iter_end != e || ranges[x].dp_tile_first != first || ranges[x].dp_tile_count != count)
            FAIL("range %d differs", x);
    }
    sk_plan_header h;
    sk_plan_info(plan, &h);
    for (int t = 0; t < h.tiles; t += (h.tiles / 64 + 1)) {
        int32_t tm, tn;
        if (sk_plan_tile_coords(plan, t, &tm, &tn) != SK_OK || tm < 0 || tm >= h.tiles_m || tn < 0 || tn >= h.tiles_n) FAIL("tile coords");
    }
    uint32_t key[3];
    bloom_shape_key(plan, key);
    double us;
    sk_plan_estimate_us(plan, &us);
    sk_plan_destroy(plan);
    return 0;
}

static int bloom_case(FILE* f) {
    unsigned m_bits, k_probes, n_filters;
    int n_rec, n_query;
    if (fscanf(f, "%u %u %u %d %d", &m_bits, &k_probes, &n_filters, &n_rec, &n_query) != 5) FAIL("bad bloom line");
    std::vector<sk_bloom_record> recs(n_rec ? n_rec : 1);
    for (int i = 0; i < n_rec; i++)
        if (fscanf(f, "%u %u %u %u", &recs[i].M, &recs[i].N, &recs[i].K, &recs[i].policy_mask) != 4) FAIL("bad record");
    sk_bloom_params p{m_bits, k_probes, n_filters};
    sk_bloom_t* b = nullptr;
    if (bloom_build(recs.data(), (size_t)n_rec / 2, &p, &b) != SK_OK) FAIL("bloom_build failed");
    for (int i = n_rec / 2; i < n_rec; i++)
        if (bloom_insert(b, &recs[i]) != SK_OK) FAIL("bloom_insert failed");
    for (unsigned fl = 0; fl < n_filters; fl++) {
        const uint64_t* words;
        size_t nw;
        if (bloom_bits(b, (int)fl, &words, &nw) != SK_OK || nw != m_bits / 64) FAIL("bloom_bits failed");
        uint64_t fold = 0, pop = 0;
        for (size_t w = 0; w < nw; w++) { fold ^= words[w] * (2 * w + 1); pop += (uint64_t)__builtin_popcountll(words[w]); }
        unsigned long long want_fold, want_pop;
        if (fscanf(f, "%llu %llu", &want_fold, &want_pop) != 2) FAIL("bad fold");
        if (fold != want_fold || pop != want_pop) FAIL("filter %u differs", fl);
    }
    std::vector<uint32_t> sizes(3 * (n_query ? n_query : 1)), masks(n_query ? n_query : 1), want(n_query ? n_query : 1);
    for (int i = 0; i < n_query; i++)
        if (fscanf(f, "%u %u %u %u", &sizes[3 * i], &sizes[3 * i + 1], &sizes[3 * i + 2], &want[i]) != 4) FAIL("bad query");
    if (bloom_query_many(b, sizes.data(), (size_t)n_query, masks.data()) != SK_OK) FAIL("bloom_query_many failed");
    for (int i = 0; i < n_query; i++) {
        uint32_t one = 0;
        if (bloom_query(b, sizes[3 * i], sizes[3 * i + 1], sizes[3 * i + 2], &one) != SK_OK || one != masks[i] || one != want[i]) FAIL("query %d differs", i);
    }
    bloom_destroy(b);
    return 0;
}

// The multiply-shift division the kernels use for their index arithmetic equals n / d for every divisor and
// every numerator below 2^31 (checked: all small divisors and seeded random ones, numerators at and next to
// every multiple boundary that matters and at the top of the range).
static int fast_div_case() {
    uint64_t state = 12345;
    auto next = [&]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(state >> 33); };
    for (int c = 0; c < 70000; c++) {
        const uint32_t d = c < 5000 ? (uint32_t)c + 1 : c < 5032 ? 1u << (c - 5000) % 31 : 1 + next() % (1u << (1 + next() % 30));
        const sk_fast_div f = sk_make_fast_div(d);
        if (f.shift < 31 || f.shift > 62 || (uint64_t)f.mul * d < (1ull << f.shift)) FAIL("bad constants for %u", d);
        const uint32_t top = 0x7FFFFFFFu;
        uint32_t ns[12] = {0, 1, d - 1, d, d + 1, top, top - 1, top / d * d, top / d * d - 1, next() & top, next() & top, (next() % 1024) * d + d - 1};
        for (uint32_t n : ns) {
            if (n > top) continue;
            if (sk_fast_div_apply(n, f) != n / d) FAIL("%u / %u: got %u", n, d, sk_fast_div_apply(n, f));
        }
    }
    const sk_fast_div zero = sk_make_fast_div(0);
    if (zero.mul != 0 || zero.shift != 0) FAIL("divisor 0");
    return 0;
}

int main(int argc, char** argv) {
    if (argc != 2) FAIL("usage: sanitizer_driver CASES");
    if (fast_div_case()) return 1;
    FILE* f = fopen(argv[1], "r");
    if (!f) FAIL("cannot open %s", argv[1]);
    char kind[16];
    int n_plan = 0, n_bloom = 0;
    while (fscanf(f, "%15s", kind) == 1) {
        if (!strcmp(kind, "plan")) { if (plan_case(f)) return 1; n_plan++; }
        else if (!strcmp(kind, "bloom")) { if (bloom_case(f)) return 1; n_bloom++; }
        else FAIL("unknown case kind %s", kind);
    }
    fclose(f);
    // error paths must leave their out-parameters alone and leak nothing
    sk_plan_t* none = nullptr;
    if (sk_plan(0, 1, 1, 0, nullptr, &none) == SK_OK || none) FAIL("bad size accepted");
    if (sk_plan(1, 1, 1, 99, nullptr, &none) == SK_OK || none) FAIL("bad policy accepted");
    printf("ok %d plans %d bloom sets\n", n_plan, n_bloom);
    return 0;
}
