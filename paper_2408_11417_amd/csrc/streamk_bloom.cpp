// Bloom-filter policy selector (Sec. 4.2): one bit array per scheduling policy,
// keyed by a 32-bit Murmur3 hash of the problem size.  Host code, integers only.
#include <cstring>
#include <new>
#include <vector>
#include "streamk.h"

struct sk_bloom_t {
    uint32_t m_bits, k_probes, n_filters;
    std::vector<std::vector<uint64_t>> filters;
};

namespace {

inline uint32_t rotl(uint32_t v, int r) { return (v << r) | (v >> (32 - r)); }

inline uint32_t scramble(uint32_t k) {
    k *= 0xCC9E2D51u;
    k = rotl(k, 15);
    return k * 0x1B873593u;
}

inline uint32_t avalanche(uint32_t h) {
    h ^= h >> 16; h *= 0x85EBCA6Bu;
    h ^= h >> 13; h *= 0xC2B2AE35u;
    return h ^ (h >> 16);
}

uint32_t murmur3(const uint8_t* p, size_t len, uint32_t seed) {
    uint32_t h = seed;
    size_t i = 0;
    for (; i + 4 <= len; i += 4) {
        const uint32_t k = (uint32_t)p[i] | (uint32_t)p[i + 1] << 8 | (uint32_t)p[i + 2] << 16 | (uint32_t)p[i + 3] << 24;
        h = rotl(h ^ scramble(k), 13) * 5u + 0xE6546B64u;
    }
    if (i < len) {
        uint32_t k = 0;
        for (size_t j = len; j-- > i;) k = (k << 8) | p[j];
        h ^= scramble(k);
    }
    return avalanche(h ^ (uint32_t)len);
}

// Three-word key specialisation of the same hash (no tail, length 12).
inline uint32_t hash_key(uint32_t M, uint32_t N, uint32_t K, uint32_t seed) {
    uint32_t h = seed;
    h = rotl(h ^ scramble(M), 13) * 5u + 0xE6546B64u;
    h = rotl(h ^ scramble(N), 13) * 5u + 0xE6546B64u;
    h = rotl(h ^ scramble(K), 13) * 5u + 0xE6546B64u;
    return avalanche(h ^ 12u);
}

void insert(sk_bloom_t* b, const sk_bloom_record& r) {
    for (uint32_t p = 0; p < b->n_filters; p++) {
        if (!((r.policy_mask >> p) & 1u)) continue;
        for (uint32_t i = 0; i < b->k_probes; i++) {
            const uint32_t bit = hash_key(r.M, r.N, r.K, p * b->k_probes + i) % b->m_bits;
            b->filters[p][bit >> 6] |= (uint64_t)1 << (bit & 63);
        }
    }
}

}  // namespace

extern "C" uint32_t bloom_murmur3_32(const void* key, size_t len, uint32_t seed) {
    return murmur3(static_cast<const uint8_t*>(key), key ? len : 0, seed);
}

extern "C" int bloom_build(const sk_bloom_record* recs, size_t n, const sk_bloom_params* params, sk_bloom_t** out) {
    if (!out || (!recs && n)) return SK_ERR_INVALID_ARG;
    sk_bloom_params p{};
    if (params) p = *params;
    if (!p.m_bits) p.m_bits = 95872;
    if (!p.k_probes) p.k_probes = 7;
    if (!p.n_filters) p.n_filters = SK_NUM_POLICIES;
    if (p.m_bits % 64 || p.n_filters > 32 || p.k_probes > 64) return SK_ERR_INVALID_ARG;
    sk_bloom_t* b = new (std::nothrow) sk_bloom_t;
    if (!b) return SK_ERR_NOMEM;
    b->m_bits = p.m_bits; b->k_probes = p.k_probes; b->n_filters = p.n_filters;
    try {
        b->filters.assign(p.n_filters, std::vector<uint64_t>(p.m_bits / 64, 0));
    } catch (const std::bad_alloc&) {
        delete b;
        return SK_ERR_NOMEM;
    }
    for (size_t i = 0; i < n; i++) insert(b, recs[i]);
    *out = b;
    return SK_OK;
}

extern "C" int bloom_insert(sk_bloom_t* bloom, const sk_bloom_record* rec) {
    if (!bloom || !rec) return SK_ERR_INVALID_ARG;
    insert(bloom, *rec);
    return SK_OK;
}

extern "C" int bloom_query(const sk_bloom_t* bloom, int64_t M, int64_t N, int64_t K, uint32_t* mask_out) {
    if (!bloom || !mask_out) return SK_ERR_INVALID_ARG;
    const int64_t lim = 0xFFFFFFFFll;
    if (M < 0 || N < 0 || K < 0 || M > lim || N > lim || K > lim) return SK_ERR_INVALID_ARG;
    uint32_t mask = 0;
    for (uint32_t p = 0; p < bloom->n_filters; p++) {
        const uint64_t* w = bloom->filters[p].data();
        bool hit = true;
        for (uint32_t i = 0; i < bloom->k_probes && hit; i++) {
            const uint32_t bit = hash_key((uint32_t)M, (uint32_t)N, (uint32_t)K, p * bloom->k_probes + i) % bloom->m_bits;
            hit = (w[bit >> 6] >> (bit & 63)) & 1u;
        }
        if (hit) mask |= 1u << p;
    }
    *mask_out = mask;
    return SK_OK;
}

extern "C" int bloom_query_many(const sk_bloom_t* bloom, const uint32_t* sizes, size_t n, uint32_t* masks_out) {
    if (!bloom || (!sizes && n) || (!masks_out && n)) return SK_ERR_INVALID_ARG;
    for (size_t q = 0; q < n; q++) {
        uint32_t mask = 0;
        for (uint32_t p = 0; p < bloom->n_filters; p++) {
            const uint64_t* w = bloom->filters[p].data();
            bool hit = true;
            for (uint32_t i = 0; i < bloom->k_probes && hit; i++) {
                const uint32_t bit = hash_key(sizes[3 * q], sizes[3 * q + 1], sizes[3 * q + 2], p * bloom->k_probes + i) % bloom->m_bits;
                hit = (w[bit >> 6] >> (bit & 63)) & 1u;
            }
            if (hit) mask |= 1u << p;
        }
        masks_out[q] = mask;
    }
    return SK_OK;
}

extern "C" int bloom_bits(const sk_bloom_t* bloom, int filter, const uint64_t** words, size_t* n_words) {
    if (!bloom || !words || !n_words || filter < 0 || (uint32_t)filter >= bloom->n_filters) return SK_ERR_INVALID_ARG;
    *words = bloom->filters[filter].data();
    *n_words = bloom->filters[filter].size();
    return SK_OK;
}

extern "C" int bloom_winner_mask(const int64_t* times_ns, size_t n, uint32_t tol_permille, uint32_t* mask_out) {
    if (!times_ns || !mask_out || n < 1 || n > 32 || tol_permille > 1000000u) return SK_ERR_INVALID_ARG;
    int64_t best = times_ns[0];
    for (size_t p = 0; p < n; p++) {
        if (times_ns[p] < 0 || times_ns[p] > (int64_t)1 << 40) return SK_ERR_INVALID_ARG;     // (keeps the products below in 64 bits)
        if (times_ns[p] < best) best = times_ns[p];
    }
    uint32_t mask = 0;
    for (size_t p = 0; p < n; p++)
        if (times_ns[p] * 1000 <= best * (1000 + (int64_t)tol_permille)) mask |= 1u << p;
    *mask_out = mask;
    return SK_OK;
}

// Serialised form (little-endian): u32 magic "SKBF", u32 version, u32 m_bits, u32 k_probes,
// u32 n_filters, then n_filters * m_bits / 64 words of 64 bits, filter by filter.
namespace {
constexpr uint32_t BLOOM_MAGIC = 0x46424B53u, BLOOM_VERSION = 1u;
void put_u32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; i++) p[i] = (uint8_t)(v >> (8 * i)); }
uint32_t get_u32(const uint8_t* p) { return (uint32_t)p[0] | (uint32_t)p[1] << 8 | (uint32_t)p[2] << 16 | (uint32_t)p[3] << 24; }
}  // namespace

extern "C" int bloom_serialize(const sk_bloom_t* bloom, void* buf, size_t cap, size_t* n_bytes) {
    if (!bloom || !n_bytes) return SK_ERR_INVALID_ARG;
    const size_t words = (size_t)bloom->n_filters * (bloom->m_bits / 64), need = 20 + 8 * words;
    *n_bytes = need;
    if (!buf || cap < need) return buf || cap ? SK_ERR_INVALID_ARG : SK_OK;     // (NULL, 0) asks for the size only
    uint8_t* p = static_cast<uint8_t*>(buf);
    put_u32(p, BLOOM_MAGIC); put_u32(p + 4, BLOOM_VERSION); put_u32(p + 8, bloom->m_bits);
    put_u32(p + 12, bloom->k_probes); put_u32(p + 16, bloom->n_filters);
    p += 20;
    for (const std::vector<uint64_t>& f : bloom->filters)
        for (uint64_t w : f) {
            put_u32(p, (uint32_t)w); put_u32(p + 4, (uint32_t)(w >> 32));
            p += 8;
        }
    return SK_OK;
}

extern "C" int bloom_deserialize(const void* buf, size_t n_bytes, sk_bloom_t** out) {
    if (!buf || !out || n_bytes < 20) return SK_ERR_INVALID_ARG;
    const uint8_t* p = static_cast<const uint8_t*>(buf);
    if (get_u32(p) != BLOOM_MAGIC || get_u32(p + 4) != BLOOM_VERSION) return SK_ERR_INVALID_ARG;
    const uint32_t m_bits = get_u32(p + 8), k_probes = get_u32(p + 12), n_filters = get_u32(p + 16);
    if (!m_bits || m_bits % 64 || !k_probes || k_probes > 64 || !n_filters || n_filters > 32) return SK_ERR_INVALID_ARG;
    const size_t words = (size_t)n_filters * (m_bits / 64);
    if (n_bytes != 20 + 8 * words) return SK_ERR_INVALID_ARG;
    sk_bloom_t* b = new (std::nothrow) sk_bloom_t;
    if (!b) return SK_ERR_NOMEM;
    b->m_bits = m_bits; b->k_probes = k_probes; b->n_filters = n_filters;
    try {
        b->filters.assign(n_filters, std::vector<uint64_t>(m_bits / 64, 0));
    } catch (const std::bad_alloc&) {
        delete b;
        return SK_ERR_NOMEM;
    }
    p += 20;
    for (std::vector<uint64_t>& f : b->filters)
        for (uint64_t& w : f) {
            w = (uint64_t)get_u32(p) | (uint64_t)get_u32(p + 4) << 32;
            p += 8;
        }
    *out = b;
    return SK_OK;
}

extern "C" void bloom_destroy(sk_bloom_t* bloom) { delete bloom; }
