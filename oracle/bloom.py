"""Bloom-filter oracle: one filter per scheduling policy, keyed by a Murmur hash of (M, N, K).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Pure-Python integers.

What it follows (Sec. 4.2)
--------------------------
* Seven filters, one per Stream-K++ policy; a problem size is inserted into the
  filter of every policy that is a winner for it.
* Keys are derived from (M, N, K) with a Murmur hash.
* Each filter is sized for 10 000 problem sizes.
* A query checks all seven filters and returns the policies that may apply; a
  policy that was inserted is never rejected (no false negatives).

Readings taken where the paper is silent
----------------------------------------
B1  Hash = MurmurHash3, 32-bit variant, over the 12-byte key made of M, N, K as
    little-endian unsigned 32-bit integers.
B2  "Seven distinct hash functions, one per filter": filter p uses k = 7 probes
    with seeds p*k + i (i = 0..k-1), so every filter has its own hash family and
    every probe its own seed.
B3  10 000 keys at a 1 % false-positive target gives
    m = ceil(-n ln p / ln^2 2) = 95 851 bits, rounded up to whole 64-bit words:
    m = 95 872.  The constant is fixed, not recomputed in floating point.
    Bit j lives in word j // 64 at bit position j % 64.
"""

N_FILTERS = 7
K_PROBES = 7
M_BITS = 95872
MASK32 = 0xFFFFFFFF


def _rotl32(x, r):
    return ((x << r) | (x >> (32 - r))) & MASK32


def murmur3_32(data, seed):
    """MurmurHash3 (x86, 32-bit) of a bytes object, written from the published algorithm:
    4-byte little-endian blocks are scrambled (multiply, rotate 15, multiply) and
    mixed into the state (xor, rotate 13, times 5 plus a constant); the 1-3 tail
    bytes are scrambled the same way without the state mix; the length is xored
    in and the state is finalised by the xor-shift / multiply avalanche."""
    c1, c2 = 0xCC9E2D51, 0x1B873593
    h = seed & MASK32
    n = len(data)
    nblocks = n // 4
    for b in range(nblocks):
        k = int.from_bytes(data[4 * b:4 * b + 4], "little")
        k = (k * c1) & MASK32
        k = _rotl32(k, 15)
        k = (k * c2) & MASK32
        h ^= k
        h = _rotl32(h, 13)
        h = (h * 5 + 0xE6546B64) & MASK32
    tail = data[4 * nblocks:]
    if tail:
        k = int.from_bytes(tail, "little")
        k = (k * c1) & MASK32
        k = _rotl32(k, 15)
        k = (k * c2) & MASK32
        h ^= k
    h ^= n
    h ^= h >> 16
    h = (h * 0x85EBCA6B) & MASK32
    h ^= h >> 13
    h = (h * 0xC2B2AE35) & MASK32
    h ^= h >> 16
    return h


def key_bytes(M, N, K):
    """Reading B1: the 12-byte key."""
    return b"".join(int(v).to_bytes(4, "little") for v in (M, N, K))


def probe_positions(M, N, K, policy, m_bits=M_BITS, k_probes=K_PROBES):
    """Bit positions that (M, N, K) touches in the filter of `policy` (reading B2)."""
    kb = key_bytes(M, N, K)
    return [murmur3_32(kb, policy * k_probes + i) % m_bits for i in range(k_probes)]


class BloomSet:
    """The seven filters.  `words[p]` is filter p as a list of 64-bit words (reading B3)."""

    def __init__(self, m_bits=M_BITS, k_probes=K_PROBES, n_filters=N_FILTERS):
        if m_bits < 64 or m_bits % 64 or k_probes < 1 or n_filters < 1:
            raise ValueError("bad Bloom parameters")
        self.m_bits, self.k_probes, self.n_filters = m_bits, k_probes, n_filters
        self.words = [[0] * (m_bits // 64) for _ in range(n_filters)]

    def insert(self, M, N, K, policy_mask):
        """Insert the size into the filter of every policy whose bit is set in the mask."""
        for p in range(self.n_filters):
            if (policy_mask >> p) & 1:
                for j in probe_positions(M, N, K, p, self.m_bits, self.k_probes):
                    self.words[p][j // 64] |= 1 << (j % 64)

    def query(self, M, N, K):
        """Mask of the policies whose filter holds all k bits of the key."""
        mask = 0
        for p in range(self.n_filters):
            if all((self.words[p][j // 64] >> (j % 64)) & 1
                   for j in probe_positions(M, N, K, p, self.m_bits, self.k_probes)):
                mask |= 1 << p
        return mask

    def popcount(self, p):
        return sum(bin(w).count("1") for w in self.words[p])


def build(records, m_bits=M_BITS, k_probes=K_PROBES, n_filters=N_FILTERS):
    """records: iterable of (M, N, K, policy_mask)."""
    bs = BloomSet(m_bits, k_probes, n_filters)
    for M, N, K, mask in records:
        bs.insert(M, N, K, mask)
    return bs


def shape_key(header):
    """Key for sizes outside the profiled set (extension; Sec. 4.2 keys by the exact size, which
    never matches an unseen size): tile shape, full waves of tiles capped at 3, fill of the
    remainder wave in quarters of the grid rounded up, floor(log2(iterations per tile)) capped at
    12.  `header` is the plan header of the scheduler oracle."""
    g = header["grid"]
    waves = min(header["tiles"] // g, 3)
    fill = -(-4 * (header["tiles"] % g) // g)
    lg = min(header["iters_per_tile"].bit_length() - 1, 12)
    return (header["blk_m"] << 16 | header["blk_n"], waves << 8 | fill, lg << 16 | header["blk_k"])


def winner_mask(times, tol):
    """Mask of the policies whose time is within (1 + tol) of the best one (Sec. 4.2 inserts
    the winning configurations; Sec. 5.2's tolerance thresholds widen "winning").
    The comparison is done in integers on times given in nanoseconds: t*1000 <= best*(1000+tol_permille)."""
    best = min(times)
    permille = int(round(tol * 1000))
    mask = 0
    for p, t in enumerate(times):
        if t * 1000 <= best * (1000 + permille):
            mask |= 1 << p
    return mask


def pruning_rate(masks, n_filters=N_FILTERS):
    """Fraction of (size, policy) evaluations that the candidate masks eliminate (Sec. 4.2)."""
    kept = sum(bin(m).count("1") for m in masks)
    return 1.0 - kept / float(n_filters * len(masks))
