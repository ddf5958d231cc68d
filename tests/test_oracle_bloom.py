"""Pins for the Bloom oracle: published hash vectors, a library hash, and the set properties
that Sec. 4.2 of the paper relies on (no false negatives, sizing for 10 000 keys)."""
import math
import os
import random

import pytest

from oracle import bloom as Bm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kats():
    for line in open(os.path.join(GOLDEN, "murmur3_32_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, seed, want = line.split()
        yield (b"" if key == "-" else bytes.fromhex(key)), int(seed, 16), int(want, 16)


def test_murmur3_known_answers():
    rows = list(_kats())
    assert len(rows) == 18
    for key, seed, want in rows:
        assert Bm.murmur3_32(key, seed) == want


def test_murmur3_matches_library_implementation():
    sk = pytest.importorskip("sklearn.utils")
    rng = random.Random(0)
    for _ in range(2000):
        key = bytes(rng.getrandbits(8) for _ in range(rng.randint(0, 40)))
        seed = rng.getrandbits(32)
        assert Bm.murmur3_32(key, seed) == sk.murmurhash3_32(key, seed=seed, positive=True)
    for M, N, K in [(1, 64, 16), (8192, 8192, 65536), (3840, 4224, 4096)]:
        kb = Bm.key_bytes(M, N, K)
        assert len(kb) == 12 and int.from_bytes(kb[4:8], "little") == N
        assert Bm.murmur3_32(kb, 48) == sk.murmurhash3_32(kb, seed=48, positive=True)


def test_filter_size_for_ten_thousand_keys_at_one_percent():
    m = math.ceil(-10000 * math.log(0.01) / math.log(2) ** 2)
    assert m == 95851
    assert Bm.M_BITS == 64 * math.ceil(m / 64) == 95872
    assert Bm.K_PROBES == round(Bm.M_BITS / 10000 * math.log(2)) == 7
    assert Bm.N_FILTERS == 7


def _records(n, seed):
    rng = random.Random(seed)
    recs = {}
    while len(recs) < n:
        key = tuple(16 * rng.randint(1, 1024) for _ in range(3))
        recs[key] = rng.randint(1, 127)
    return [(M, N, K, mask) for (M, N, K), mask in recs.items()]


def test_no_false_negatives_and_structure():
    recs = _records(923, 1)
    bs = Bm.build(recs)
    for M, N, K, mask in recs:
        assert Bm.BloomSet.query(bs, M, N, K) & mask == mask
    for p in range(7):
        inserts = sum((mask >> p) & 1 for *_, mask in recs)
        assert 0 < bs.popcount(p) <= Bm.K_PROBES * inserts
        assert len(bs.words[p]) == Bm.M_BITS // 64 and all(0 <= w < 2 ** 64 for w in bs.words[p])


def test_empty_filter_rejects_everything_and_single_insert_sets_its_probe_bits():
    bs = Bm.BloomSet()
    assert bs.query(512, 512, 512) == 0
    bs.insert(512, 512, 512, 1 << 3)
    pos = set(Bm.probe_positions(512, 512, 512, 3))
    assert all(0 <= j < Bm.M_BITS for j in pos)
    assert bs.popcount(3) == len(pos) and all(bs.popcount(p) == 0 for p in range(7) if p != 3)
    for j in pos:
        assert (bs.words[3][j // 64] >> (j % 64)) & 1
    assert bs.query(512, 512, 512) == 1 << 3


def test_insertion_order_and_duplicates_do_not_matter():
    recs = _records(300, 2)
    a = Bm.build(recs)
    b = Bm.build(list(reversed(recs)) + recs[:50])
    assert a.words == b.words


def test_filters_use_distinct_hash_families():
    pos = [tuple(Bm.probe_positions(4096, 4096, 4096, p)) for p in range(7)]
    assert len(set(pos)) == 7
    assert len({j for t in pos for j in t}) > 40


def test_false_positive_rate_matches_theory():
    n = 10000
    recs = [(16 * (i % 1000 + 1), 16 * (i // 1000 + 1), 48, 1) for i in range(n)]
    bs = Bm.build(recs)
    rng = random.Random(3)
    trials, fp = 20000, 0
    for _ in range(trials):
        M, N, K = rng.randint(1, 10 ** 6), rng.randint(1, 10 ** 6), 49   # K = 49 never inserted
        fp += bs.query(M, N, K) & 1
    theory = (1 - math.exp(-Bm.K_PROBES * n / Bm.M_BITS)) ** Bm.K_PROBES
    assert 0.006 < theory < 0.011
    assert abs(fp / trials - theory) < 0.004


def test_winner_mask_and_pruning_rate():
    times = [100, 104, 121, 120, 300, 99, 150]
    assert Bm.winner_mask(times, 0.0) == 1 << 5
    assert Bm.winner_mask(times, 0.05) == (1 << 5) | (1 << 0)
    assert Bm.winner_mask(times, 0.20) == 0b0100011
    assert Bm.pruning_rate([0b1, 0b11, 0b0, 0b1111111]) == pytest.approx(1 - 10 / 28)
