"""The host code of the library (planner, Bloom selector) under AddressSanitizer and UBSan.

streamk_plan.cpp and streamk_bloom.cpp are compiled host-only with g++ and both sanitizers (runtime
linked statically, reports fatal) together with tests/host/sanitizer_driver.cpp, which replays cases
written here by the CPU oracle - random schedules under every policy, tile order, batch order and
segment order; Bloom sets with random records and queries - and compares every number.  CPU only."""
import os
import random
import shutil
import subprocess

import pytest

from oracle import bloom as Bm
from oracle import schedule as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2408_11417_amd", "csrc")


def _write_cases(path, n_plans=400, n_blooms=6, seed=7):
    rng = random.Random(seed)
    with open(path, "w") as f:
        for _ in range(n_plans):
            bm, bn, bk = rng.choice([16, 32, 64, 128, 256]), rng.choice([64, 128, 256]), rng.choice([16, 32, 64, 128])
            M, N, K = rng.randint(1, 9 * bm), rng.randint(1, 7 * bn), rng.randint(1, 40 * bk)
            g = rng.choice([1, 3, 8, 24, 37, 64, 256])
            policy, order = rng.randrange(8), rng.randrange(2)
            dp_first, k_aligned = rng.randrange(2), rng.randrange(2)
            p = S.plan(M, N, K, policy, bm, bn, bk, g, order, dp_first=bool(dp_first), k_aligned=bool(k_aligned))
            f.write("plan %d %d %d %d %d %d %d %d %d %d %d %d\n" % (M, N, K, policy, bm, bn, bk, g, order, dp_first, k_aligned, len(p.segments)))
            for s in p.segments:
                f.write("%d %d %d %d %d\n" % tuple(s))
            for r in p.ranges:
                f.write("%d %d %d %d\n" % tuple(r))
        for i in range(n_blooms):
            m_bits, k_probes, n_filters = rng.choice([64, 640, Bm.M_BITS]), rng.choice([1, 3, 7]), rng.choice([1, 7, 32])
            recs = [(rng.randrange(1, 1 << rng.choice([8, 16, 32])), rng.randrange(1, 1 << 20), rng.randrange(1, 1 << 16),
                     rng.randrange(1 << n_filters)) for _ in range(rng.choice([0, 1, 50, 400]))]
            bs = Bm.build(recs, m_bits, k_probes, n_filters)
            queries = [r[:3] for r in recs[:40]] + [(rng.randrange(1, 1 << 20), rng.randrange(1, 1 << 20), rng.randrange(1, 1 << 20)) for _ in range(60)]
            f.write("bloom %d %d %d %d %d\n" % (m_bits, k_probes, n_filters, len(recs), len(queries)))
            for r in recs:
                f.write("%d %d %d %d\n" % r)
            for p in range(n_filters):
                fold = 0
                for w, word in enumerate(bs.words[p]):
                    fold ^= (word * (2 * w + 1)) & 0xFFFFFFFFFFFFFFFF
                f.write("%d %d\n" % (fold, bs.popcount(p)))
            for q in queries:
                f.write("%d %d %d %d\n" % (q + (bs.query(*q),)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_and_bloom_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe, cases = str(tmp_path / "sanitizer_driver"), str(tmp_path / "cases.txt")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "streamk_plan.cpp"), os.path.join(CSRC, "streamk_bloom.cpp"),
           os.path.join(ROOT, "tests", "host", "sanitizer_driver.cpp"), "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    _write_cases(cases)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe, cases], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert res.stdout.strip().startswith("ok 400 plans 6 bloom sets"), res.stdout[-2000:]
