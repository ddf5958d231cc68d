"""Host side of libstreamk.so against the oracles, bit for bit: schedules, Bloom bits, hash;
plus the ABI surface (every declared symbol exported) and the error paths.  No GPU needed."""
import ctypes
import os
import random
import re

import pytest
from hypothesis import given, settings, strategies as st

import paper_2408_11417_amd as sk
from oracle import schedule as S
from oracle import bloom as Bm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "streamk.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:sk|bloom)_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sk.binding.EXPORTS)
    lib = ctypes.CDLL(sk.binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_public_header_is_plain_c_and_links(tmp_path):
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    exe = str(tmp_path / "header_is_c")
    lib_dir = os.path.dirname(sk.binding.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host", "header_is_c.c"), "-L", lib_dir, "-l:libstreamk.so", "-Wl,-rpath," + lib_dir,
           "-Wl,--allow-shlib-undefined", "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), (res.returncode, res.stdout[-2000:])


def _plan_pair(M, N, K, policy, blk, g, order=None, dp_first=False, k_aligned=None):
    p = sk.sk_plan(M, N, K, policy, blk, g, tile_order=order)
    try:
        assert sk.sk_plan_info(p)["segment_order"] == sk.SK_SEGMENTS_K_ALIGNED        # the library's default
        assert sk.sk_plan_info(p)["batch_order"] == sk.SK_STREAMK_FIRST and sk.sk_plan_info(p)["fixup"] == sk.SK_FIXUP_FLAGS
        if dp_first:
            sk.sk_plan_set_batch_order(p, sk.SK_DATA_PARALLEL_FIRST)
        if k_aligned is not None:
            sk.sk_plan_set_segment_order(p, sk.SK_SEGMENTS_K_ALIGNED if k_aligned else sk.SK_SEGMENTS_ASCENDING)
        else:
            k_aligned = True
        info = sk.sk_plan_info(p)
        assert info["segment_order"] == int(k_aligned) and info["batch_order"] == int(dp_first)
        o = S.plan(M, N, K, policy, *blk, g, order=info["tile_order"], dp_first=dp_first, k_aligned=k_aligned)
        step = max(1, info["tiles"] // 500)
        for t in list(range(0, info["tiles"], step)) + [info["tiles"] - 1]:
            assert sk.sk_plan_tile_coords(p, t) == S.tile_coords(t, info["tiles_m"], info["tiles_n"], info["tile_order"])
        return info, sk.sk_plan_ranges(p), sk.sk_plan_segments(p), o
    finally:
        sk.sk_plan_destroy(p)


def _assert_same(info, ranges, segs, o):
    for key in ("tiles_m", "tiles_n", "tiles", "iters_per_tile", "total_iters", "sk_tiles", "dp_tiles",
                "sk_iters", "iters_per_wg", "dp_waves", "grid", "blk_m", "blk_n", "blk_k", "policy", "tile_order"):
        assert info[key] == o.header[key], key
    assert ranges == [tuple(r) for r in o.ranges]
    assert segs == [tuple(s) for s in o.segments]


@settings(max_examples=400, deadline=None)
@given(st.tuples(st.integers(1, 3000), st.integers(1, 3000), st.integers(1, 5000)),
       st.tuples(st.sampled_from([16, 32, 64, 128, 256]), st.sampled_from([16, 64, 128, 256]),
                 st.sampled_from([8, 32, 64, 128])),
       st.sampled_from([1, 2, 3, 7, 8, 64, 104, 256, 304]), st.integers(0, 7))
def test_schedule_bit_exact_random(shape, blk, g, policy):
    _assert_same(*_plan_pair(*shape, policy, blk, g, order=(shape[0] + policy) % 2, dp_first=shape[1] % 3 == 0,
                             k_aligned=shape[2] % 2 == 0))


@pytest.mark.parametrize("policy", range(8))
@pytest.mark.parametrize("shape,blk", [((512, 512, 512), (128, 128, 32)),
                                       ((3840, 4224, 4096), (256, 128, 32)),
                                       ((3840, 4224, 4096), (256, 128, 64)),
                                       ((16, 8192, 8192), (16, 128, 64)),
                                       ((128, 8192, 8192), (128, 128, 64)),
                                       ((8192, 8192, 8192), (256, 256, 64)),
                                       ((1, 64, 65536), (16, 128, 64)),
                                       ((16384, 16384, 16384), (256, 256, 64))])
def test_schedule_bit_exact_benchmark_configs(shape, blk, policy):
    _assert_same(*_plan_pair(*shape, policy, blk, 256))


def test_plan_defaults_and_errors():
    p = sk.sk_plan(8192, 8192, 8192, sk.SK_POLICY_DP)
    info = sk.sk_plan_info(p)
    assert (info["grid"], info["in_dtype"], info["out_dtype"]) == (256, sk.SK_BF16, sk.SK_BF16)
    # 32 x 32 tiles: an XCD's 32 tiles are one tile row (1 + 32 operand blocks) or an 8 x 4 block (8 + 4)
    assert info["tile_order"] == sk.SK_ORDER_GROUPED
    q = sk.sk_plan(8192, 8192, 8192, sk.SK_POLICY_ALL_SK)
    assert sk.sk_plan_info(q)["tile_order"] == sk.SK_ORDER_GROUPED         # the choice does not depend on the policy
    sk.sk_plan_destroy(q)
    # one row of 64 tiles (cfg3): 8 tiles per XCD span 1 row and 8 columns either way -> the plain order;
    # a single row of low tiles keeps the hardware workgroup order, everything else is renumbered per XCD
    q = sk.sk_plan(16, 8192, 8192, sk.SK_POLICY_ALL_SK)
    assert sk.sk_plan_info(q)["tile_order"] == sk.SK_ORDER_ROW_MAJOR and sk.sk_plan_info(q)["xcd_remap"] == 0
    sk.sk_plan_destroy(q)
    assert info["xcd_remap"] == 1
    for shape, blk, remap in (((128, 8192, 8192), (128, 128, 64), 1), ((128, 8192, 8192), (64, 128, 64), 1),
                              ((64, 8192, 8192), (64, 128, 64), 0), ((8192, 128, 8192), (64, 128, 64), 1)):
        q = sk.sk_plan(*shape, sk.SK_POLICY_ALL_SK, blk)
        assert sk.sk_plan_info(q)["xcd_remap"] == remap
        sk.sk_plan_destroy(q)
    # 4 tile rows x 256 tile columns of 256 x 128 tiles: a row-major XCD chunk spans 1 x 32 blocks
    # (256 + 32 * 128 operand rows and columns), a grouped one 4 x 8 (4 * 256 + 8 * 128)
    q = sk.sk_plan(1024, 32768, 4096, sk.SK_POLICY_DP, (256, 128, 64))
    assert sk.sk_plan_info(q)["tile_order"] == sk.SK_ORDER_GROUPED
    sk.sk_plan_destroy(q)
    with pytest.raises(sk.StreamKError):
        sk.sk_plan_tile_coords(p, info["tiles"])
    assert (info["blk_m"], info["blk_n"], info["blk_k"]) == sk.sk_default_tile(8192, 8192, 8192)
    assert info["has_kernel"] == 1
    assert sk.sk_workspace_bytes(p) >= 256 * info["blk_m"] * info["blk_n"] * 4
    sk.sk_plan_destroy(p)
    p = sk.sk_plan(64, 64, 64, 0, in_dtype=sk.SK_FP8_E4M3)
    assert sk.sk_plan_info(p)["out_dtype"] == sk.SK_BF16
    sk.sk_plan_destroy(p)
    for bad in [dict(M=0), dict(policy=8), dict(policy=-1), dict(in_dtype=sk.SK_F32), dict(out_dtype=sk.SK_FP8_E4M3),
                dict(blk=(-1, 16, 16)), dict(grid=-2), dict(tile_order=2)]:
        args = dict(M=64, N=64, K=64, policy=0)
        args.update(bad)
        with pytest.raises(sk.StreamKError) as e:
            sk.sk_plan(**args)
        assert e.value.status == sk.SK_ERR_INVALID_ARG
    assert sk.sk_workspace_bytes(None) == 0
    assert sk.sk_status_str(sk.SK_ERR_WORKSPACE).startswith("workspace")


def test_gemm_rejects_bad_arguments_without_touching_the_gpu():
    p = sk.sk_plan(512, 512, 512, sk.SK_POLICY_ALL_SK, (128, 128, 32))
    assert sk.sk_gemm_status(0, 256, 512, p) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_gemm_status(256, 512, 768, None) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_gemm_status(256, 520, 768, p) == sk.SK_ERR_INVALID_ARG          # misaligned B
    assert sk.sk_gemm_status(256, 512, 768, p) == sk.SK_ERR_WORKSPACE            # split tiles, no workspace
    sk.sk_plan_destroy(p)
    p = sk.sk_plan(512, 512, 512, sk.SK_POLICY_DP, (48, 48, 16))
    assert sk.sk_plan_info(p)["has_kernel"] == 0
    assert sk.sk_gemm_status(256, 512, 768, p) == sk.SK_ERR_UNSUPPORTED
    sk.sk_plan_destroy(p)


def test_gemm_rejects_sizes_beyond_the_kernels_index_range():
    # the kernels index A and B with 32-bit byte offsets and D with 32-bit element offsets; larger
    # problems are refused up front (planning them is still allowed)
    for M, N, K in ((1 << 16, 64, 1 << 15), (64, 1 << 16, 1 << 15), (1 << 16, 1 << 16, 64)):
        p = sk.sk_plan(M, N, K, sk.SK_POLICY_DP)
        assert sk.sk_plan_info(p)["tiles"] >= 1
        assert sk.sk_gemm_status(256, 512, 768, p) == sk.SK_ERR_UNSUPPORTED
        sk.sk_plan_destroy(p)
    # just inside the range: gets as far as the workspace check (the plan splits tiles), nothing is launched
    p = sk.sk_plan((1 << 16) - 16, 64, (1 << 14) + 64, sk.SK_POLICY_ALL_SK, (256, 128, 64), 250)
    assert any(seg[4] != sk.SK_ROLE_FULL for seg in sk.sk_plan_segments(p))
    assert sk.sk_gemm_status(256, 512, 768, p) == sk.SK_ERR_WORKSPACE
    sk.sk_plan_destroy(p)


def test_fixup_mode_setter_and_workspace_need():
    import ctypes
    lib = sk.binding._lib
    assert lib.sk_plan_set_batch_order(None, 0) == sk.SK_ERR_INVALID_ARG
    assert lib.sk_plan_set_segment_order(None, 0) == sk.SK_ERR_INVALID_ARG
    p = sk.sk_plan(512, 384, 512, sk.SK_POLICY_ALL_SK, (128, 128, 32), 256, sk.SK_F16)
    flags_bytes = sk.sk_workspace_bytes(p)
    assert flags_bytes >= 256 * 128 * 128 * 4
    assert lib.sk_plan_set_fixup(p, 2) == sk.SK_ERR_INVALID_ARG
    assert lib.sk_plan_set_batch_order(p, 2) == sk.SK_ERR_INVALID_ARG
    assert lib.sk_plan_set_segment_order(p, 2) == sk.SK_ERR_INVALID_ARG
    assert lib.sk_plan_set_fixup(None, 0) == sk.SK_ERR_INVALID_ARG
    sk.sk_plan_set_fixup(p, sk.SK_FIXUP_ATOMIC)
    # atomic mode with a 16-bit output: flag / status lines + an fp32 image of D
    assert sk.sk_workspace_bytes(p) == flags_bytes - 256 * 128 * 128 * 4 + 512 * 384 * 4
    assert sk.sk_gemm_status(256, 512, 768, p) == sk.SK_ERR_WORKSPACE            # image lives in the workspace
    sk.sk_plan_set_fixup(p, sk.SK_FIXUP_FLAGS)
    assert sk.sk_workspace_bytes(p) == flags_bytes
    sk.sk_plan_destroy(p)
    # fp32 output: D itself is accumulated into, no image in the workspace
    p = sk.sk_plan(512, 384, 512, sk.SK_POLICY_ALL_SK, (128, 128, 32), 256, sk.SK_F16, sk.SK_F32)
    sk.sk_plan_set_fixup(p, sk.SK_FIXUP_ATOMIC)
    assert sk.sk_workspace_bytes(p) == flags_bytes - 256 * 128 * 128 * 4
    sk.sk_plan_destroy(p)


def test_kernel_info_names_the_kernel_of_a_launch():
    lib = sk.binding._lib
    assert lib.sk_plan_kernel_info(None, None, None, None) == sk.SK_ERR_INVALID_ARG
    assert lib.sk_plan_set_kernel_variant(None, 1) == sk.SK_ERR_INVALID_ARG
    expect = {(256, 256, 64): 512, (256, 128, 64): 512, (128, 128, 64): 512, (64, 128, 64): 512, (32, 128, 64): 256, (16, 128, 64): 256}
    for blk, threads in expect.items():
        p = sk.sk_plan(1000, 1000, 1000, sk.SK_POLICY_ALL_SK, blk, 256, sk.SK_BF16)
        info = sk.sk_plan_kernel_info(p)
        assert info["variant"] == 0 and info["threads"] == threads and 0 < info["lds_bytes"] <= 160 * 1024
        assert lib.sk_plan_kernel_info(p, None, None, None) == sk.SK_OK
        assert lib.sk_plan_set_kernel_variant(p, -1) == sk.SK_ERR_INVALID_ARG
        sk.sk_plan_set_kernel_variant(p, 1)                        # a 4-wave layout where the tile has one
        alt = sk.sk_plan_kernel_info(p)
        assert (alt["variant"], alt["threads"]) == ((1, 256) if blk[0] >= 64 else (0, threads))
        sk.sk_plan_set_fixup(p, sk.SK_FIXUP_ATOMIC)                # the atomic set has no variants
        assert sk.sk_plan_kernel_info(p)["variant"] == 0
        sk.sk_plan_destroy(p)
    # a plan without split tiles on the 256 x 256 tile: the library itself takes the four-wave kernel
    for dt, blk in ((sk.SK_BF16, (256, 256, 64)), (sk.SK_FP8_E4M3, (256, 256, 128))):
        p = sk.sk_plan(1024, 1024, 512, sk.SK_POLICY_DP, blk, 256, dt)       # 8 (4) k-iterations per tile: too shallow for it
        assert sk.sk_plan_kernel_info(p)["threads"] == 512
        sk.sk_plan_destroy(p)
        p = sk.sk_plan(1024, 1024, 6144, sk.SK_POLICY_DP, blk, 256, dt)
        info = sk.sk_plan_kernel_info(p)
        assert (info["variant"], info["threads"]) == (1, 256)
        sk.sk_plan_set_kernel_variant(p, 3)                            # the eight-wave kernel, whatever the plan
        info = sk.sk_plan_kernel_info(p)
        assert (info["variant"], info["threads"]) == (3, 512)
        sk.sk_plan_destroy(p)
        p = sk.sk_plan(1000, 1000, 1000, sk.SK_POLICY_ALL_SK, blk, 256, dt)     # split tiles: eight waves
        assert sk.sk_plan_kernel_info(p)["threads"] == 512
        sk.sk_plan_destroy(p)
    p = sk.sk_plan(1000, 1000, 1000, sk.SK_POLICY_DP, (64, 64, 64), 256, sk.SK_BF16)   # a tile without a kernel
    assert lib.sk_plan_kernel_info(p, None, None, None) == sk.SK_ERR_UNSUPPORTED
    sk.sk_plan_destroy(p)


# ---- Bloom -----------------------------------------------------------------------------------

def test_hash_bit_exact_with_oracle():
    rng = random.Random(5)
    for _ in range(3000):
        key = bytes(rng.getrandbits(8) for _ in range(rng.randint(0, 33)))
        seed = rng.getrandbits(32)
        assert sk.bloom_murmur3_32(key, seed) == Bm.murmur3_32(key, seed)


def _records(n, seed):
    rng = random.Random(seed)
    return [(16 * rng.randint(1, 1024), 16 * rng.randint(1, 1024), 16 * rng.randint(1, 4096), rng.randint(0, 127))
            for _ in range(n)]


@pytest.mark.parametrize("params", [(0, 0, 0), (1024, 3, 7), (64, 1, 2), (95872, 7, 7)])
def test_bloom_bits_and_queries_bit_exact_with_oracle(params):
    recs = _records(923, 7)
    b = sk.bloom_build(recs, *params)
    o = Bm.build(recs, *(p or d for p, d in zip(params, (Bm.M_BITS, Bm.K_PROBES, Bm.N_FILTERS))))
    for f in range(o.n_filters):
        assert sk.bloom_bits(b, f) == o.words[f]
    rng = random.Random(8)
    probes = [r[:3] for r in recs[:200]] + [(rng.randint(1, 70000), rng.randint(1, 70000), rng.randint(1, 70000)) for _ in range(800)]
    for M, N, K in probes:
        assert sk.bloom_query(b, M, N, K) == o.query(M, N, K)
    for M, N, K, mask in recs:                                   # no false negatives
        assert sk.bloom_query(b, M, N, K) & mask == mask & ((1 << o.n_filters) - 1)
    sk.bloom_destroy(b)


@pytest.mark.parametrize("params", [(0, 0, 0), (640, 3, 5)])
def test_bloom_serialised_filters_round_trip_bit_exact(params):
    # the byte string holds exactly the oracle's words (little-endian, filter by filter) behind a 20-byte
    # header, and filters rebuilt from it answer like the oracle
    recs = _records(300, 11)
    b = sk.bloom_build(recs, *params)
    o = Bm.build(recs, *(p or d for p, d in zip(params, (Bm.M_BITS, Bm.K_PROBES, Bm.N_FILTERS))))
    data = sk.bloom_serialize(b)
    assert len(data) == 20 + o.n_filters * o.m_bits // 8
    assert data[:4] == b"SKBF" and int.from_bytes(data[4:8], "little") == 1
    assert [int.from_bytes(data[8 + 4 * i:12 + 4 * i], "little") for i in range(3)] == [o.m_bits, o.k_probes, o.n_filters]
    body = b"".join(w.to_bytes(8, "little") for f in range(o.n_filters) for w in o.words[f])
    assert data[20:] == body
    c = sk.bloom_deserialize(data)
    for f in range(o.n_filters):
        assert sk.bloom_bits(c, f) == o.words[f]
    rng = random.Random(12)
    for M, N, K in [r[:3] for r in recs[:100]] + [(rng.randint(1, 70000), rng.randint(1, 70000), rng.randint(1, 70000)) for _ in range(300)]:
        assert sk.bloom_query(c, M, N, K) == o.query(M, N, K)
    lib = sk.binding._lib
    out, n = ctypes.c_void_p(), ctypes.c_size_t()
    bad = [data[:-1], data + b"x", b"XKBF" + data[4:], data[:4] + (2).to_bytes(4, "little") + data[8:],
           data[:8] + (65).to_bytes(4, "little") + data[12:], data[:19]]
    for d in bad:
        buf = (ctypes.c_ubyte * len(d)).from_buffer_copy(d)
        assert lib.bloom_deserialize(buf, len(d), ctypes.byref(out)) == sk.SK_ERR_INVALID_ARG and not out.value
    small = (ctypes.c_ubyte * 16)()
    assert lib.bloom_serialize(b, small, 16, ctypes.byref(n)) == sk.SK_ERR_INVALID_ARG and n.value == len(data)
    assert lib.bloom_serialize(None, None, 0, ctypes.byref(n)) == sk.SK_ERR_INVALID_ARG
    sk.bloom_destroy(b)
    sk.bloom_destroy(c)


@settings(max_examples=200, deadline=None)
@given(st.tuples(st.integers(1, 20000), st.integers(1, 20000), st.integers(1, 70000)),
       st.sampled_from([(256, 256, 64), (128, 128, 64), (32, 128, 64), (16, 128, 32)]),
       st.sampled_from([7, 104, 256]))
def test_shape_key_bit_exact_with_oracle(shape, blk, g):
    p = sk.sk_plan(*shape, 0, blk, g)
    o = S.plan(*shape, 0, *blk, g)
    assert sk.bloom_shape_key(p) == Bm.shape_key(o.header)
    sk.sk_plan_destroy(p)


def test_shape_key_values_by_hand():
    # 3840 x 4224 x 4096 at 256 x 128 x 64 on 256 workgroups: 495 tiles = 1 full wave + 239 tiles
    # (239 / 256 -> 4 quarters), 64 iterations per tile -> log2 = 6
    p = sk.sk_plan(3840, 4224, 4096, 0, (256, 128, 64), 256)
    assert sk.bloom_shape_key(p) == (256 << 16 | 128, 1 << 8 | 4, 6 << 16 | 64)
    sk.sk_plan_destroy(p)
    # 8192^3 at 256 x 256 x 64: 1024 tiles = 4 waves (capped at 3), no remainder, 128 iterations -> 7
    p = sk.sk_plan(8192, 8192, 8192, 0, (256, 256, 64), 256)
    assert sk.bloom_shape_key(p) == (256 << 16 | 256, 3 << 8 | 0, 7 << 16 | 64)
    sk.sk_plan_destroy(p)


def test_bloom_insert_after_build_and_errors():
    b = sk.bloom_build([])
    assert sk.bloom_query(b, 512, 512, 512) == 0
    sk.bloom_insert(b, 512, 512, 512, 0b1000001)
    assert sk.bloom_query(b, 512, 512, 512) == 0b1000001
    o = Bm.build([(512, 512, 512, 0b1000001)])
    assert all(sk.bloom_bits(b, f) == o.words[f] for f in range(7))
    with pytest.raises(sk.StreamKError):
        sk.bloom_query(b, -1, 2, 3)
    with pytest.raises(sk.StreamKError):
        sk.bloom_query(b, 2 ** 32, 2, 3)
    with pytest.raises(sk.StreamKError):
        sk.bloom_bits(b, 7)
    sk.bloom_destroy(b)
    with pytest.raises(sk.StreamKError):
        sk.bloom_build([], 100, 7, 7)                             # not a multiple of 64


def test_plan_estimate_properties():
    def est(M, N, K, policy, blk, grid=256, dtype=sk.SK_BF16):
        p = sk.sk_plan(M, N, K, policy, blk, grid, dtype, sk.SK_BF16)
        try:
            return sk.sk_plan_estimate_us(p)
        finally:
            sk.sk_plan_destroy(p)
    blk = (256, 256, 64)
    one = est(4096, 4096, 4096, sk.SK_POLICY_DP, blk)                 # 256 tiles: one wave
    two = est(8192, 4096, 4096, sk.SK_POLICY_DP, blk)                 # 512 tiles: two waves
    assert one > 0 and abs(two - 2 * one) < 1e-9 * two
    for policy in range(1, 7):                                       # whole waves: every policy is the same schedule
        assert abs(est(8192, 4096, 4096, policy, blk) - two) < 1e-6 * two
    # 257 tiles: the second, almost empty wave costs the data-parallel policy a whole tile time; a
    # Stream-K batch over the 257 tiles (SK2_DP here) costs one iteration more per workgroup plus an exchange
    dp = est(4096 + 256, 4096, 4096, sk.SK_POLICY_DP, (256, 256, 64))   # 17 x 16 = 272 tiles
    sk2 = est(4096 + 256, 4096, 4096, sk.SK_POLICY_SK2_DP, (256, 256, 64))
    assert dp > 1.9 * one and one < sk2 < 0.75 * dp
    # 210 tiles of 256 x 256 over a short K: splitting saves a sixth of the iterations, but 250 workgroups
    # then park and fetch a 256 KB partial tile each - measured 99 us against 64 us data-parallel
    assert est(2560, 5280, 2160, sk.SK_POLICY_DP, blk) < est(2560, 5280, 2160, sk.SK_POLICY_ALL_SK, blk)
    # ... while small tiles over a long K gain from the split (48 tiles of 32 x 128: 7.4 us against 9.0 us is
    # a tie for the model, 128 iterations per tile are not)
    assert est(512, 272, 8192, sk.SK_POLICY_ALL_SK, (32, 128, 64)) < est(512, 272, 8192, sk.SK_POLICY_DP, (32, 128, 64))
    # longer K costs more, bigger tiles cost more per tile
    assert est(4096, 4096, 8192, 0, blk) > one and est(4096, 4096, 4096, 0, (128, 128, 64)) > 0
    p = sk.sk_plan(4096, 4096, 4096, 0, (256, 256, 128), 256, sk.SK_FP8_E4M3, sk.SK_BF16)
    us = ctypes.c_double()
    lib = sk.binding._lib
    # 8-bit tiles are modelled as the 16-bit shape of the same footprint with half the blk_k: same time per iteration
    assert lib.sk_plan_estimate_us(p, ctypes.byref(us)) == sk.SK_OK
    assert abs(us.value - est(4096, 4096, 2048, 0, blk)) < 1e-9 * us.value
    q = sk.sk_plan(4096, 4096, 4096, 0, (64, 64, 64), 256, sk.SK_BF16)          # a shape without constants
    assert lib.sk_plan_estimate_us(q, ctypes.byref(us)) == sk.SK_ERR_UNSUPPORTED
    sk.sk_plan_destroy(q)
    assert lib.sk_plan_estimate_us(p, None) == sk.SK_ERR_INVALID_ARG and lib.sk_plan_estimate_us(None, ctypes.byref(us)) == sk.SK_ERR_INVALID_ARG
    sk.sk_plan_destroy(p)
    p = sk.sk_plan(512, 512, 512, 0, (128, 128, 32), 256, sk.SK_F16, sk.SK_F16)   # blk_k = 32: the per-iteration time scales with blk_k
    assert sk.sk_plan_estimate_us(p) > 0
    sk.sk_plan_destroy(p)


def test_seeded_suites_are_reproducible_and_in_range():
    from paper_2408_11417_amd import inputs
    a, b = inputs.sweep_shapes(500, 4), inputs.sweep_shapes(500, 4)
    assert a == b and len(a) == 500
    assert all(64 <= d <= 16384 and d % 16 == 0 for s in a for d in s)
    p = inputs.paper_suite()
    assert p == inputs.paper_suite() and len(p) == 923 and len(set(p)) == 923
    for M, N, K in p:                                     # powers of two inside the ranges of Sec. 5.1
        assert all(d & (d - 1) == 0 for d in (M, N, K))
        assert 1 <= M <= 8192 and 64 <= N <= 8192 and 16 <= K <= 65536
    assert len(inputs.paper_suite(1456)) == 1456 == len(set(inputs.paper_suite(1456)))      # the whole grid


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "--gpus must be 1" in (res.stderr + res.stdout)
