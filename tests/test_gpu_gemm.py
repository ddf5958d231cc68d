"""Parity of the HIP Stream-K GEMM (through the C ABI) with the CPU oracle, on a real MI355X.

Tolerances (the benchmark spec): max relative error <= 1e-2 with fp16 / bf16 output and
<= 1e-4 on the fp32-accumulator output, with err = max |d - ref| / max(|ref|, rms(ref)).
Integer-valued inputs are exact in fp32 under every schedule, so they are compared bit-exactly.
"""
import numpy as np
import pytest
import torch

import paper_2408_11417_amd as sk
from paper_2408_11417_amd import inputs
from oracle import gemm as G
from oracle import schedule as S
from tests.gpu_util import Runner, to_device

pytestmark = pytest.mark.gpu
TOL_16, TOL_32 = 1e-2, 1e-4
ODT = {inputs.F16: G.F16, inputs.BF16: G.BF16, inputs.E4M3: G.E4M3}


def _run_and_compare(A, B, dtype, policy, blk, grid=256, out_dtype=None, rows=None, ref=None, exact=False,
                     fixup=sk.SK_FIXUP_FLAGS, launches=1, dp_first=False, k_aligned=True, variant=0):
    M, K = A.shape
    N = B.shape[1]
    print("case M=%d N=%d K=%d dtype=%d policy=%s blk=%s grid=%d out=%s fixup=%d dp_first=%d k_aligned=%d" %
          (M, N, K, dtype, sk.POLICY_NAMES[policy], blk, grid, out_dtype, fixup, dp_first, k_aligned), flush=True)
    r = Runner(M, N, K, policy, blk, grid, dtype, out_dtype, fixup=fixup, dp_first=dp_first, k_aligned=k_aligned, variant=variant)
    try:
        # the library's schedule for this very launch equals the oracle's
        o = S.plan(M, N, K, policy, r.info["blk_m"], r.info["blk_n"], r.info["blk_k"], r.info["grid"], r.info["tile_order"],
                   dp_first=dp_first, k_aligned=k_aligned)
        assert sk.sk_plan_segments(r.plan) == [tuple(s) for s in o.segments]
        assert r.info["segment_order"] == int(k_aligned) and r.info["batch_order"] == int(dp_first) and r.info["fixup"] == fixup
        dA, dB = to_device(A), to_device(B)
        for _ in range(launches):
            r.run(dA, dB)
        assert r.check() == sk.SK_OK
        d = r.result()
    finally:
        r.close()
    if ref is None:
        ref = G.gemm_fp64(A, B, ODT[dtype], rows=rows)
    if rows is not None:
        d = d[rows]
    if exact:
        assert np.array_equal(d, ref)
        return 0.0
    err = G.rel_error(d, ref)
    tol = TOL_32 if out_dtype == sk.SK_F32 else TOL_16
    assert err <= tol, "rel err %.3e > %.1e" % (err, tol)
    return err


@pytest.mark.parametrize("policy", range(8))
def test_config1_fp16_512_all_policies(policy):
    c = inputs.config1()
    ref = G.gemm_fp64(c["A"], c["B"], G.F16)
    _run_and_compare(c["A"], c["B"], inputs.F16, policy, c["blk"], c["grid"], ref=ref)
    _run_and_compare(c["A"], c["B"], inputs.F16, policy, c["blk"], c["grid"], out_dtype=sk.SK_F32, ref=ref)


TILES = [(128, 128, 32, 4), (128, 128, 64, 4), (256, 128, 64, 4), (256, 256, 64, 8), (64, 128, 64, 4),
         (32, 128, 64, 4), (16, 128, 64, 4)]


@pytest.mark.parametrize("dtype", [inputs.BF16, inputs.F16])
@pytest.mark.parametrize("blk", [t[:3] for t in TILES])
def test_integer_inputs_bit_exact_every_tile_and_policy(blk, dtype):
    # several tiles in each direction plus a ragged tail; grid 24 so that tiles are split unevenly
    M, N, K = 2 * blk[0] + 40, 3 * blk[1] + 72, 5 * blk[2] + 24
    A, B = inputs.small_int_pair(M, N, K, dtype, 21)
    ref = G.gemm_fp64(A, B, ODT[dtype])
    for policy in range(8):
        _run_and_compare(A, B, dtype, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True)


# wave layouts that are compiled in beside the default one of their tile (4 waves as 2 x 2; for the
# 256 x 256 tile also the 8-wave kernel with the coarser MAC loop), chosen with sk_plan_set_kernel_variant
VARIANT_TILES = [(1, (256, 128, 64)), (1, (256, 256, 64)), (1, (128, 128, 64)), (1, (64, 128, 64)), (2, (256, 256, 64)), (3, (256, 256, 64)),
                 (3, (256, 128, 64)), (3, (128, 128, 64))]


@pytest.mark.parametrize("variant,blk", VARIANT_TILES)
def test_alternative_wave_layouts_integer_exact(variant, blk):
    r = Runner(512, 512, 512, sk.SK_POLICY_DP, blk, 24, inputs.BF16, sk.SK_F32, variant=variant)
    info = sk.sk_plan_kernel_info(r.plan)
    r.close()
    assert info["variant"] == variant and info["threads"] == (256 if variant == 1 else 512)
    M, N, K = 2 * blk[0] + 40, 3 * blk[1] + 72, 5 * blk[2] + 24
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 24)
    ref = G.gemm_fp64(A, B, G.BF16)
    for policy in range(8):
        _run_and_compare(A, B, inputs.BF16, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True, variant=variant)
    A, B = inputs.uniform_pair(M, N, K, inputs.F16, 25)        # 16-bit epilogue, aligned and unaligned rows
    _run_and_compare(A, B, inputs.F16, sk.SK_POLICY_ALL_SK, blk, grid=24, variant=variant)
    A, B = inputs.uniform_pair(M + 3, N + 5, K + 1, inputs.BF16, 26)
    _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_SK1_DP, blk, grid=24, variant=variant)


@pytest.mark.parametrize("blk,variant", [((128, 128, 64), 0), ((128, 128, 64), 1), ((256, 256, 64), 3), ((256, 256, 64), 1),
                                         ((256, 128, 64), 0), ((32, 128, 64), 0), ((16, 128, 64), 0), ((128, 128, 32), 0)])
def test_many_interior_tiles_per_workgroup_short_k(blk, variant):
    # eight whole interior tiles per workgroup, one after the other, with 1, 2, 3 and 5 k-iterations each: the first
    # requests of a tile go out before the previous tile's epilogue, and the first wait of its MAC loop leaves
    # that epilogue's stores in flight - for every depth of the start-up of the ring, 16-bit and fp32 output
    M, N = 4 * blk[0], 16 * blk[1]
    for iters in (1, 2, 3, 5):
        K = iters * blk[2]
        A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 90 + iters)
        ref = G.gemm_fp64(A, B, G.BF16)
        for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_SK2_DP):
            _run_and_compare(A, B, inputs.BF16, policy, blk, grid=8, out_dtype=sk.SK_F32, ref=ref, exact=True, variant=variant, launches=2)
        _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_DP, blk, grid=8, ref=ref, variant=variant)            # bf16 output


@pytest.mark.parametrize("blk,variant", [((256, 256, 128), 1), ((256, 256, 128), 3), ((128, 256, 128), 0)])
def test_many_interior_tiles_per_workgroup_short_k_fp8(blk, variant):
    M, N = 4 * blk[0], 8 * blk[1]
    for iters in (1, 2, 3, 5):
        K = iters * blk[2]
        A, B = inputs.small_int_pair(M, N, K, inputs.E4M3, 95 + iters)
        ref = G.gemm_fp64(A, B, G.E4M3)
        _run_and_compare(A, B, inputs.E4M3, sk.SK_POLICY_DP, blk, grid=8, out_dtype=sk.SK_F32, ref=ref, exact=True, variant=variant, launches=2)
        _run_and_compare(A, B, inputs.E4M3, sk.SK_POLICY_SK1_DP, blk, grid=8, ref=ref, variant=variant)        # bf16 output


@pytest.mark.parametrize("shape", [(77, 101, 203), (1, 64, 16), (5, 7, 3), (130, 129, 1), (300, 8, 2049), (16, 264, 520)])
def test_ragged_and_unaligned_shapes(shape):
    M, N, K = shape
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 22)
    ref = G.gemm_fp64(A, B, G.BF16)
    for blk in [(128, 128, 32), (16, 128, 64), (64, 128, 64)]:
        for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
            _run_and_compare(A, B, inputs.BF16, policy, blk, grid=16, out_dtype=sk.SK_F32, ref=ref, exact=True)
    A, B = inputs.uniform_pair(M, N, K, inputs.F16, 23)
    _run_and_compare(A, B, inputs.F16, sk.SK_POLICY_ALL_SK, (128, 128, 32), grid=256)


def test_bit_identical_run_to_run_and_flag_reuse():
    c = inputs.config1()
    dA, dB = to_device(c["A"]), to_device(c["B"])
    r = Runner(512, 512, 512, sk.SK_POLICY_ALL_SK, c["blk"], 256, inputs.F16, sk.SK_F32)
    first = r.run(dA, dB).clone()
    for i in range(30):                      # same workspace and flags, back to back on one stream
        D = r.run(dA, dB)
        if i % 10 == 9:
            assert torch.equal(D, first)
    assert r.check() == sk.SK_OK
    # another plan sharing nothing but the stream, interleaved
    r2 = Runner(512, 512, 512, sk.SK_POLICY_SK2_DP, (128, 128, 64), 256, inputs.F16, sk.SK_F32)
    for _ in range(5):
        r2.run(dA, dB)
        assert torch.equal(r.run(dA, dB), first)
    ref = G.gemm_fp64(c["A"], c["B"], G.F16)
    assert G.rel_error(r2.result(), ref) <= TOL_32
    r.close()
    r2.close()


def test_flag_exchange_soak_two_plans_one_workspace():
    """2000 launches on one stream alternating a plan whose tiles are reduced flat (15 contributors) and
    one reduced in two levels (about 60 per tile), both on the same workspace memory: every result must
    be bit-identical to the plan's first one and no owner may time out.  Stops at the first failure."""
    c = inputs.config1()
    A2, B2 = inputs.uniform_pair(64, 208, 7872, inputs.BF16, 77)
    dA1, dB1, dA2, dB2 = to_device(c["A"]), to_device(c["B"]), to_device(A2), to_device(B2)
    r1 = Runner(512, 512, 512, sk.SK_POLICY_ALL_SK, c["blk"], 256, inputs.F16, sk.SK_F32)
    r2 = Runner(64, 208, 7872, sk.SK_POLICY_ALL_SK, (32, 128, 64), 256, inputs.BF16, sk.SK_F32)
    try:
        # one workspace for both plans (the larger need), as a serving loop would hold it
        need = max(sk.sk_workspace_bytes(r1.plan), sk.sk_workspace_bytes(r2.plan))
        ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        base = (ws.data_ptr() + 255) // 256 * 256
        sk.sk_plan_set_workspace(r1.plan, base, need)
        sk.sk_plan_set_workspace(r2.plan, base, need)
        first1, first2 = r1.run(dA1, dB1).clone(), r2.run(dA2, dB2).clone()
        assert r1.check() == sk.SK_OK and r2.check() == sk.SK_OK
        assert G.rel_error(r1.result(first1), G.gemm_fp64(c["A"], c["B"], G.F16)) <= TOL_32
        assert G.rel_error(r2.result(first2), G.gemm_fp64(A2, B2, G.BF16)) <= TOL_32
        for i in range(1000):
            d1 = r1.run(dA1, dB1)
            d2 = r2.run(dA2, dB2)
            if i % 8 == 7 or i == 999:            # compare (and with it synchronise) every eighth pair; the launches in between queue up back to back
                assert torch.equal(d1, first1), "flat plan differs at launch pair %d" % i
                assert torch.equal(d2, first2), "two-level plan differs at launch pair %d" % i
                assert r1.check() == sk.SK_OK and r2.check() == sk.SK_OK, "time-out at launch pair %d" % i
            else:
                d1.fill_(0)                        # so that a launch that stores nothing cannot pass
                d2.fill_(0)
    finally:
        r1.close()
        r2.close()


def test_owner_timeout_is_reported_and_every_wave_exits():
    c = inputs.config1()
    dA, dB = to_device(c["A"]), to_device(c["B"])
    r = Runner(512, 512, 512, sk.SK_POLICY_ALL_SK, c["blk"], 256, inputs.F16, sk.SK_F32)
    sk.sk_plan_set_spin_limit(r.plan, 0)     # owners give up at the first unsuccessful poll
    r.run(dA, dB)
    st = r.check()                           # the launch must come back either way
    assert st in (sk.SK_OK, sk.SK_ERR_TIMEOUT)
    ref = G.gemm_fp64(c["A"], c["B"], G.F16)
    if st == sk.SK_OK:
        assert G.rel_error(r.result(), ref) <= TOL_32
    sk.sk_plan_set_spin_limit(r.plan, 1 << 24)
    r.run(dA, dB)
    assert r.check() == sk.SK_OK             # status word was cleared by the previous check
    assert G.rel_error(r.result(), ref) <= TOL_32
    r.close()


@pytest.mark.parametrize("policy", range(7))
def test_config2_wave_quantisation_sampled_rows(policy):
    c = inputs.config2()
    rows = inputs.sample_rows(c["M"], 48, 100 + policy)
    _run_and_compare(c["A"], c["B"], inputs.BF16, policy, c["blk"], 256, rows=rows)


@pytest.mark.parametrize("M", [16, 32, 64, 128])
def test_config3_skinny(M):
    c = inputs.config3(M)
    ref = G.gemm_fp64(c["A"], c["B"], G.BF16)
    for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(c["A"], c["B"], inputs.BF16, policy, None, 256, ref=ref)
    _run_and_compare(c["A"], c["B"], inputs.BF16, sk.SK_POLICY_ALL_SK, None, 256, out_dtype=sk.SK_F32, ref=ref)
    if M == 16:
        # B is 128 MiB and read once here: the launches above and these request it non-temporally; the
        # lowest tile and the four-wave 64-row kernel take that path too
        _run_and_compare(c["A"], c["B"], inputs.BF16, sk.SK_POLICY_ALL_SK, (16, 128, 64), 256, ref=ref)
        _run_and_compare(c["A"], c["B"], inputs.BF16, sk.SK_POLICY_DP, (64, 128, 64), 256, ref=ref, variant=1)
        A, B = inputs.small_int_pair(16, 8192, 8192, inputs.BF16, 77, lo=-2, hi=2)
        _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_SK2_DP, None, 256, out_dtype=sk.SK_F32, exact=True)


def _config5_all_policies(dtype):
    # every one of the 32 tile rows (256 rows each) is sampled three times - its first row, a row in the
    # lower wave's half, a random one - and every column of those rows is compared; all seven policies
    c = inputs.config5(dtype)
    rows = inputs.sample_rows_per_band(c["M"], 256, 3, 5 + dtype)
    assert len(set(rows // 256)) == 32 and len(set(rows // 128)) >= 60
    ref = G.gemm_fp64(c["A"], c["B"], ODT[dtype], rows=rows)
    for policy in range(7):
        _run_and_compare(c["A"], c["B"], dtype, policy, None, 256, rows=rows, ref=ref)
    _run_and_compare(c["A"], c["B"], dtype, sk.SK_POLICY_SK3_DP, None, 256, out_dtype=sk.SK_F32, rows=rows, ref=ref)


def test_config5_large_square_bf16_all_policies_every_tile_row():
    _config5_all_policies(inputs.BF16)


# ---- 8-bit (e4m3) inputs ---------------------------------------------------------------------------

@pytest.mark.parametrize("blk", [(256, 256, 128), (128, 256, 128)])
def test_fp8_integer_inputs_bit_exact(blk):
    M, N, K = 2 * blk[0] + 40, 2 * blk[1] + 80, 3 * blk[2] + 48
    A, B = inputs.small_int_pair(M, N, K, inputs.E4M3, 31)
    ref = G.gemm_fp64(A, B, G.E4M3)
    for policy in range(8):
        _run_and_compare(A, B, inputs.E4M3, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True)
    if blk[0] == 256:       # the four-wave kernel (the library's choice for plans without split tiles) under every policy
        for policy in range(8):
            _run_and_compare(A, B, inputs.E4M3, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True, variant=1)
        _run_and_compare(A, B, inputs.E4M3, sk.SK_POLICY_ALL_SK, blk, grid=24, ref=ref, variant=1)      # bf16 output
    # unaligned K and N take the element-wise guarded path
    A, B = inputs.small_int_pair(70, 300, 203, inputs.E4M3, 32)
    ref = G.gemm_fp64(A, B, G.E4M3)
    for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(A, B, inputs.E4M3, policy, blk, grid=16, out_dtype=sk.SK_F32, ref=ref, exact=True)


@pytest.mark.parametrize("blk,shape", [((256, 256, 128), (256, 512, 8448)), ((128, 256, 128), (128, 256, 8704))])
def test_fp8_tiles_shared_by_many_workgroups(blk, shape):
    # 65 and 67 contributors per tile: two-level reduction, block by block for the 256 x 256 tile
    M, N, K = shape
    A, B = inputs.small_int_pair(M, N, K, inputs.E4M3, 34)
    ref = G.gemm_fp64(A, B, G.E4M3)
    for policy in (sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(A, B, inputs.E4M3, policy, blk, grid=256, out_dtype=sk.SK_F32, ref=ref, exact=True, launches=2)
    _run_and_compare(A, B, inputs.E4M3, sk.SK_POLICY_ALL_SK, blk, grid=256, out_dtype=sk.SK_F32, ref=ref, exact=True, k_aligned=False)
    _run_and_compare(A, B, inputs.E4M3, sk.SK_POLICY_ALL_SK, blk, grid=256, ref=ref)          # bf16 output


def test_fp8_uniform_inputs_medium():
    A, B = inputs.uniform_pair(520, 776, 1040, inputs.E4M3, 33)
    ref = G.gemm_fp64(A, B, G.E4M3)
    for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(A, B, inputs.E4M3, policy, None, 256, ref=ref)                       # bf16 output
        _run_and_compare(A, B, inputs.E4M3, policy, None, 256, out_dtype=sk.SK_F32, ref=ref)


def test_config5_large_square_fp8_all_policies_every_tile_row():
    _config5_all_policies(inputs.E4M3)


# ---- atomic-add fix-up (the accumulation step of Algorithm 1): same schedules, partial tiles added into a zeroed fp32 image

@pytest.mark.parametrize("blk", [t[:3] for t in TILES])
def test_atomic_fixup_integer_inputs_bit_exact(blk):
    # integer-valued inputs: every summation order gives the same fp32 result, so the comparison is exact
    # although the order of the atomic adds is not fixed; two launches in a row: the image is cleared each time
    M, N, K = 2 * blk[0] + 40, 3 * blk[1] + 72, 5 * blk[2] + 24
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 22)
    ref = G.gemm_fp64(A, B, G.BF16)
    for policy in (0, 1, 2, 6):
        _run_and_compare(A, B, inputs.BF16, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True,
                         fixup=sk.SK_FIXUP_ATOMIC, launches=2)


@pytest.mark.parametrize("policy", range(7))
def test_atomic_fixup_config1_fp16(policy):
    # 16-bit output goes through the fp32 image in the workspace and the conversion kernel
    c = inputs.config1()
    ref = G.gemm_fp64(c["A"], c["B"], G.F16)
    _run_and_compare(c["A"], c["B"], inputs.F16, policy, c["blk"], c["grid"], ref=ref, fixup=sk.SK_FIXUP_ATOMIC, launches=2)
    _run_and_compare(c["A"], c["B"], inputs.F16, policy, c["blk"], c["grid"], out_dtype=sk.SK_F32, ref=ref,
                     fixup=sk.SK_FIXUP_ATOMIC)


@pytest.mark.parametrize("shape", [(77, 101, 203), (1, 64, 16), (130, 129, 1), (300, 8, 2049), (333, 515, 777)])
def test_atomic_fixup_ragged_shapes(shape):
    M, N, K = shape
    A, B = inputs.uniform_pair(M, N, K, inputs.BF16, 9)
    ref = G.gemm_fp64(A, B, G.BF16)
    for policy in (1, 6):
        _run_and_compare(A, B, inputs.BF16, policy, None, grid=256, ref=ref, fixup=sk.SK_FIXUP_ATOMIC)
        _run_and_compare(A, B, inputs.BF16, policy, None, grid=40, out_dtype=sk.SK_F32, ref=ref, fixup=sk.SK_FIXUP_ATOMIC)


def test_atomic_fixup_fp8_and_unsupported_tile():
    blk = (128, 256, 128)
    M, N, K = 2 * blk[0] + 40, 2 * blk[1] + 72, 5 * blk[2] + 24
    A, B = inputs.small_int_pair(M, N, K, inputs.E4M3, 5)
    ref = G.gemm_fp64(A, B, G.E4M3)
    _run_and_compare(A, B, inputs.E4M3, 6, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True, fixup=sk.SK_FIXUP_ATOMIC)
    # a tile shape without an atomic kernel is refused, not run some other way
    r = Runner(600, 600, 600, 6, (256, 256, 32), 24, sk.SK_BF16, sk.SK_F32, fixup=sk.SK_FIXUP_ATOMIC)
    try:
        a = torch.zeros((600, 600), dtype=torch.int16, device="cuda")
        st = sk.sk_gemm_status(a.data_ptr(), a.data_ptr(), r.D.data_ptr(), r.plan, torch.cuda.current_stream().cuda_stream)
        assert st == sk.SK_ERR_UNSUPPORTED
    finally:
        r.close()


@pytest.mark.parametrize("fixup", [sk.SK_FIXUP_FLAGS, sk.SK_FIXUP_ATOMIC])
def test_hip_graph_replay_matches_eager(fixup):
    # a captured launch holds no memset node and no per-launch argument: replays, with eager work and
    # synchronisations in between, must give the eager result every time (integer inputs: exact under both fix-ups)
    M = N = K = 512
    A, B = inputs.small_int_pair(M, N, K, inputs.F16, 31)
    dA, dB = to_device(A), to_device(B)
    r = Runner(M, N, K, sk.SK_POLICY_ALL_SK, (128, 128, 32), 256, inputs.F16, sk.SK_F32, fixup=fixup)
    try:
        eager = r.run(dA, dB).clone()            # also the first use of the kernel (not allowed under capture)
        assert r.check() == sk.SK_OK
        assert np.array_equal(eager.cpu().numpy().astype(np.float64), G.gemm_fp64(A, B, G.F16))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            r.run(dA, dB)
        for i in range(6):
            r.D.fill_(-1.0)                      # eager work between the replays
            if i % 2:
                assert torch.equal(r.run(dA, dB), eager)   # and eager launches of the same plan
                r.D.fill_(-2.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(r.D, eager), "replay %d differs" % i
        assert r.check() == sk.SK_OK
    finally:
        r.close()


@pytest.mark.parametrize("index", list(range(7, 500, 45)))
def test_sweep_shapes_sampled_rows(index):
    # sizes of the 500-shape tuning sweep, under the library's own tile choice as the sweep runs them
    M, N, K = inputs.sweep_shapes(500, 4)[index]
    A, B = inputs.uniform_pair(M, N, K, inputs.BF16, 100 + index)
    rows = inputs.sample_rows(M, 6, index)
    ref = G.gemm_fp64(A, B, G.BF16, rows=rows)
    for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(A, B, inputs.BF16, policy, None, rows=rows, ref=ref)


def _paper_suite_cases():
    # power-of-two sizes of the paper-shaped suite, small enough for the fp64 oracle on sampled rows;
    # the extremes of every dimension are among them
    suite = inputs.paper_suite()
    small = [s for s in suite if s[0] * s[1] * s[2] <= 1 << 31]
    keep = small[::40]
    for want in (min(small), max(small, key=lambda s: s[2]), min(small, key=lambda s: (s[2], -s[0])), max(small, key=lambda s: s[0])):
        if want not in keep:
            keep.append(want)
    return keep


@pytest.mark.parametrize("shape", _paper_suite_cases())
def test_paper_suite_shapes_fp16_sampled_rows(shape):
    M, N, K = shape
    A, B = inputs.uniform_pair(M, N, K, inputs.F16, 200 + M % 97 + K % 89)
    rows = inputs.sample_rows(M, min(M, 6), K)
    ref = G.gemm_fp64(A, B, G.F16, rows=rows)
    for policy in (sk.SK_POLICY_DP, sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(A, B, inputs.F16, policy, None, rows=rows, ref=ref)


@pytest.mark.parametrize("blk,shape", [((32, 128, 64), (64, 208, 7872)), ((16, 128, 64), (48, 256, 6208)),
                                       ((64, 128, 64), (128, 128, 16448)), ((128, 128, 64), (128, 256, 8256)),
                                       ((32, 128, 64), (32, 1024, 4160)), (None, (112, 128, 3552)),
                                       # 128 accumulators per lane: reduced block by block, two contributors per
                                       # round trip; 32 - 33 contributors per tile, then 67 (an odd one left over)
                                       ((256, 256, 64), (300, 512, 4160)), ((256, 256, 64), (256, 256, 4352))])
def test_tiles_shared_by_many_workgroups(blk, shape):
    # few tiles, long K: 16 ... 120 contributors per tile, reduced in two levels (groups of 8 behind a leader)
    M, N, K = shape
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 41)
    ref = G.gemm_fp64(A, B, G.BF16)
    for policy in (sk.SK_POLICY_SK1_DP, sk.SK_POLICY_ALL_SK):
        _run_and_compare(A, B, inputs.BF16, policy, blk, grid=256, out_dtype=sk.SK_F32, ref=ref, exact=True, launches=3)
    A, B = inputs.uniform_pair(M, N, K, inputs.BF16, 42)
    ref = G.gemm_fp64(A, B, G.BF16)
    _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_ALL_SK, blk, grid=256, ref=ref)
    # the order of the additions is fixed: bit-identical from run to run
    dA, dB = to_device(A), to_device(B)
    r = Runner(M, N, K, sk.SK_POLICY_ALL_SK, blk, 256, inputs.BF16, sk.SK_F32)
    try:
        first = r.run(dA, dB).clone()
        for _ in range(5):
            assert torch.equal(r.run(dA, dB), first)
        assert r.check() == sk.SK_OK
    finally:
        r.close()


@pytest.mark.parametrize("blk", [(16, 128, 64), (32, 128, 64), (64, 128, 64), (128, 128, 64)])
def test_every_small_contributor_count(blk):
    # 1 ... 9 contributors per tile: the owner fetches them in groups (2 to 8 per round trip, by tile) and
    # the ones left over together - every group size and every remainder occurs
    bm, bn, bk = blk
    for c in range(1, 10):
        M, N, K = bm, 2 * bn, bk * 3 * (c + 1)
        A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 50 + c)
        ref = G.gemm_fp64(A, B, G.BF16)
        _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_ALL_SK, blk, grid=2 * (c + 1), out_dtype=sk.SK_F32, ref=ref, exact=True, launches=2)
        _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_ALL_SK, blk, grid=2 * (c + 1), out_dtype=sk.SK_BF16, ref=ref)     # sums beyond 256 round in bf16
        _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_ALL_SK, blk, grid=2 * (c + 1), out_dtype=sk.SK_F32, ref=ref, exact=True, k_aligned=False)


@pytest.mark.parametrize("blk", [(128, 128, 64), (256, 128, 64), (256, 256, 64), (32, 128, 64)])
def test_data_parallel_batches_first(blk):
    # Sec. 3.2's earlier hybrid: the same work, data-parallel tiles before the Stream-K iterations, under both fix-ups
    M, N, K = 5 * blk[0] + 40, 6 * blk[1] + 72, 7 * blk[2] + 24          # 42 tiles on 24 workgroups: 18 + 24
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 51)
    ref = G.gemm_fp64(A, B, G.BF16)
    for policy in (1, 2, 6):
        for fixup in (sk.SK_FIXUP_FLAGS, sk.SK_FIXUP_ATOMIC):
            _run_and_compare(A, B, inputs.BF16, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True,
                             fixup=fixup, launches=2, dp_first=True)


# ---- Algorithm 1's own segment order (ascending iterations, the first workgroup of a tile owns it); every
# ---- other test runs the library's default, the k-aligned order ----------------------------------

@pytest.mark.parametrize("blk", [(128, 128, 64), (256, 128, 64), (256, 256, 64), (64, 128, 64), (32, 128, 64), (16, 128, 64)])
def test_ascending_order_integer_exact(blk):
    # 42 tiles on 24 workgroups (two pieces per workgroup, hybrids and all-Stream-K), both batch orders, both fix-ups
    M, N, K = 5 * blk[0] + 40, 6 * blk[1] + 72, 7 * blk[2] + 24
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 61)
    ref = G.gemm_fp64(A, B, G.BF16)
    for policy in (1, 2, 3, 6):
        for fixup in (sk.SK_FIXUP_FLAGS, sk.SK_FIXUP_ATOMIC):
            _run_and_compare(A, B, inputs.BF16, policy, blk, grid=24, out_dtype=sk.SK_F32, ref=ref, exact=True,
                             fixup=fixup, launches=2, dp_first=policy == 2, k_aligned=False)


@pytest.mark.parametrize("shape,blk,grid", [
    ((64, 208, 7872), (32, 128, 64), 256),      # 4 tiles, ~64 workgroups each: two-level reduction
    ((100, 128, 40000), (16, 128, 64), 200),    # 7 tiles, ragged groups
    ((128, 256, 4096), (64, 128, 64), 37),      # 4 tiles over 37 workgroups: flat reduction with 9-10 contributors
    ((512, 512, 512), (128, 128, 32), 256),     # cfg1's shape: 16 workgroups per tile, one iteration each
])
def test_ascending_order_tiles_shared_by_many_workgroups(shape, blk, grid):
    M, N, K = shape
    A, B = inputs.small_int_pair(M, N, K, inputs.BF16, 62)
    ref = G.gemm_fp64(A, B, G.BF16)
    _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_ALL_SK, blk, grid=grid, out_dtype=sk.SK_F32, ref=ref, exact=True,
                     launches=3, k_aligned=False)
    A, B = inputs.uniform_pair(M, N, K, inputs.BF16, 63)
    _run_and_compare(A, B, inputs.BF16, sk.SK_POLICY_ALL_SK, blk, grid=grid, launches=2, k_aligned=False)


def test_ascending_order_config2_rows_and_fp8():
    c = inputs.config2()
    rows = inputs.sample_rows_per_band(c["M"], 256, 3, 9)       # every one of the 15 tile rows, both wave halves
    ref = G.gemm_fp64(c["A"], c["B"], G.BF16, rows=rows)
    for policy in (1, 3, 6):
        _run_and_compare(c["A"], c["B"], inputs.BF16, policy, c["blk"], c["grid"], rows=rows, ref=ref, k_aligned=False)
    A, B = inputs.uniform_pair(1000, 1100, 2100, inputs.E4M3, 64)
    for policy in (1, 6):
        _run_and_compare(A, B, inputs.E4M3, policy, (256, 256, 128), 24, k_aligned=False)


# ---- the tuning sweep and the Bloom selection on the device (Sec. 4.2, Sec. 5.1's profiler protocol) -----------

def test_sweep_then_selector_on_first_sizes_and_two_skinny_ones(tmp_path):
    """The sweep itself - not a sample of its sizes - on the first 16 sizes of the 500-size list plus two
    skinny ones: every size is timed under the seven policies, the result of its fastest policy (one of
    the launches the sweep makes) is compared with the oracle on sampled rows, and the records feed the
    selector: no false negatives, the selected policy is a candidate (or the fall-back when the filters
    know nothing), and it is never slower than every candidate."""
    from paper_2408_11417_amd import sweep, selector
    shapes = inputs.sweep_shapes(500, 4)[:16] + [(16, 8192, 8192), (64, 4096, 4096)]
    checked = []

    def verify(rec, policy, A, B, D):
        M, N, K = rec["M"], rec["N"], rec["K"]
        rows = inputs.sample_rows_per_band(M, rec["tile"][0], 2, M + K)[:24]
        ref = G.gemm_fp64(A, B, G.BF16, rows=rows)
        err = G.rel_error(G.decode_numpy(D[rows], G.BF16), ref)
        print("sweep size %dx%dx%d tile %s best %s err %.2e" % (M, N, K, rec["tile"], sk.POLICY_NAMES[policy], err), flush=True)
        assert err <= TOL_16
        checked.append((M, N, K))

    records = sweep.run(shapes, str(tmp_path / "sweep.json"), verbose=False, check_every=0, verify=verify)
    assert checked == shapes and len(records) == len(shapes)
    for r in records:
        assert len(r["time_ns"]) == 7 and min(r["time_ns"]) > 0
    split = 14
    for mode in ("shape", "exact"):
        out = selector.evaluate(records, split, 0.2, mode)
        assert out["false_negatives"] == 0 and out["held_out_sizes"] == len(shapes) - split
        assert 0.0 <= out["pruning_rate_build"] < 1.0
    sel = selector.PolicySelector(records[:split], 0.2, "shape")
    try:
        for r in records:
            p, mask, fell_back = sel.select(r, r["time_ns"])
            cands = [q for q in range(7) if (mask >> q) & 1]
            assert (p in cands) or (fell_back and not cands)
            if cands:
                assert r["time_ns"][p] == min(r["time_ns"][q] for q in cands)
        for r in records[:split]:                      # every winner that was inserted comes back
            want = selector.winner_mask(r["time_ns"], 0.2)
            assert want & ~sel.candidates(r) == 0
    finally:
        sel.close()


# ---- seeded random configurations: everything against everything --------------------------------------------------

def _random_cases(n, seed):
    import random
    rng = random.Random(seed)
    tiles16 = [(128, 128, 32), (128, 128, 64), (256, 128, 64), (256, 256, 64), (64, 128, 64), (32, 128, 64), (16, 128, 64)]
    cases = []
    for _ in range(n):
        fp8 = rng.random() < 0.2
        blk = rng.choice([(256, 256, 128), (128, 256, 128)]) if fp8 else rng.choice(tiles16)
        tiles_m, tiles_n, iters = rng.randint(1, 5), rng.randint(1, 6), rng.randint(1, 9)
        aligned = rng.random() < 0.7
        M = tiles_m * blk[0] - rng.choice([0, 0, 1, 17, blk[0] // 2])
        N = tiles_n * blk[1] - (rng.choice([0, 0, 8, 24, 64]) if aligned else rng.choice([1, 3, 13]))
        K = iters * blk[2] - (rng.choice([0, 0, 8, 16, 40]) if aligned else rng.choice([1, 5, 11]))
        M, N, K = max(M, 1), max(N, 8 if aligned else 1), max(K, 8 if aligned else 1)
        grid = rng.choice([4, 8, 13, 24, 64, 256])
        variant = rng.choice([0, 0, 1, 3])
        cases.append(dict(M=M, N=N, K=K, blk=blk, dtype=inputs.E4M3 if fp8 else rng.choice([inputs.BF16, inputs.F16]),
                          policy=rng.randrange(8), grid=grid, out_f32=rng.random() < 0.6, variant=variant,
                          atomic=(not fp8 or blk[0] == 128) and variant == 0 and blk != (256, 256, 32) and rng.random() < 0.15,
                          dp_first=rng.random() < 0.2, k_aligned=rng.random() < 0.75, seed=rng.randrange(1 << 20)))
    return cases


@pytest.mark.parametrize("chunk", range(6))
def test_seeded_random_configurations_integer_exact(chunk):
    # 20 configurations per chunk: tile family, wave layout, policy, grid, ragged or unaligned sizes, output type, fix-up
    # mode, batch order and segment order drawn together; integer-valued inputs, so every result must be exact
    for c in _random_cases(120, 2024)[chunk * 20:(chunk + 1) * 20]:
        A, B = inputs.small_int_pair(c["M"], c["N"], c["K"], c["dtype"], c["seed"])
        ref = G.gemm_fp64(A, B, ODT[c["dtype"]])
        out = sk.SK_F32 if c["out_f32"] else None
        fixup = sk.SK_FIXUP_ATOMIC if c["atomic"] else sk.SK_FIXUP_FLAGS
        if out is None:
            # 16-bit outputs hold these integers exactly as long as they stay below 2^8 (bf16) / 2^11 (fp16): compare with a tolerance instead
            _run_and_compare(A, B, c["dtype"], c["policy"], c["blk"], grid=c["grid"], ref=ref, fixup=fixup, launches=2,
                             dp_first=c["dp_first"], k_aligned=c["k_aligned"], variant=c["variant"])
        else:
            _run_and_compare(A, B, c["dtype"], c["policy"], c["blk"], grid=c["grid"], out_dtype=out, ref=ref, exact=True, fixup=fixup,
                             launches=2, dp_first=c["dp_first"], k_aligned=c["k_aligned"], variant=c["variant"])
