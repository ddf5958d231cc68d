"""sk_gemm_static (the entry point that allocates nothing: its flag lines and partial tiles live in an
array inside the library) against sk_gemm on the same plans, through the C ABI: two calls in a row on
the same GPU, the second with a smaller input, both with tiles split over many workgroups so that the
array is really used; results must be bit-identical (same kernels, fixed reduction order) and within
the 16-bit tolerance of the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2408_11417_amd as sk
from paper_2408_11417_amd import inputs
from oracle import gemm as G
from tests.gpu_util import Runner, to_device

pytestmark = pytest.mark.gpu


def _both(M, N, K, policy, blk, seed, out_dtype=None):
    print("no-alloc case M=%d N=%d K=%d policy=%s blk=%s" % (M, N, K, sk.POLICY_NAMES[policy], blk), flush=True)
    A, B = inputs.uniform_pair(M, N, K, inputs.BF16, seed)
    dA, dB = to_device(A), to_device(B)
    stream = torch.cuda.current_stream().cuda_stream
    r = Runner(M, N, K, policy, blk, 256, inputs.BF16, out_dtype)
    try:
        assert sk.sk_workspace_bytes(r.plan) <= (257 * 128 + 384 + 256 * 256 * 256 * 4)
        want = r.run(dA, dB).clone()                       # sk_gemm with a caller-owned workspace
        assert r.check() == sk.SK_OK
        got = torch.full_like(want, -1)
        before = torch.cuda.memory_allocated()
        sk.sk_gemm_static(dA.data_ptr(), dB.data_ptr(), got.data_ptr(), r.plan, stream)
        sk.sk_gemm_static(dA.data_ptr(), dB.data_ptr(), got.data_ptr(), r.plan, stream)   # flags are reusable
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got, want)
        ref = G.gemm_fp64(A, B, G.BF16)
        d = r.result(got)
        assert G.rel_error(d, ref) <= (1e-4 if out_dtype == sk.SK_F32 else 1e-2)
    finally:
        r.close()


def test_static_scratch_entry_matches_sk_gemm_two_calls_second_smaller():
    _both(520, 776, 4160, sk.SK_POLICY_ALL_SK, (128, 128, 64), 71)       # 35 tiles over 256 workgroups: 7-8 contributors each
    _both(200, 264, 2080, sk.SK_POLICY_SK1_DP, (64, 128, 64), 72, sk.SK_F32)   # smaller: 12 tiles, two-level reduction
    _both(300, 512, 1040, sk.SK_POLICY_DP, None, 73)                      # no split tile: no scratch use at all


def test_static_scratch_entry_refuses_what_does_not_fit():
    a = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    # a grid of 512 workgroups with 256 x 256 tiles needs 128 MiB of partial tiles: beyond the array
    plan = sk.sk_plan(600, 600, 4096, sk.SK_POLICY_ALL_SK, (256, 256, 64), 512, sk.SK_BF16)
    try:
        assert sk.binding._lib.sk_gemm_static(a.data_ptr(), a.data_ptr(), a.data_ptr(), plan, stream) == sk.SK_ERR_WORKSPACE
    finally:
        sk.sk_plan_destroy(plan)
    # the atomic fix-up with a 16-bit output keeps an fp32 image of D, which has no bound
    plan = sk.sk_plan(600, 600, 600, sk.SK_POLICY_ALL_SK, (128, 128, 64), 256, sk.SK_BF16)
    try:
        sk.sk_plan_set_fixup(plan, sk.SK_FIXUP_ATOMIC)
        assert sk.binding._lib.sk_gemm_static(a.data_ptr(), a.data_ptr(), a.data_ptr(), plan, stream) == sk.SK_ERR_UNSUPPORTED
    finally:
        sk.sk_plan_destroy(plan)
    assert sk.binding._lib.sk_gemm_static(None, None, None, None, None) == sk.SK_ERR_INVALID_ARG
