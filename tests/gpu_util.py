"""Helpers for the GPU parity tests: device buffers through torch (memory and streams only)."""
import numpy as np
import torch

import paper_2408_11417_amd as sk
from oracle import gemm as G

OUT_TORCH = {sk.SK_F16: torch.int16, sk.SK_BF16: torch.int16, sk.SK_F32: torch.float32}


def to_device(bits):
    """numpy storage bit patterns (uint16 / uint8) -> device tensor with the same bytes."""
    view = bits.view(np.int16) if bits.dtype == np.uint16 else bits.view(np.uint8)
    return torch.from_numpy(np.ascontiguousarray(view)).cuda()


class Runner:
    """One plan with its workspace; run() launches sk_gemm on torch's current stream."""

    def __init__(self, M, N, K, policy, blk=None, grid=0, in_dtype=sk.SK_BF16, out_dtype=None, tile_order=None,
                 fixup=sk.SK_FIXUP_FLAGS, dp_first=False, k_aligned=True, variant=0):
        self.plan = sk.sk_plan(M, N, K, policy, blk, grid, in_dtype, out_dtype, tile_order)
        sk.sk_plan_set_fixup(self.plan, fixup)
        if dp_first:
            sk.sk_plan_set_batch_order(self.plan, sk.SK_DATA_PARALLEL_FIRST)
        sk.sk_plan_set_segment_order(self.plan, sk.SK_SEGMENTS_K_ALIGNED if k_aligned else sk.SK_SEGMENTS_ASCENDING)
        sk.sk_plan_set_kernel_variant(self.plan, variant)
        self.info = sk.sk_plan_info(self.plan)
        nbytes = sk.sk_workspace_bytes(self.plan)
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        base = (self.ws.data_ptr() + 255) // 256 * 256
        sk.sk_plan_set_workspace(self.plan, base, nbytes)
        self.D = torch.empty((M, N), dtype=OUT_TORCH[self.info["out_dtype"]], device="cuda")

    def run(self, dA, dB, D=None):
        D = self.D if D is None else D
        sk.sk_gemm(dA.data_ptr(), dB.data_ptr(), D.data_ptr(), self.plan, torch.cuda.current_stream().cuda_stream)
        return D

    def check(self):
        return sk.sk_plan_check(self.plan, torch.cuda.current_stream().cuda_stream)

    def result(self, D=None):
        """Output as float64 (decoded by the oracle's numpy decoder)."""
        D = self.D if D is None else D
        torch.cuda.synchronize()
        h = D.cpu().numpy()
        od = self.info["out_dtype"]
        if od == sk.SK_F32:
            return h.astype(np.float64)
        return G.decode_numpy(h.view(np.uint16), G.F16 if od == sk.SK_F16 else G.BF16)

    def close(self):
        sk.sk_plan_destroy(self.plan)
        self.plan = None
