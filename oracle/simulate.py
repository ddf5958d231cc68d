"""Schedule-executing simulator: runs a plan segment by segment on the CPU.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

It proves, without a GPU, that a schedule from oracle/schedule.py together with
the workspace-and-flags fix-up (Sec. 5.3's alternative to the atomic adds at the
end of Algorithm 1's loop body) computes the GEMM: every segment runs Algorithm 1's
MAC_loop over its k-iterations into an fp32 accumulator tile; a
CONTRIB segment parks its tile in the workspace slot of its workgroup; an OWNER
adds the parked tiles of its contributors in the schedule's reduction order and
stores; a FULL segment stores directly.  Contributors always execute before the
owner reads them here because the simulator runs all CONTRIB segments first;
on the device the flags provide that ordering.
"""
import numpy as np

from . import schedule as S


def run_plan(p, A, B):
    """A (M x K), B (K x N): float64 arrays holding the decoded input values.
    Returns D (M x N) float32: what the fp32-accumulator path produces."""
    h = p.header
    M, N, K = h["M"], h["N"], h["K"]
    bm, bn, bk, ipt = h["blk_m"], h["blk_n"], h["blk_k"], h["iters_per_tile"]
    D = np.full((M, N), np.nan, dtype=np.float32)
    written = np.zeros((M, N), dtype=np.int32)
    workspace = {}

    def mac_loop(seg):
        tm, tn = S.tile_coords(seg.tile, h["tiles_m"], h["tiles_n"], h["tile_order"])
        r0, r1 = tm * bm, min((tm + 1) * bm, M)
        c0, c1 = tn * bn, min((tn + 1) * bn, N)
        acc = np.zeros((r1 - r0, c1 - c0), dtype=np.float32)
        for it in range(seg.k_begin, seg.k_end):
            k0, k1 = it * bk, min((it + 1) * bk, K)
            acc = (acc.astype(np.float64) + A[r0:r1, k0:k1] @ B[k0:k1, c0:c1]).astype(np.float32)
        return (r0, r1, c0, c1), acc

    for seg in p.segments:
        if seg.role == S.ROLE_CONTRIB:
            assert seg.wg not in workspace, "one workspace slot per workgroup"
            workspace[seg.wg] = (seg.tile, mac_loop(seg)[1])
    for seg in p.segments:
        if seg.role == S.ROLE_CONTRIB:
            continue
        (r0, r1, c0, c1), acc = mac_loop(seg)
        if seg.role == S.ROLE_OWNER:
            for c in S.contributors(p, seg):
                tile, part = workspace.pop(c)
                assert tile == seg.tile
                acc = acc + part                   # fp32 add, in reduction order
        D[r0:r1, c0:c1] = acc
        written[r0:r1, c0:c1] += 1
    assert not workspace, "unconsumed partial tiles"
    assert (written == 1).all(), "every output element is stored exactly once"
    return D
