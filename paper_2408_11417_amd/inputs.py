"""Seeded synthetic inputs for the Stream-K GEMM workloads.

This module serves both the tests' CPU oracle and the GPU path, so it holds
none of the method's arithmetic: only random draws, the rounding of fp32 draws
to a storage type, and the shape lists of the benchmark configurations.
Everything is numpy; values are returned as raw storage bit patterns
(uint16 for fp16 / bf16, uint8 for e4m3) so that both sides start from the
same bits.

The shapes and value distributions stand in for the paper's FP16 benchmark
suite (Sec. 5.1), whose member list is not published.
"""
import numpy as np

F16, BF16, E4M3 = 0, 1, 2
DTYPE_NAMES = {F16: "f16", BF16: "bf16", E4M3: "e4m3"}


def to_bf16_bits(x):
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def to_f16_bits(x):
    """fp32 -> IEEE binary16 bit patterns (numpy rounds to nearest even)."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def _e4m3_magnitudes():
    # the 127 finite non-negative e4m3 values, index = bit pattern 0x00..0x7E
    vals = []
    for b in range(127):
        e, f = b >> 3, b & 7
        vals.append(f * 2.0 ** -9 if e == 0 else (8 + f) * 2.0 ** (e - 10))
    return np.array(vals, dtype=np.float64)


def to_e4m3_bits(x):
    """fp32 -> OCP e4m3 bit patterns, round to nearest even, saturating at +-448."""
    x = np.ascontiguousarray(x, dtype=np.float32).astype(np.float64)
    mags = _e4m3_magnitudes()
    a = np.minimum(np.abs(x), mags[-1])
    hi = np.clip(np.searchsorted(mags, a, side="left"), 0, 126)
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = mags[hi] - a, a - mags[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    return code | (np.signbit(x).astype(np.uint8) << 7)


def to_bits(x, dtype):
    return {F16: to_f16_bits, BF16: to_bf16_bits, E4M3: to_e4m3_bits}[dtype](x)


def uniform_pair(M, N, K, dtype, seed):
    """A (M x K), B (K x N) with values uniform in [-1, 1]."""
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1.0, 1.0, size=(M, K)).astype(np.float32)
    B = rng.uniform(-1.0, 1.0, size=(K, N)).astype(np.float32)
    return to_bits(A, dtype), to_bits(B, dtype)


def normal_pair(M, N, K, dtype, seed, sigma):
    """A (M x K), B (K x N) with values normal(0, sigma)."""
    rng = np.random.default_rng(seed)
    A = (rng.standard_normal(size=(M, K)) * sigma).astype(np.float32)
    B = (rng.standard_normal(size=(K, N)) * sigma).astype(np.float32)
    return to_bits(A, dtype), to_bits(B, dtype)


def small_int_pair(M, N, K, dtype, seed, lo=-3, hi=3):
    """Integer-valued inputs: every product and partial sum is exact in fp32, so any
    schedule must reproduce the exact result."""
    rng = np.random.default_rng(seed)
    A = rng.integers(lo, hi + 1, size=(M, K)).astype(np.float32)
    B = rng.integers(lo, hi + 1, size=(K, N)).astype(np.float32)
    return to_bits(A, dtype), to_bits(B, dtype)


# ---- the benchmark configurations -------------------------------------------------------------

def config1():
    """fp16 512^3, uniform [-1,1], seed 0; 128x128x32 tiles on a 256-workgroup grid."""
    A, B = uniform_pair(512, 512, 512, F16, 0)
    return dict(name="cfg1_f16_512", M=512, N=512, K=512, dtype=F16, out_dtype=F16,
                blk=(128, 128, 32), grid=256, A=A, B=B)


def config2():
    """bf16 3840 x 4224 x 4096 (495 tiles at 256x128: the wave-quantisation case),
    normal(0,1)/sqrt(K), seed 1."""
    M, N, K = 3840, 4224, 4096
    A, B = normal_pair(M, N, K, BF16, 1, 1.0 / np.sqrt(K))
    return dict(name="cfg2_bf16_wavequant", M=M, N=N, K=K, dtype=BF16, out_dtype=BF16,
                blk=(256, 128, 64), grid=256, A=A, B=B)


def config3(M):
    """bf16 skinny decode-style GEMM, M in {16,32,64,128}, N = K = 8192, normal(0, 0.02), seed 2."""
    N = K = 8192
    A, B = normal_pair(M, N, K, BF16, 2, 0.02)
    return dict(name="cfg3_bf16_skinny_M%d" % M, M=M, N=N, K=K, dtype=BF16, out_dtype=BF16,
                blk=None, grid=256, A=A, B=B)


def config5(dtype=BF16, size=8192):
    """Large square GEMM, bf16 or e4m3 inputs, uniform [-1,1], seed 3, bf16 output."""
    A, B = uniform_pair(size, size, size, dtype, 3)
    return dict(name="cfg5_%s_%d" % (DTYPE_NAMES[dtype], size), M=size, N=size, K=size,
                dtype=dtype, out_dtype=BF16, blk=None, grid=256, A=A, B=B)


def sweep_shapes(n=500, seed=4, lo=64, hi=16384):
    """Config 4: n (M, N, K) triples, each dimension log-uniform in [lo, hi] rounded to a
    multiple of 16.  The first 80 % are the build split, the rest are held out."""
    rng = np.random.default_rng(seed)
    raw = np.exp(rng.uniform(np.log(lo), np.log(hi), size=(n, 3)))
    dims = np.clip(np.round(raw / 16.0).astype(np.int64) * 16, lo, hi)
    return [tuple(int(v) for v in row) for row in dims]


def paper_suite(n=923, seed=5):
    """A suite shaped like the paper's (Sec. 5.1): dimensions in powers of two, M from 1 to 8192, N from
    64 to 8192, K from 16 to 65536.  That grid has 14 x 8 x 13 = 1456 sizes; the paper used 923 of
    them and does not list which, so this is a seeded sample of n of them, in random order (the
    first 80 % serve as build split, the rest are held out)."""
    grid = [(1 << m, 1 << nn, 1 << k) for m in range(0, 14) for nn in range(6, 14) for k in range(4, 17)]
    rng = np.random.default_rng(seed)
    pick = rng.permutation(len(grid))[:n]
    return [grid[i] for i in pick]


def sample_rows(M, n, seed):
    """n distinct seeded row indices of an M-row matrix (always including first and last)."""
    rng = np.random.default_rng(seed)
    n = min(n, M)
    rows = set([0, M - 1])
    while len(rows) < n:
        rows.add(int(rng.integers(0, M)))
    return np.array(sorted(rows), dtype=np.int64)


def sample_rows_per_band(M, band, per_band, seed):
    """Seeded row indices that hit every band of `band` consecutive rows: in each band its first
    row, one row of its second half and per_band - 2 random ones (all clipped to M), plus the
    last row of the matrix."""
    rng = np.random.default_rng(seed)
    rows = {M - 1}
    for b0 in range(0, M, band):
        hi = min(b0 + band, M)
        rows.add(b0)
        rows.add(min(b0 + band // 2 + int(rng.integers(0, max(band // 2, 1))), hi - 1))
        for _ in range(max(per_band - 2, 0)):
            rows.add(int(rng.integers(b0, hi)))
    return np.array(sorted(rows), dtype=np.int64)
