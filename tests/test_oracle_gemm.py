"""Pins for the GEMM oracle: storage decoders against the format definitions and numpy, the
triple loop against brute force, a library matmul, and closed-form special cases."""
import os

import numpy as np
import pytest

from oracle import gemm as G
from paper_2408_11417_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CODES = {"f16": G.F16, "bf16": G.BF16, "e4m3": G.E4M3}


def test_decoders_on_format_spot_values():
    n = 0
    for line in open(os.path.join(GOLDEN, "storage_formats.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, bits, expr = line.split()
        want = float(eval(expr, {"__builtins__": {}}))
        assert G.decode_c([int(bits, 16)], CODES[name])[0] == want
        assert G.decode_numpy(np.array([int(bits, 16)]), CODES[name])[0] == want
        n += 1
    assert n == 19


@pytest.mark.parametrize("dtype,count", [(G.F16, 65536), (G.BF16, 65536), (G.E4M3, 256)])
def test_c_decoder_equals_numpy_decoder_on_every_bit_pattern(dtype, count):
    bits = np.arange(count)
    with np.errstate(all="ignore"):
        a, b = G.decode_c(bits, dtype), G.decode_numpy(bits, dtype)
    assert np.array_equal(np.isnan(a), np.isnan(b))
    ok = ~np.isnan(a)
    assert np.array_equal(a[ok], b[ok]) and np.array_equal(np.signbit(a[ok]), np.signbit(b[ok]))


def test_e4m3_has_no_infinity_and_two_nans():
    v = G.decode_c(np.arange(256), G.E4M3)
    assert not np.isinf(v).any() and np.isnan(v).sum() == 2 and np.nanmax(v) == 448.0


@pytest.mark.parametrize("dtype", [G.F16, G.BF16, G.E4M3])
def test_input_rounding_roundtrips_through_the_oracle_decoder(dtype):
    rng = np.random.default_rng(0)
    x = rng.uniform(-2, 2, size=4000).astype(np.float32)
    bits = inputs.to_bits(x, dtype)
    back = G.decode_numpy(bits, dtype)
    ulp = {G.F16: 2.0 ** -10, G.BF16: 2.0 ** -7, G.E4M3: 2.0 ** -3}[dtype]
    assert np.all(np.abs(back - x) <= np.maximum(np.abs(x), 2.0 ** -6) * ulp / 2 * 1.0001)
    assert np.array_equal(inputs.to_bits(back.astype(np.float32), dtype), bits)   # already representable


def test_bruteforce_16cubed_python_loops_bit_identical():
    A, B = inputs.uniform_pair(16, 16, 16, inputs.F16, 7)
    a, b = G.decode_numpy(A, G.F16), G.decode_numpy(B, G.F16)
    ref = np.empty((16, 16))
    for i in range(16):
        for j in range(16):
            acc = 0.0
            for k in range(16):
                acc += float(a[i, k]) * float(b[k, j])
            ref[i, j] = acc
    assert np.array_equal(G.gemm_fp64(A, B, G.F16, order=0), ref)
    assert np.array_equal(G.gemm_fp64(A, B, G.F16, order=1), ref)


@pytest.mark.parametrize("dtype", [G.F16, G.BF16, G.E4M3])
def test_loop_orders_bit_identical_and_close_to_numpy_matmul(dtype):
    A, B = inputs.uniform_pair(37, 53, 129, dtype, 3)
    d0, d1 = G.gemm_fp64(A, B, dtype, order=0), G.gemm_fp64(A, B, dtype, order=1)
    assert np.array_equal(d0, d1)
    ref = G.gemm_numpy(A, B, dtype)
    assert np.max(np.abs(d0 - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_transposed_or_swapped_operands_would_be_caught():
    # a non-square, non-symmetric case: row i of a one-hot A picks row perm[i] of B
    M, K, N = 5, 9, 7
    perm = [3, 8, 0, 5, 1]
    a = np.zeros((M, K), dtype=np.float32)
    for i, p in enumerate(perm):
        a[i, p] = 1.0
    b = np.arange(K * N, dtype=np.float32).reshape(K, N) - 20
    D = G.gemm_fp64(inputs.to_bits(a, inputs.BF16), inputs.to_bits(b, inputs.BF16), G.BF16)
    assert np.array_equal(D, b[perm].astype(np.float64))


def test_all_ones_gives_K_and_signs_are_kept():
    M, N, K = 4, 6, 2048
    ones = np.ones((M, K), dtype=np.float32)
    D = G.gemm_fp64(inputs.to_bits(ones, inputs.F16), inputs.to_bits(np.ones((K, N), np.float32), inputs.F16), G.F16)
    assert np.all(D == K)
    D = G.gemm_fp64(inputs.to_bits(-ones, inputs.F16), inputs.to_bits(np.ones((K, N), np.float32), inputs.F16), G.F16)
    assert np.all(D == -K)


def test_sampled_rows_equal_the_same_rows_of_the_full_product():
    A, B = inputs.normal_pair(64, 40, 96, inputs.BF16, 9, 0.5)
    full = G.gemm_fp64(A, B, G.BF16)
    rows = inputs.sample_rows(64, 9, 1)
    assert rows[0] == 0 and rows[-1] == 63 and len(set(rows)) == 9
    assert np.array_equal(G.gemm_fp64(A, B, G.BF16, rows=rows), full[rows])


def test_accumulation_is_really_fp64():
    # 1 + 2^-20 * 2^-20 ... : products below fp32 resolution must survive
    K = 4
    a = np.array([[1.0, 2.0 ** -12, 2.0 ** -12, -1.0]], dtype=np.float32)
    b = np.array([[1.0], [2.0 ** -13], [2.0 ** -13], [1.0]], dtype=np.float32)
    D = G.gemm_fp64(inputs.to_bits(a, inputs.F16), inputs.to_bits(b, inputs.F16), G.F16)
    assert D[0, 0] == 2.0 ** -24


def test_bad_arguments():
    A, B = inputs.uniform_pair(4, 4, 4, inputs.F16, 0)
    with pytest.raises(ValueError):
        G.gemm_fp64(A, B[:3], G.F16)
    with pytest.raises(TypeError):
        G.gemm_fp64(A.astype(np.float32), B, G.F16)
    with pytest.raises(ValueError):
        G.gemm_fp64(A, B, G.F16, rows=[7])


def test_rel_error_metric():
    ref = np.array([[1.0, -2.0], [0.0, 4.0]])
    assert G.rel_error(ref, ref) == 0.0
    d = ref + np.array([[0.01, 0.0], [0.0, 0.0]])
    assert G.rel_error(d, ref) == pytest.approx(0.01 / np.sqrt(21 / 4))
