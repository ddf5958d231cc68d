/* GEMM oracle: D = A * B by the textbook definition, accumulated in fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  Not part of the product library; shares no code
 * with it.  Built by oracle/gemm.py (gcc -O2 -fopenmp).
 *
 * Definition followed (Sec. 1 of the paper, "general matrix multiplication";
 * Sec. 3.1: the MAC iterations of all output tiles together compute exactly
 * this): D[i][j] = sum over k = 0..K-1, in ascending k, of A[i][k] * B[k][j],
 * with A row-major M x K, B row-major K x N, D row-major M x N.  The inputs are
 * the stored fp16 / bf16 / fp8-e4m3 bit patterns, decoded exactly to double;
 * products of two such values are exact in double and the running sum is kept
 * in double and never rounded to a narrower type.
 *
 * Two loop orders are offered.  order 0 is the definition as written (i, j, k).
 * order 1 (i, k, j) walks B by rows so that large problems finish in reasonable
 * time; every D[i][j] still receives its products in ascending k, so the two
 * are bit-identical (a test checks that).
 *
 * Storage formats (decoded here from their public definitions):
 *   fp16   IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.
 *   bf16   the upper 16 bits of an IEEE binary32.
 *   e4m3   OCP 8-bit float: 1 sign, 4 exponent (bias 7), 3 fraction bits, no
 *          infinities, S.1111.111 is NaN, largest finite value 448.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_E4M3 = 2 };

static double decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

static double decode_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double decode_e4m3(uint8_t b)
{
    int sign = (b >> 7) & 1, e = (b >> 3) & 0xF, f = b & 7;
    double v;
    if (e == 0)
        v = ldexp((double)f, -9);                  /* subnormal: f * 2^-3 * 2^-6 */
    else if (e == 15 && f == 7)
        v = NAN;
    else
        v = ldexp(1.0 + (double)f / 8.0, e - 7);
    return sign ? -v : v;
}

/* Decode one stored element to double.  Exported so that tests can pin the decoders. */
double oracle_decode(uint32_t bits, int dtype)
{
    switch (dtype) {
    case ORACLE_F16:  return decode_f16((uint16_t)bits);
    case ORACLE_BF16: return decode_bf16((uint16_t)bits);
    case ORACLE_E4M3: return decode_e4m3((uint8_t)bits);
    default:          return NAN;
    }
}

/* Every bit pattern of the storage type decoded once, so that the loops below
 * read a value with one lookup instead of re-running the decoder per product. */
static double *decode_table(int dtype)
{
    uint32_t n = dtype == ORACLE_E4M3 ? 256u : 65536u;
    double *t = malloc(n * sizeof *t);
    if (t)
        for (uint32_t b = 0; b < n; b++)
            t[b] = oracle_decode(b, dtype);
    return t;
}

static inline double elem(const void *p, int64_t idx, int dtype, const double *table)
{
    if (dtype == ORACLE_E4M3)
        return table[((const uint8_t *)p)[idx]];
    return table[((const uint16_t *)p)[idx]];
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* D (n_rows x N doubles, or M x N when rows == NULL) = selected rows of A*B.
 * rows: optional list of row indices of A to compute (sampled-row mode for
 * shapes too large to finish in full); same definition for each row.
 * Returns 0, or -1 on a bad argument. */
int oracle_gemm(const void *A, const void *B, double *D, int64_t M, int64_t N, int64_t K,
                int dtype, const int64_t *rows, int64_t n_rows, int order)
{
    if (!A || !B || !D || M < 1 || N < 1 || K < 1 || dtype < 0 || dtype > 2)
        return -1;
    if (!rows)
        n_rows = M;
    for (int64_t r = 0; r < n_rows; r++)
        if (rows && (rows[r] < 0 || rows[r] >= M))
            return -1;

    double *table = decode_table(dtype);
    if (!table)
        return -1;

    if (order == 0) {
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < n_rows; r++) {
            int64_t i = rows ? rows[r] : r;
            for (int64_t j = 0; j < N; j++) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; k++)
                    acc += elem(A, i * K + k, dtype, table) * elem(B, k * N + j, dtype, table);
                D[r * N + j] = acc;
            }
        }
        free(table);
        return 0;
    }

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; r++) {
        int64_t i = rows ? rows[r] : r;
        double *drow = D + r * N;
        for (int64_t j = 0; j < N; j++)
            drow[j] = 0.0;
        for (int64_t k = 0; k < K; k++) {
            double a = elem(A, i * K + k, dtype, table);
            for (int64_t j = 0; j < N; j++)
                drow[j] += a * elem(B, k * N + j, dtype, table);
        }
    }
    free(table);
    return 0;
}
