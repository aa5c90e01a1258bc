/*
 * CPU oracle for C = A x B  --  TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * Only the tests, the smoke check and the benchmark's "cpu_baseline" leg may
 * call this file.  It shares no code, header, table or helper with the GPU
 * library.  It is deliberately plain: one loop nest that is the textbook
 * definition of the sparse-dense product C = A x B, A sparse and B dense (paper,
 * Section 2.2), with the operand precision of
 * the paper's Problem Configuration (Section 4.1): A and B hold IEEE binary16
 * values.  The paper accumulates in fp32; this oracle widens every operand
 * exactly to fp64 and accumulates in fp64 in stored (CSR) order, so it is
 * strictly more accurate than any summation order a GPU kernel may pick.
 *
 * For every output it also returns S[i][j] = sum_k |a_ik| |b_kj|, the scale
 * the acceptance test |C_gpu - C| <= 1e-4 * S is stated against.
 *
 * No blocking, no fusion, no reordering, no hand vectorisation.  Rows are
 * distributed over OpenMP threads; each output element is one serial fp64 sum
 * whose terms arrive in CSR order (the loop over stored entries is outside the
 * loop over the N columns, so a_ik is widened once per entry).
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 -> binary64, exact (every binary16 value is a binary64 value). */
static double half_to_double(uint16_t h)
{
    const uint64_t sign = (uint64_t)(h >> 15) << 63;
    const int expo = (h >> 10) & 0x1f;
    const uint64_t frac = h & 0x3ff;
    union { uint64_t u; double d; } w;
    if (expo == 0) {
        /* zero and subnormals: frac * 2^-24, exact in binary64 */
        w.d = (double)frac * 0x1p-24;
        w.u |= sign;
    } else if (expo == 31) {
        w.u = sign | 0x7ff0000000000000ull | (frac << 42);   /* inf / nan */
    } else {
        /* rebias the exponent (15 -> 1023) and left-align the 10 fraction bits in 52 */
        w.u = sign | ((uint64_t)(expo - 15 + 1023) << 52) | (frac << 42);
    }
    return w.d;
}

void oracle_half_to_double(const uint16_t *in, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = half_to_double(in[i]);
}

/*
 * rows == NULL : compute all n_rows rows; C and S are [n_rows][N].
 * rows != NULL : compute the n_sel listed rows; C and S are [n_sel][N], row t
 *                of the output is row rows[t] of the product.
 * S may be NULL.  Returns the number of threads used.
 */
int oracle_spmm(int64_t n_rows, const int64_t *row_ptr, const int32_t *col_idx,
                const uint16_t *val, const uint16_t *B, int64_t N,
                const int64_t *rows, int64_t n_sel, double *C, double *S, int nthreads)
{
    const int64_t n_out = rows ? n_sel : n_rows;
    int used = 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    used = nthreads;
#pragma omp parallel for schedule(dynamic, 64) num_threads(nthreads)
#endif
    for (int64_t t = 0; t < n_out; ++t) {
        const int64_t i = rows ? rows[t] : t;
        double *c = C + t * N;
        double *s = S ? S + t * N : NULL;
        for (int64_t j = 0; j < N; ++j) {
            c[j] = 0.0;
            if (s) s[j] = 0.0;
        }
        /* stored order: every c[j] receives its terms for p = row_ptr[i], row_ptr[i]+1, ... */
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            const double a = half_to_double(val[p]);
            const uint16_t *b_row = B + (int64_t)col_idx[p] * N;
            for (int64_t j = 0; j < N; ++j) {
                const double b = half_to_double(b_row[j]);
                c[j] += a * b;
                if (s) s[j] += fabs(a) * fabs(b);
            }
        }
    }
    return used;
}
