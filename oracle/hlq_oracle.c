/* CPU oracle for the HLQ bit-serial LUT GEMV/GEMM path -- plain C, fp64.
 * TEST INFRASTRUCTURE ONLY: loaded by tests, the smoke check and the benchmark's
 * cpu_baseline leg.  Shares nothing with the HIP library and never sees its packed
 * layout.
 *
 * Definition (Eq. 3 / Eq. 6 of the paper, then an ordinary matrix product):
 *     W^[k,n] = sum_{j<q} s_j[k/G, n] * bit_j(codes[k,n]) + z[k/G, n]
 *     Y[m,n]  = sum_{k<K} X[m,k] * W^[k,n]            (k ascending, fp64)
 * Inputs are the unpacked tensors: codes u8 [K,N] (bit j = plane j, App. B),
 * scales fp16 [q,K/G,N], zeros fp16 [K/G,N], X fp16 [M,ldx].
 *
 * Pinned in tests/test_oracle_c.py against the numpy oracle, exact-rational brute
 * force, and the closed-form special cases.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE binary16 -> double, written out by field (no compiler half type needed). */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = (double)frac * 5.9604644775390625e-08;           /* frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? (0.0 / 0.0) : (1.0 / 0.0);
    } else {
        double p = 1.0;
        int e = expo - 15, i;
        for (i = 0; i < (e < 0 ? -e : e); ++i) p *= 2.0;
        v = (1.0 + (double)frac / 1024.0) * (e < 0 ? 1.0 / p : p);
    }
    return sign ? -v : v;
}

int hlq_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Y[m, c] for the listed columns (cols == NULL: all N columns, c == n).
 * Y is [M, ldy] doubles; column c of Y corresponds to weight column cols[c].
 * Returns 0, or -1 on a bad argument. */
int hlq_oracle_gemm_f64(int64_t K, int64_t N, int q, int G, int64_t M,
                        const uint8_t *codes, const uint16_t *scales,
                        const uint16_t *zeros, const uint16_t *X, int64_t ldx,
                        double *Y, int64_t ldy, const int64_t *cols, int64_t ncols)
{
    if (!codes || !scales || !zeros || !X || !Y) return -1;
    if (q < 1 || q > 8 || G < 1 || K % G != 0 || M < 0) return -1;
    if (!cols) ncols = N;
    const int64_t ngroups = K / G;

    /* activations to fp64 once */
    double *xd = (double *)malloc((size_t)(M > 0 ? M : 1) * (size_t)K * sizeof(double));
    if (!xd) return -1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            xd[m * K + k] = half_to_double(X[m * ldx + k]);

    #pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < ncols; ++c) {
        const int64_t n = cols ? cols[c] : c;
        /* reconstruct column n of W^ once (Eq. 3), then one dot product per row */
        double *w = (double *)malloc((size_t)K * sizeof(double));
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = k / G;
            double v = half_to_double(zeros[g * N + n]);
            for (int j = 0; j < q; ++j)
                if ((codes[k * N + n] >> j) & 1)
                    v += half_to_double(scales[((int64_t)j * ngroups + g) * N + n]);
            w[k] = v;
        }
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += xd[m * K + k] * w[k];
            Y[m * ldy + c] = acc;
        }
        free(w);
    }
    free(xd);
    return 0;
}
