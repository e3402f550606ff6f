/*
 * CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT PATH.
 *
 * Plain fp64 evaluation of the binary-coded linear layer of GPTQT
 * (arXiv 2407.02891).  Only tests, the smoke check and the bench's CPU
 * baseline may load this library; the HIP library never does and shares
 * no source, header, table or helper with it.
 *
 * What is computed (paper Eq. 3, dequantisation line, and Eq. 11, the fused
 * inference form):
 *
 *     W[m][k] = sum_{i=0..q-1} alpha[m][k/g][i] * s_i[m][k]  (+ z[m][k/g])
 *     Y[j][m] = sum_{k=0..N-1} W[m][k] * X[j][k]
 *
 * with s_i in {-1,+1}.  The paper fixes neither the bit encoding nor the
 * packing; the readings used here are: bit 1 <-> +1, bit 0 <-> -1; plane
 * words are uint32, least-significant bit first along N (bit j of word w is
 * column 32*w + j).  alpha, z and X are IEEE binary16 bit patterns and are
 * widened exactly; every sum is a left-to-right fp64 sum in the index order
 * written above.  No blocking, no reordering, no tables.
 *
 * Canonical operand layout (row-major, all host memory):
 *     planes [q][M][N/32] uint32     alpha [M][N/g][q] uint16
 *     z      [M][N/g]     uint16 or NULL
 *     X      [b][N]       uint16     Y [b][M] double     W [M][N] double
 *
 * Return value of the int functions: 0 on success, 1 on a bad argument.
 *
 * Pins (tests/test_oracle_pins.py): the binary16 widening against numpy for
 * all 65536 patterns; the paper's Eq. 6/9/10/11 worked values; the
 * round trip linear-int -> binary coding -> dequant == S*W_int + qbias;
 * q = 1 sign matrix against an int64 matvec; the all-ones popcount closed
 * form; unit-vector column probes; bcq_ref_brute against bcq_ref_gemm; and
 * algebraic invariants.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 bit pattern -> double, exact (subnormals, signed zero,
 * infinities and NaN included). */
double bcq_ref_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);            /* subnormal or zero */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + frac), expo - 25);
    return sign ? -v : v;
}

static int bad_shape(int64_t M, int64_t N, int q, int64_t g)
{
    return M <= 0 || N <= 0 || q < 1 || q > 8 || g <= 0 || N % 32 != 0 ||
           N % g != 0;
}

/* sign of weight (m,k) in plane i: +1 if the stored bit is 1, else -1 */
static double plane_sign(const uint32_t *planes, int64_t M, int64_t N, int i,
                         int64_t m, int64_t k)
{
    uint32_t word = planes[((int64_t)i * M + m) * (N / 32) + (k >> 5)];
    return ((word >> (k & 31)) & 1u) ? 1.0 : -1.0;
}

/* One dequantised row, Eq. 3 (dequant) / Eq. 11: planes summed in order
 * i = 0..q-1, then the group offset added. */
static void dequant_row(const uint32_t *planes, const uint16_t *alpha,
                        const uint16_t *z, int64_t M, int64_t N, int q,
                        int64_t g, int64_t m, double *wrow)
{
    int64_t G = N / g;
    for (int64_t k = 0; k < N; ++k) {
        int64_t grp = k / g;
        double w = 0.0;
        for (int i = 0; i < q; ++i) {
            double a = bcq_ref_half_to_double(alpha[(m * G + grp) * q + i]);
            w += a * plane_sign(planes, M, N, i, m, k);
        }
        if (z)
            w += bcq_ref_half_to_double(z[m * G + grp]);
        wrow[k] = w;
    }
}

/* Dense W[M][N] in fp64. */
int bcq_ref_dequant(const uint32_t *planes, const uint16_t *alpha,
                    const uint16_t *z, int64_t M, int64_t N, int q, int64_t g,
                    double *W)
{
    if (!planes || !alpha || !W || bad_shape(M, N, q, g))
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        dequant_row(planes, alpha, z, M, N, q, g, m, W + m * N);
    return 0;
}

/* Y[j][m] = sum_k W[m][k] * X[j][k], X given as binary16 bit patterns. */
int bcq_ref_dense_matmul(const double *W, const uint16_t *X, int64_t M,
                         int64_t N, int64_t b, double *Y)
{
    if (!W || !X || !Y || M <= 0 || N <= 0 || b <= 0)
        return 1;
    double *xd = (double *)malloc(sizeof(double) * (size_t)(b * N));
    if (!xd)
        return 1;
    for (int64_t t = 0; t < b * N; ++t)
        xd[t] = bcq_ref_half_to_double(X[t]);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t j = 0; j < b; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < N; ++k)
                acc += W[m * N + k] * xd[j * N + k];
            Y[j * M + m] = acc;
        }
    }
    free(xd);
    return 0;
}

/* The whole path: dequantise, then dense product.  Rows are dequantised one
 * at a time into a scratch row so that the largest layers fit in memory; the
 * arithmetic is that of bcq_ref_dequant followed by bcq_ref_dense_matmul. */
int bcq_ref_gemm(const uint32_t *planes, const uint16_t *alpha,
                 const uint16_t *z, const uint16_t *X, int64_t M, int64_t N,
                 int q, int64_t g, int64_t b, double *Y)
{
    if (!planes || !alpha || !X || !Y || b <= 0 || bad_shape(M, N, q, g))
        return 1;
    double *xd = (double *)malloc(sizeof(double) * (size_t)(b * N));
    if (!xd)
        return 1;
    for (int64_t t = 0; t < b * N; ++t)
        xd[t] = bcq_ref_half_to_double(X[t]);
    int failed = 0;
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)N);
        if (!wrow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t m = 0; m < M; ++m) {
            if (!wrow)
                continue;
            dequant_row(planes, alpha, z, M, N, q, g, m, wrow);
            for (int64_t j = 0; j < b; ++j) {
                double acc = 0.0;
                for (int64_t k = 0; k < N; ++k)
                    acc += wrow[k] * xd[j * N + k];
                Y[j * M + m] = acc;
            }
        }
        free(wrow);
    }
    free(xd);
    return failed;
}

/* Independent second evaluation, in the grouped order of Eq. 11 and with its
 * own unpacking (byte-wise, via shifts on the byte index): per group, the
 * signed activation sum of each plane is scaled by its alpha; the offset
 * multiplies the plain activation sum of the group.  No dense W. */
int bcq_ref_brute(const uint32_t *planes, const uint16_t *alpha,
                  const uint16_t *z, const uint16_t *X, int64_t M, int64_t N,
                  int q, int64_t g, int64_t b, double *Y)
{
    if (!planes || !alpha || !X || !Y || b <= 0 || bad_shape(M, N, q, g))
        return 1;
    const uint8_t *bytes = (const uint8_t *)planes; /* little-endian host */
    int64_t G = N / g;
    for (int64_t j = 0; j < b; ++j) {
        for (int64_t m = 0; m < M; ++m) {
            double y = 0.0;
            for (int64_t grp = 0; grp < G; ++grp) {
                double xsum = 0.0;
                for (int64_t k = grp * g; k < (grp + 1) * g; ++k)
                    xsum += bcq_ref_half_to_double(X[j * N + k]);
                for (int i = 0; i < q; ++i) {
                    const uint8_t *row = bytes + (((int64_t)i * M + m) * (N / 8));
                    double ssum = 0.0;
                    for (int64_t k = grp * g; k < (grp + 1) * g; ++k) {
                        int bit = (row[k / 8] >> (k % 8)) & 1;
                        double xv = bcq_ref_half_to_double(X[j * N + k]);
                        ssum += bit ? xv : -xv;
                    }
                    y += bcq_ref_half_to_double(alpha[(m * G + grp) * q + i]) * ssum;
                }
                if (z)
                    y += bcq_ref_half_to_double(z[m * G + grp]) * xsum;
            }
            Y[j * M + m] = y;
        }
    }
    return 0;
}

/* Number of threads the parallel loops above will use. */
int bcq_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void bcq_ref_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}
