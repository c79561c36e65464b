/*
 * CPU oracle for the dual trit-plane linear layer (PTQTP decode hot path).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition the
 * HIP kernels are checked against.  It shares no code, header, table or helper
 * with the GPU library, and nothing in the product path may call it.
 *
 * What it computes (paper, Sec. "Magnitude-Topology Decoupling", Eq. 1-2, with
 * the group-wise scales of paragraph "Batch Processing", G columns per group):
 *
 *     W^  = diag-by-group(alpha1) * T1 + diag-by-group(alpha2) * T2
 *     y[m,n] = sum_k W^[n,k] * x[m,k]
 *
 * evaluated in the scale-after-plane-product order of Eq. 1:
 *
 *     y[m,n] = sum_g ( alpha1[n,g] * sum_{k in g} T1[n,k] x[m,k]
 *                    + alpha2[n,g] * sum_{k in g} T2[n,k] x[m,k] )
 *
 * The method is a re-association of this sum (Sec. "Inference Efficiency":
 * a product with a trit is a sign flip, a copy or a zero), so the oracle is the
 * definition itself, in index order, in double precision.  alpha and x arrive
 * as IEEE binary16 bit patterns and are widened exactly.
 *
 * Also here: the canonical 2-bit storage of a trit plane (Appendix "memory
 * model": each trit plane is stored as a 2-bit datatype), four trits per byte.
 *
 * Pins (tests/, -m "not gpu"): dense reconstruction + library matmul, brute
 * force on hand-sized inputs, unit-vector probes, linearity, group locality,
 * the closed-form byte count, exhaustive pack/unpack round trip, and the
 * binary16 decoder against every one of the 65536 bit patterns.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>

#define ORACLE_OK          0
#define ORACLE_ERR_SHAPE   1   /* non-positive size or K not a multiple of the group */
#define ORACLE_ERR_TRIT    2   /* a plane entry outside {-1, 0, +1} */
#define ORACLE_ERR_CODE    3   /* canonical byte stream holds the unused 2-bit code */

/* IEEE 754 binary16 -> binary64, exact (subnormals, infinities, NaN included). */
double ptqtp_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e    = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (e == 0)        v = ldexp((double)frac, -24);              /* zero / subnormal */
    else if (e == 31)  v = frac ? NAN : INFINITY;
    else               v = ldexp((double)(1024 + frac), e - 25);  /* 1.f * 2^(e-15) */
    return sign ? -v : v;
}

static int check_planes(const int8_t *T1, const int8_t *T2, int64_t count)
{
    for (int64_t i = 0; i < count; ++i) {
        if (T1[i] < -1 || T1[i] > 1 || T2[i] < -1 || T2[i] > 1) return ORACLE_ERR_TRIT;
    }
    return ORACLE_OK;
}

/*
 * Forward pass with fp64 activations (the fp16 entry point below widens and
 * calls this; linearity tests call it directly with arbitrary doubles).
 *
 *   T1, T2 : [N, K] row-major int8 trits
 *   a1, a2 : [N, K/G] row-major binary16 bit patterns
 *   x      : [M, K] row-major double
 *   y      : [M, N] row-major double, overwritten
 *   bound  : [M, N] or NULL; receives the L1 bound
 *            sum_k (|alpha1 T1| + |alpha2 T2|)[n,k] * |x[m,k]|
 *   threads: OpenMP threads over output rows n (1 = serial)
 */
int ptqtp_oracle_forward_f64x(const int8_t *T1, const int8_t *T2,
                              const uint16_t *a1, const uint16_t *a2,
                              const double *x,
                              int64_t M, int64_t N, int64_t K, int64_t G,
                              double *y, double *bound, int threads)
{
    if (M <= 0 || N <= 0 || K <= 0 || G <= 0 || K % G != 0) return ORACLE_ERR_SHAPE;
    int rc = check_planes(T1, T2, N * K);
    if (rc != ORACLE_OK) return rc;
    const int64_t NG = K / G;
    if (threads < 1) threads = 1;

#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const int8_t *t1 = T1 + n * K;
        const int8_t *t2 = T2 + n * K;
        for (int64_t m = 0; m < M; ++m) {
            const double *xm = x + m * K;
            double acc = 0.0, bnd = 0.0;
            for (int64_t g = 0; g < NG; ++g) {
                double s1 = 0.0, s2 = 0.0, b1 = 0.0, b2 = 0.0;
                for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                    s1 += (double)t1[k] * xm[k];
                    s2 += (double)t2[k] * xm[k];
                    b1 += fabs((double)t1[k]) * fabs(xm[k]);
                    b2 += fabs((double)t2[k]) * fabs(xm[k]);
                }
                double al1 = ptqtp_oracle_half_to_double(a1[n * NG + g]);
                double al2 = ptqtp_oracle_half_to_double(a2[n * NG + g]);
                acc += al1 * s1 + al2 * s2;
                bnd += fabs(al1) * b1 + fabs(al2) * b2;
            }
            y[m * N + n] = acc;
            if (bound) bound[m * N + n] = bnd;
        }
    }
    return ORACLE_OK;
}

/* Same, with x given as binary16 bit patterns [M, K] (the layer's real input type). */
int ptqtp_oracle_forward(const int8_t *T1, const int8_t *T2,
                         const uint16_t *a1, const uint16_t *a2,
                         const uint16_t *x16, double *x_scratch /* [M*K] */,
                         int64_t M, int64_t N, int64_t K, int64_t G,
                         double *y, double *bound, int threads)
{
    if (M <= 0 || K <= 0) return ORACLE_ERR_SHAPE;
    for (int64_t i = 0; i < M * K; ++i) x_scratch[i] = ptqtp_oracle_half_to_double(x16[i]);
    return ptqtp_oracle_forward_f64x(T1, T2, a1, a2, x_scratch, M, N, K, G, y, bound, threads);
}

/*
 * Canonical 2-bit storage of one trit plane: row-major, byte b of row n holds
 * trits 4b .. 4b+3 in bit fields [1:0], [3:2], [5:4], [7:6].
 * Code: 00 -> 0, 01 -> +1, 11 -> -1 (2-bit two's complement); 10 is unused.
 * K must be a multiple of 4.  out has N*K/4 bytes.
 */
int ptqtp_oracle_pack_canonical(const int8_t *T, int64_t N, int64_t K, uint8_t *out)
{
    if (N <= 0 || K <= 0 || K % 4 != 0) return ORACLE_ERR_SHAPE;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t b = 0; b < K / 4; ++b) {
            unsigned byte = 0;
            for (int j = 0; j < 4; ++j) {
                int t = T[n * K + 4 * b + j];
                if (t < -1 || t > 1) return ORACLE_ERR_TRIT;
                unsigned code = (unsigned)t & 3u;      /* -1 -> 11, 0 -> 00, +1 -> 01 */
                byte |= code << (2 * j);
            }
            out[n * (K / 4) + b] = (uint8_t)byte;
        }
    }
    return ORACLE_OK;
}

int ptqtp_oracle_unpack_canonical(const uint8_t *in, int64_t N, int64_t K, int8_t *T)
{
    if (N <= 0 || K <= 0 || K % 4 != 0) return ORACLE_ERR_SHAPE;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t b = 0; b < K / 4; ++b) {
            unsigned byte = in[n * (K / 4) + b];
            for (int j = 0; j < 4; ++j) {
                unsigned code = (byte >> (2 * j)) & 3u;
                if (code == 2u) return ORACLE_ERR_CODE;
                T[n * K + 4 * b + j] = (int8_t)(code == 3u ? -1 : (int)code);
            }
        }
    }
    return ORACLE_OK;
}

/*
 * Storage of one quantised linear layer in bits (Appendix "memory model",
 * M_PTQTP): two planes at 2 bits per entry plus two binary16 scales per
 * (row, group):  2*n*d*2 + ceil(d/G)*2n*16.
 */
int64_t ptqtp_oracle_model_bits(int64_t n, int64_t d, int64_t G)
{
    int64_t groups = (d + G - 1) / G;
    return 2 * n * d * 2 + groups * 2 * n * 16;
}
