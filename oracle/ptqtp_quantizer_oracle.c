/*
 * CPU oracle for the PTQTP quantizer (paper, Sec. "Dual Trit-planes Approximation" and
 * "Progressive Optimization"; Alg. "Approximation Process of PTQTP" and Alg. "Progressive and
 * Adaptive Regularization"; appendix "Implementation Details").
 *
 * TEST INFRASTRUCTURE ONLY: shares no code with the HIP library; nothing in the product path
 * may call it.
 *
 * The method is an iteration, so this follows the algorithm's steps in the paper's order, one
 * (row, group) unit at a time ("Batch Processing": W is reshaped to rows of G entries and every
 * such row is decomposed on its own):
 *
 *   init   T1 = T2 = sign(w) with 0 -> +1, alpha = [1, 1], lambda = 1e-8
 *   repeat t = 1 .. T_max
 *     S = [T1' T2'],  A = S'S + lambda I2,  b = S'w                         (ridge normal equations)
 *     kappa = ||A||_F * ||A^-1||_F;  if kappa >= 1e6: lambda <- min(1, lambda * sqrt(kappa / 1e6))
 *            and A is rebuilt with the new lambda     (reading: lambda is raised BEFORE the solve,
 *            as the appendix text says; the algorithm listing shows the update after it)
 *     alpha = A^-1 b     by the closed-form 2x2 inverse (appendix "Computational Complexity")
 *     every element: (T1, T2) <- argmin over the 9 pairs (c1, c2) in {-1,0,1}^2 of
 *            (w - alpha1 c1 - alpha2 c2)^2, first minimum in the order c1 = -1,0,1 (outer),
 *            c2 = -1,0,1 (inner)                       (reading: the paper leaves ties open)
 *     stop when || alpha_t - alpha_(t-1) ||_F over the whole matrix < eps   (second listing)
 *
 * Precision.  Everything is binary64, one operation at a time (this file is compiled with
 * -ffp-contract=off, so no fused multiply-add changes a rounding): the trit choice is an integer
 * decided by floating point, and the GPU kernel that is checked against this file performs the
 * same binary64 operations in the same order, so both sides reach the same bits.  The only long
 * sums, b = S'w, are accumulated exactly in 64-bit integers (w is binary16: w * 2^24 is an
 * integer below 2^40) and converted once.  The convergence norm is accumulated in index order.
 *
 * Pins (tests/, -m "not gpu"): zero iterations return the initialisation; the first solve against
 * its closed form (identical planes: alpha1 = alpha2 = sum|w| / (2G + lambda), lambda raised once before
 * the solve); alpha against an independent solution of the ridge normal equations at every iteration;
 * every trit pair against brute force over the nine candidates; the tie order on exact ties; the
 * error never increasing in the trit step (the monotonicity the paper states); exactly ternary rows
 * recovered; exact invariance under power-of-two scaling; equivariance under permutations inside a
 * group; independence of units with a global stopping rule; the binary16 rounding against numpy's
 * on every finite value and every exact tie; the stopping rule on a run whose changes straddle eps
 * between the norm and its square.  A further test plants one mistake at a time in a copy of this
 * file (a dropped term, a wrong sign or index, a changed constant) and requires a pin to fail.
 * What the paper leaves open (the order of the lambda update, the order of ties, which of the two
 * stopping rules) is a reading, not a pin.  The cap lambda_max = 1 cannot be reached from the
 * prescribed start at G = 128 (one raise multiplies lambda by sqrt(kappa / 1e6), and kappa is about
 * 2G / lambda: the fixed point is 2G / 1e6); it is pinned on one unit of 2^20 equal weights, where
 * T1 = T2 stays a fixed point of the search and lambda climbs from 1e-8 to the cap in five raises.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#define QO_OK 0
#define QO_ERR_SHAPE 1

static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, frac = h & 0x3ff;
    double v;
    if (e == 0) v = ldexp((double)frac, -24);
    else if (e == 31) v = frac ? NAN : INFINITY;
    else v = ldexp((double)(1024 + frac), e - 25);
    return sign ? -v : v;
}

/* w * 2^24 as an exact integer (w finite binary16) */
static int64_t half_bits_to_fixed(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, frac = h & 0x3ff;
    int64_t v;
    if (e == 0) v = frac;
    else v = (int64_t)(1024 + frac) << (e - 1);
    return sign ? -v : v;
}

/* binary64 -> binary16 bits, ONE rounding to nearest even (storage of alpha: the memory model
 * keeps the scales in FP16) */
static uint16_t double_to_half_bits(double f)
{
    union { double f; uint64_t u; } v = { f };
    const uint16_t sign = (uint16_t)((v.u >> 48) & 0x8000u);
    const uint64_t absu = v.u & 0x7fffffffffffffffull;
    if (absu > 0x7ff0000000000000ull) return (uint16_t)(sign | 0x7e00u);          /* NaN */
    const double a = fabs(f);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);                          /* rounds to infinity */
    /* the binary16 grid around a: spacing 2^(e-10) for normals (e >= -14), 2^-24 below */
    int e;
    (void)frexp(a, &e);                                                           /* a = m * 2^e, m in [0.5, 1) */
    e -= 1;                                                                       /* a in [2^e, 2^(e+1)) */
    if (e < -14 || a == 0.0) e = -14;                                             /* subnormal range, zero */
    const double q = ldexp(a, 10 - e);                                            /* exact: in units of the spacing */
    double r = floor(q);
    const double rem = q - r;                                                     /* exact */
    if (rem > 0.5 || (rem == 0.5 && fmod(r, 2.0) == 1.0)) r += 1.0;
    uint32_t units = (uint32_t)r;                                                 /* 0 .. 2048 */
    uint32_t out;
    if (e == -14 && units < 1024u) out = units;                                   /* subnormal or zero */
    else {
        if (units == 2048u) { units = 1024u; e += 1; }
        out = (uint32_t)((e + 15) << 10) + (units - 1024u);
    }
    return (uint16_t)(sign | out);
}

/* one ridge solve + trit search for one unit of G entries; returns the squared change of alpha */
static double unit_iteration(const uint16_t *w16, int G, int8_t *t1, int8_t *t2, double *alpha, double *lambda)
{
    int s11 = 0, s22 = 0, s12 = 0;
    int64_t B1 = 0, B2 = 0;
    for (int j = 0; j < G; ++j) {
        int64_t wf = half_bits_to_fixed(w16[j]);
        s11 += t1[j] * t1[j];
        s22 += t2[j] * t2[j];
        s12 += t1[j] * t2[j];
        B1 += t1[j] * wf;
        B2 += t2[j] * wf;
    }
    const double b1 = ldexp((double)B1, -24), b2 = ldexp((double)B2, -24);     /* exact */
    double lam = *lambda;
    const double A12 = (double)s12;
    double A11 = (double)s11 + lam, A22 = (double)s22 + lam;
    double p = A11 * A22;
    const double qq = A12 * A12;
    double det = p - qq;
    /* A^-1 = (1 / det) * [[A22, -A12], [-A12, A11]]  (closed form of the appendix), kappa = ||A||_F * ||A^-1||_F */
    double sq = A11 * A11;
    sq = sq + A12 * A12;
    sq = sq + A12 * A12;
    sq = sq + A22 * A22;
    const double nA = sqrt(sq);
    double rdet = 1.0 / det;
    double i11 = A22 * rdet, i12 = -A12 * rdet, i22 = A11 * rdet;
    double si = i11 * i11;
    si = si + i12 * i12;
    si = si + i12 * i12;
    si = si + i22 * i22;
    const double nAi = sqrt(si);
    const double kappa = nA * nAi;
    if (!(kappa < 1.0e6)) {                       /* also taken when kappa is inf or NaN (det == 0) */
        const double grow = sqrt(kappa / 1.0e6);
        double nl = lam * grow;
        if (!(nl <= 1.0)) nl = 1.0;               /* lambda_max = 1, also for inf / NaN */
        lam = nl;
        A11 = (double)s11 + lam;
        A22 = (double)s22 + lam;
        p = A11 * A22;
        det = p - qq;
        rdet = 1.0 / det;
        i11 = A22 * rdet;
        i12 = -A12 * rdet;
        i22 = A11 * rdet;
    }
    *lambda = lam;
    /* alpha = A^-1 b */
    const double m11 = i11 * b1, m12 = i12 * b2;
    const double m21 = i12 * b1, m22 = i22 * b2;
    const double a1 = m11 + m12, a2 = m21 + m22;
    for (int j = 0; j < G; ++j) {
        const double w = half_bits_to_double(w16[j]);
        double best = INFINITY;
        int bc1 = 0, bc2 = 0;
        for (int c1 = -1; c1 <= 1; ++c1)
            for (int c2 = -1; c2 <= 1; ++c2) {
                const double v = (double)c1 * a1 + (double)c2 * a2;   /* products by -1, 0, 1 are exact */
                const double d = w - v;
                const double e = d * d;
                if (e < best) { best = e; bc1 = c1; bc2 = c2; }
            }
        t1[j] = (int8_t)bc1;
        t2[j] = (int8_t)bc2;
    }
    const double d1 = a1 - alpha[0], d2 = a2 - alpha[1];
    alpha[0] = a1;
    alpha[1] = a2;
    const double q1 = d1 * d1, q2 = d2 * d2;
    return q1 + q2;
}

/*
 * W: binary16 bits [N, K] row-major.  Outputs T1, T2 int8 [N, K]; a1_f64, a2_f64 double [N, K/G]
 * (the iteration's alpha); a1_h, a2_h binary16 bits of the same (what is stored).  Returns the number
 * of iterations performed in *iters and, if asked, the per-unit lambda.  max_iters >= 0 (0 returns the
 * initial state), eps >= 0.
 */
int ptqtp_oracle_quantize(const uint16_t *W, int64_t N, int64_t K, int64_t G, int max_iters, double eps,
                          int8_t *T1, int8_t *T2, double *a1_f64, double *a2_f64, uint16_t *a1_h, uint16_t *a2_h,
                          double *lambda_out /* [N*K/G] or NULL */, int *iters)
{
    if (N <= 0 || K <= 0 || G <= 0 || K % G != 0 || max_iters < 0) return QO_ERR_SHAPE;
    const int64_t NG = K / G, units = N * NG;
    double *lambda = (double *)malloc(sizeof(double) * (size_t)units);
    double *alpha = (double *)malloc(sizeof(double) * 2 * (size_t)units);
    if (!lambda || !alpha) { free(lambda); free(alpha); return QO_ERR_SHAPE; }
    for (int64_t i = 0; i < N * K; ++i) {
        const double w = half_bits_to_double(W[i]);
        const int8_t s = (int8_t)(w < 0.0 ? -1 : 1);          /* sign(w) with 0 -> +1 */
        T1[i] = s;
        T2[i] = s;
    }
    for (int64_t u = 0; u < units; ++u) { lambda[u] = 1.0e-8; alpha[2 * u] = 1.0; alpha[2 * u + 1] = 1.0; }
    int t = 0;
    while (t < max_iters) {
        double sum = 0.0;
        for (int64_t u = 0; u < units; ++u) {
            const int64_t n = u / NG, g = u % NG, off = n * K + g * G;
            sum += unit_iteration(W + off, (int)G, T1 + off, T2 + off, alpha + 2 * u, lambda + u);
        }
        ++t;
        if (sqrt(sum) < eps) break;
    }
    for (int64_t u = 0; u < units; ++u) {
        a1_f64[u] = alpha[2 * u];
        a2_f64[u] = alpha[2 * u + 1];
        a1_h[u] = double_to_half_bits(alpha[2 * u]);
        a2_h[u] = double_to_half_bits(alpha[2 * u + 1]);
    }
    if (lambda_out) for (int64_t u = 0; u < units; ++u) lambda_out[u] = lambda[u];
    *iters = t;
    free(lambda);
    free(alpha);
    return QO_OK;
}

uint16_t ptqtp_oracle_double_to_half_bits(double f) { return double_to_half_bits(f); }
