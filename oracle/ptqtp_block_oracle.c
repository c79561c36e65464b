/*
 * CPU oracle for the steps either side of the trit-plane linears inside one
 * decoder block at decode time -- TEST INFRASTRUCTURE ONLY (see ptqtp_oracle.c;
 * shares nothing with the HIP library, nothing in the product path calls it).
 *
 * The paper replaces every linear projection of LLaMA-family decoder blocks
 * (Sec. "Experiments", setup paragraph) and leaves the rest of the block as
 * published for that family: a bias-free gated MLP
 *
 *     mlp(x) = W_down ( silu(W_gate x) * W_up x ),    silu(z) = z / (1 + exp(-z))
 *
 * and a residual stream that adds each sublayer's output to its input.  The
 * oracle is those definitions in binary64, one element at a time:
 *
 *   ptqtp_oracle_silu(z)           z / (1 + exp(-z))
 *   ptqtp_oracle_swiglu            h[m,i] = silu(y[m,i]) * y[m,I+i] for the output y [M, 2I] of a
 *                                  stacked (gate rows first, then up rows) linear
 *   ptqtp_oracle_residual_add      out[m,n] = y[m,n] + r[m,n], r given as binary16 bit patterns
 *   ptqtp_oracle_round_half        one rounding binary64 -> binary16 (nearest even), returned widened
 *
 * Pins (tests/, -m "not gpu"): silu(0) = 0, silu(z) - silu(-z) = z, the limits for large |z|,
 * the location and value of the minimum, a library sigmoid, a library silu on a dense
 * reconstruction of the whole MLP, gate/up order, and the rounding against numpy's.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>

double ptqtp_oracle_silu(double z)
{
    return z / (1.0 + exp(-z));
}

int ptqtp_oracle_swiglu(const double *y, int64_t M, int64_t I, double *h)
{
    if (M <= 0 || I <= 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t i = 0; i < I; ++i)
            h[m * I + i] = ptqtp_oracle_silu(y[m * 2 * I + i]) * y[m * 2 * I + I + i];
    return 0;
}

/* widen a binary16 bit pattern (finite values, zero, subnormals) */
static double half_bits_to_double(uint16_t hb)
{
    int sign = (hb >> 15) & 1, e = (hb >> 10) & 0x1f, frac = hb & 0x3ff;
    double v;
    if (e == 0)       v = ldexp((double)frac, -24);
    else if (e == 31) v = frac ? NAN : INFINITY;
    else              v = ldexp((double)(1024 + frac), e - 25);
    return sign ? -v : v;
}

int ptqtp_oracle_residual_add(const double *y, const uint16_t *r, int64_t count, double *out)
{
    if (count <= 0) return 1;
    for (int64_t i = 0; i < count; ++i) out[i] = y[i] + half_bits_to_double(r[i]);
    return 0;
}

/* binary64 -> nearest binary16 (ties to even), overflow to infinity, result widened again */
double ptqtp_oracle_round_half(double v)
{
    if (v != v) return v;
    double a = fabs(v);
    if (a == 0.0) return v;
    int e;
    (void)frexp(a, &e);               /* a = f * 2^e, f in [0.5, 1) : exponent of the leading bit is e-1 */
    int lead = e - 1;
    if (lead < -14) lead = -14;       /* subnormal range: fixed quantum 2^-24 */
    double quantum = ldexp(1.0, lead - 10);
    double q = nearbyint(a / quantum) * quantum;   /* default rounding mode: nearest even; the division is exact */
    if (q >= 65520.0) q = INFINITY;
    return v < 0 ? -q : q;
}

void ptqtp_oracle_round_half_array(const double *v, int64_t count, double *out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = ptqtp_oracle_round_half(v[i]);
}
