// PTQTP quantizer on MI355X: W (fp16) -> two trit planes + per-(row, group) scales.
//
// Paper: Sec. "Dual Trit-planes Approximation" (ridge normal equations A = S'S + lambda I2,
// b = S'w, alpha = A^-1 b), Sec. "Progressive Optimization" (kappa = ||A||_F ||A^-1||_F, lambda
// raised when kappa >= 1e6, capped at 1; per-element search over the nine pairs in {-1,0,1}^2),
// the two algorithm listings (initialisation T = sign(W) with 0 -> +1, alpha = [1,1],
// lambda = 1e-8; stop when the Frobenius norm of the change of all scales drops below eps) and
// the appendix closed-form 2x2 inverse.  One (row, 128-column group) unit is decomposed on its own
// ("Batch Processing").
//
// Mapping: one wave per unit, two elements per lane, state (trits) in HBM between iterations:
// 6 bytes per weight per iteration (2 read for w, 2 read + 2 written for the trit pair), so an
// iteration is HBM-bound like the forward path.  The sums S'S (small integers) and S'w (w * 2^24
// is an integer: exact in 64-bit) are wave reductions over integers; the 2x2 solve and the search
// run in binary64, one operation at a time with contraction off, so the integer decisions are
// reproducible bit for bit.  The stopping rule needs a matrix-wide sum: every iteration is two
// launches (units, then a fixed-order reduction that sets a device flag); later launches see the
// flag and return at once, so the host never synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ptqtp.h"

namespace {

constexpr int kGroup = 128;

struct QuantFlags {          // start of the workspace, 256 bytes
    int32_t done;            // set when the stopping rule fired
    int32_t iters;           // iterations performed so far
    int32_t pad[62];
};

__device__ __forceinline__ int64_t half_to_fixed24(uint32_t h) {       // w * 2^24, exact for finite w
    const int e = (h >> 10) & 0x1f;
    const int64_t frac = h & 0x3ff;
    int64_t v = e == 0 ? frac : ((frac | 0x400) << (e - 1));
    return (h & 0x8000u) ? -v : v;
}

__device__ __forceinline__ double half_to_double(uint32_t h) {
    return static_cast<double>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

// binary64 -> binary16 bits with ONE rounding to nearest even (a cast would round twice, via binary32)
__device__ __forceinline__ uint16_t double_to_half_rne(double f) {
    const uint64_t u = __builtin_bit_cast(uint64_t, f);
    const uint16_t sign = static_cast<uint16_t>((u >> 48) & 0x8000u);
    const int exp = static_cast<int>((u >> 52) & 0x7ff);
    const uint64_t mant = u & 0xfffffffffffffull;
    if (exp == 0x7ff) return static_cast<uint16_t>(sign | (mant ? 0x7e00u : 0x7c00u));
    if (exp == 0) return sign;                                  // binary64 zero / subnormal
    int e = exp - 1023;
    if (e > 15) return static_cast<uint16_t>(sign | 0x7c00u);
    const uint64_t m = mant | (1ull << 52);
    if (e >= -14) {
        uint64_t hm = m >> 42;
        const uint64_t rem = m & ((1ull << 42) - 1), half = 1ull << 41;
        if (rem > half || (rem == half && (hm & 1))) ++hm;
        if (hm == 2048) { hm = 1024; ++e; }
        if (e > 15) return static_cast<uint16_t>(sign | 0x7c00u);
        return static_cast<uint16_t>(sign | (static_cast<uint32_t>(e + 15) << 10) | static_cast<uint32_t>(hm - 1024));
    }
    const int shift = 28 - e;                                   // units of 2^-24
    if (shift > 54) return sign;
    uint64_t hm = m >> shift;
    const uint64_t rem = m & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (hm & 1))) ++hm;
    return static_cast<uint16_t>(sign | static_cast<uint32_t>(hm));
}

__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int lo = __shfl_xor(static_cast<int>(v & 0xffffffff), o, 64);
        const int hi = __shfl_xor(static_cast<int>(v >> 32), o, 64);
        v += (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
    }
    return v;
}

// One iteration for every unit.  FIRST: the state is the initialisation (no trits in memory yet).
template <bool FIRST>
__global__ void __launch_bounds__(256)
quant_iter_kernel(const uint16_t *__restrict__ W, int8_t *__restrict__ T1, int8_t *__restrict__ T2,
                  double *__restrict__ alpha, double *__restrict__ lambda, double *__restrict__ delta2,
                  const QuantFlags *__restrict__ flags, int64_t units, int64_t NG, int64_t K)
{
#pragma clang fp contract(off)
    if (flags->done) return;
    const int lane = threadIdx.x & 63;
    const int64_t u = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (u >= units) return;
    const int64_t n = u / NG, g = u % NG;
    const int64_t off = n * K + g * kGroup + 2 * lane;
    const uint32_t wp = *reinterpret_cast<const uint32_t *>(W + off);
    const uint32_t h0 = wp & 0xffffu, h1 = wp >> 16;
    int t10, t11, t20, t21;
    double lam, ap1, ap2;
    if (FIRST) {
        // sign(w) with 0 -> +1; -0.0 counts as zero
        t10 = t20 = ((h0 & 0x8000u) && (h0 & 0x7fffu)) ? -1 : 1;
        t11 = t21 = ((h1 & 0x8000u) && (h1 & 0x7fffu)) ? -1 : 1;
        lam = 1.0e-8; ap1 = 1.0; ap2 = 1.0;
    } else {
        const uint16_t p1 = *reinterpret_cast<const uint16_t *>(T1 + off);
        const uint16_t p2 = *reinterpret_cast<const uint16_t *>(T2 + off);
        t10 = static_cast<int8_t>(p1 & 0xff); t11 = static_cast<int8_t>(p1 >> 8);
        t20 = static_cast<int8_t>(p2 & 0xff); t21 = static_cast<int8_t>(p2 >> 8);
        lam = lambda[u]; ap1 = alpha[2 * u]; ap2 = alpha[2 * u + 1];
    }
    const int64_t f0 = half_to_fixed24(h0), f1 = half_to_fixed24(h1);
    // S'S: three small integers in one word (each sum is at most 128 in magnitude; s12 is signed)
    const int packed = (t10 * t10 + t11 * t11) | ((t20 * t20 + t21 * t21) << 10) | ((t10 * t20 + t11 * t21 + 2) << 20);
    const int ps = wave_sum_i32(packed);
    const int s11 = ps & 0x3ff, s22 = (ps >> 10) & 0x3ff, s12 = ((ps >> 20) & 0x3ff) - 2 * 64;
    const int64_t B1 = wave_sum_i64(t10 * f0 + t11 * f1), B2 = wave_sum_i64(t20 * f0 + t21 * f1);
    const double b1 = static_cast<double>(B1) * 0x1p-24, b2 = static_cast<double>(B2) * 0x1p-24;   // exact

    const double A12 = static_cast<double>(s12);
    double A11 = static_cast<double>(s11) + lam, A22 = static_cast<double>(s22) + lam;
    double p = A11 * A22;
    const double qq = A12 * A12;
    double det = p - qq;
    double sq = A11 * A11;
    sq = sq + A12 * A12;
    sq = sq + A12 * A12;
    sq = sq + A22 * A22;
    const double nA = __dsqrt_rn(sq);
    const double i11 = __ddiv_rn(A22, det), i12 = __ddiv_rn(-A12, det), i22 = __ddiv_rn(A11, det);
    double si = i11 * i11;
    si = si + i12 * i12;
    si = si + i12 * i12;
    si = si + i22 * i22;
    const double nAi = __dsqrt_rn(si);
    const double kappa = nA * nAi;
    if (!(kappa < 1.0e6)) {
        const double grow = __dsqrt_rn(__ddiv_rn(kappa, 1.0e6));
        double nl = lam * grow;
        if (!(nl <= 1.0)) nl = 1.0;
        lam = nl;
        A11 = static_cast<double>(s11) + lam;
        A22 = static_cast<double>(s22) + lam;
        p = A11 * A22;
        det = p - qq;
    }
    const double n1 = A22 * b1, n1b = A12 * b2;
    const double n2 = A11 * b2, n2b = A12 * b1;
    const double a1 = __ddiv_rn(n1 - n1b, det), a2 = __ddiv_rn(n2 - n2b, det);

    // nine candidate values in the order c1 = -1,0,1 (outer), c2 = -1,0,1 (inner)
    double cand[9];
#pragma unroll
    for (int c1 = -1; c1 <= 1; ++c1)
#pragma unroll
        for (int c2 = -1; c2 <= 1; ++c2) cand[(c1 + 1) * 3 + (c2 + 1)] = static_cast<double>(c1) * a1 + static_cast<double>(c2) * a2;
    uint32_t out1 = 0, out2 = 0;
#pragma unroll
    for (int el = 0; el < 2; ++el) {
        const double w = half_to_double(el ? h1 : h0);
        double best = __builtin_inf();
        int bm = 0;
#pragma unroll
        for (int m = 0; m < 9; ++m) {
            const double d = w - cand[m];
            const double e = d * d;
            if (e < best) { best = e; bm = m; }
        }
        const int c1 = bm / 3 - 1, c2 = bm % 3 - 1;
        out1 |= (static_cast<uint32_t>(c1) & 0xffu) << (8 * el);
        out2 |= (static_cast<uint32_t>(c2) & 0xffu) << (8 * el);
    }
    *reinterpret_cast<uint16_t *>(T1 + off) = static_cast<uint16_t>(out1);
    *reinterpret_cast<uint16_t *>(T2 + off) = static_cast<uint16_t>(out2);
    if (lane == 0) {
        const double d1 = a1 - ap1, d2 = a2 - ap2;
        const double q1 = d1 * d1, q2 = d2 * d2;
        alpha[2 * u] = a1;
        alpha[2 * u + 1] = a2;
        lambda[u] = lam;
        delta2[u] = q1 + q2;
    }
}

// Stopping rule: || alpha_t - alpha_(t-1) ||_F < eps over all units.  One workgroup, fixed order:
// thread i adds elements i, i+1024, ... , then a binary tree in LDS.
__global__ void __launch_bounds__(1024)
quant_check_kernel(const double *__restrict__ delta2, int64_t units, double eps, QuantFlags *flags, int t)
{
    __shared__ double part[1024];
    if (flags->done) return;
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < units; i += 1024) s += delta2[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (static_cast<int>(threadIdx.x) < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        flags->iters = t;
        if (__dsqrt_rn(part[0]) < eps) flags->done = 1;
    }
}

__global__ void quant_begin_kernel(QuantFlags *flags) {
    if (threadIdx.x == 0) { flags->done = 0; flags->iters = 0; }
}

// max_iters == 0: the initial state is the result
__global__ void __launch_bounds__(256)
quant_init_state_kernel(const uint16_t *__restrict__ W, int8_t *__restrict__ T1, int8_t *__restrict__ T2,
                        double *__restrict__ alpha, int64_t total, int64_t units)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < total) {
        const uint32_t h = W[i];
        const int8_t s = ((h & 0x8000u) && (h & 0x7fffu)) ? -1 : 1;
        T1[i] = s; T2[i] = s;
    }
    if (i < 2 * units) alpha[i] = 1.0;
}

__global__ void __launch_bounds__(256)
quant_finish_kernel(const double *__restrict__ alpha, uint16_t *__restrict__ a1, uint16_t *__restrict__ a2,
                    const QuantFlags *__restrict__ flags, int32_t *__restrict__ iters, int64_t units)
{
    const int64_t u = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (u < units) {
        a1[u] = double_to_half_rne(alpha[2 * u]);
        a2[u] = double_to_half_rne(alpha[2 * u + 1]);
    }
    if (u == 0 && iters) *iters = flags->iters;
}

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" {

size_t ptqtp_quantize_workspace_bytes(int64_t N, int64_t K, int32_t group) {
    if (group != kGroup || N <= 0 || K <= 0 || K % group != 0 || N > (1ll << 30) || K > (1ll << 30)) return 0;
    const size_t units = static_cast<size_t>(N) * static_cast<size_t>(K / group);
    return sizeof(QuantFlags) + units * 4 * sizeof(double);      // alpha (2), lambda, delta2
}

ptqtp_status ptqtp_quantize(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                            int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, int32_t *iters, void *workspace,
                            size_t workspace_bytes, void *stream_)
{
    if (!W || !T1 || !T2 || !a1 || !a2 || !workspace) return PTQTP_ERR_NULL;
    if (group != kGroup) return PTQTP_ERR_GROUP;
    if (N <= 0 || K <= 0 || K % group != 0 || N > (1ll << 30) || K > (1ll << 30) || max_iters < 0 || max_iters > 10000 ||
        !(eps >= 0.0))
        return PTQTP_ERR_SHAPE;
    const size_t need = ptqtp_quantize_workspace_bytes(N, K, group);
    if (workspace_bytes < need) return PTQTP_ERR_SIZE;
    if (!aligned(workspace, 256) || !aligned(W, 4) || !aligned(T1, 2) || !aligned(T2, 2) || !aligned(a1, 2) ||
        !aligned(a2, 2))
        return PTQTP_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int64_t NG = K / group, units = N * NG;
    QuantFlags *flags = static_cast<QuantFlags *>(workspace);
    double *alpha = reinterpret_cast<double *>(flags + 1);
    double *lambda = alpha + 2 * units;
    double *delta2 = lambda + units;
    const unsigned ublocks = static_cast<unsigned>((units + 3) / 4);
    hipLaunchKernelGGL(quant_begin_kernel, dim3(1), dim3(64), 0, stream, flags);
    if (max_iters == 0) {
        const int64_t total = N * K;
        hipLaunchKernelGGL(quant_init_state_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, stream,
                           W, T1, T2, alpha, total, units);
    }
    for (int t = 1; t <= max_iters; ++t) {
        if (t == 1)
            hipLaunchKernelGGL(quant_iter_kernel<true>, dim3(ublocks), dim3(256), 0, stream, W, T1, T2, alpha, lambda,
                               delta2, flags, units, NG, K);
        else
            hipLaunchKernelGGL(quant_iter_kernel<false>, dim3(ublocks), dim3(256), 0, stream, W, T1, T2, alpha, lambda,
                               delta2, flags, units, NG, K);
        hipLaunchKernelGGL(quant_check_kernel, dim3(1), dim3(1024), 0, stream, delta2, units, eps, flags, t);
    }
    hipLaunchKernelGGL(quant_finish_kernel, dim3(static_cast<unsigned>((units + 255) / 256)), dim3(256), 0, stream, alpha,
                       a1, a2, flags, iters, units);
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

}  // extern "C"
