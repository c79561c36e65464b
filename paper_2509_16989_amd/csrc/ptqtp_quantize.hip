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
// Mapping: 16 units per wave (four lanes x 32 elements per unit), state (trits) in HBM between iterations:
// 6 bytes per weight per iteration (2 read for w, 2 read + 2 written for the trit pair).  The kernel is
// bound by vector-ALU issue, not by that traffic: about 60 instructions per weight and iteration, of which
// the nine-candidate search takes 43 (subtract, square, compare, minimum, select per candidate).
// The sums S'S are small integers; S'w is summed in binary64, which is exact in any order here (every
// term is a multiple of 2^-24 below 2^16 in magnitude), so it equals the integer sum an exact
// implementation would form; the 2x2 solve and the search
// run in binary64, one operation at a time with contraction off, so the integer decisions are
// reproducible bit for bit.  The stopping rule needs a matrix-wide sum: every iteration is two
// launches (units, then a fixed-order reduction that sets a device flag); later launches see the
// flag and return at once, so the host never synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>

#include "ptqtp.h"

namespace {

constexpr int kGroup = 128;

struct QuantFlags {          // start of the workspace, 256 bytes
    int32_t done;            // set when the stopping rule fired
    int32_t iters;           // iterations performed so far
    int32_t pad[62];
};

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

typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// sums over the four lanes that share a unit (lanes 4i .. 4i+3)
__device__ __forceinline__ int quad_sum_i32(int v) {
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    return v;
}
__device__ __forceinline__ double quad_sum_f64(double v) {
#pragma unroll
    for (int o = 1; o <= 2; o <<= 1) {
        const uint64_t bits = __builtin_bit_cast(uint64_t, v);
        const int lo = __shfl_xor(static_cast<int>(bits & 0xffffffffu), o, 64);
        const int hi = __shfl_xor(static_cast<int>(bits >> 32), o, 64);
        v = v + __builtin_bit_cast(double, (static_cast<uint64_t>(static_cast<uint32_t>(hi)) << 32) | static_cast<uint32_t>(lo));
    }
    return v;
}


// One iteration for every unit.  A wave holds 16 units: lane l works on elements (l%4)*32 .. +31 of
// unit l/4, so the 2x2 solve (the same for all lanes of a unit) is repeated 4 times, not 64.
// FIRST: the state is the initialisation (no trits in memory yet).
template <bool FIRST>
__global__ void __launch_bounds__(256)
quant_iter_kernel(const uint16_t *__restrict__ W, int8_t *__restrict__ T1, int8_t *__restrict__ T2,
                  double *__restrict__ alpha, double *__restrict__ lambda, double *__restrict__ delta2,
                  const QuantFlags *__restrict__ flags, int64_t units, int64_t NG, int64_t K)
{
#pragma clang fp contract(off)
    if (flags->done) return;
    const int lane = threadIdx.x & 63, part = lane & 3;
    const int64_t u_raw = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * 16 + (lane >> 2);
    const bool valid = u_raw < units;
    const int64_t u = valid ? u_raw : units - 1;       // idle lanes shadow the last unit and store nothing
    const int64_t n = u / NG, g = u % NG;
    const int64_t off = n * K + g * kGroup + part * 32;

    uint32_t wv[16];                                   // 32 fp16 weights
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uintx4 v = *reinterpret_cast<const uintx4 *>(W + off + 8 * i);
        wv[4 * i] = v.x; wv[4 * i + 1] = v.y; wv[4 * i + 2] = v.z; wv[4 * i + 3] = v.w;
    }
    uint32_t tv1[8], tv2[8];                           // 32 trits per plane, one byte each
    double lam, ap1, ap2;
    if (FIRST) {
        lam = 1.0e-8; ap1 = 1.0; ap2 = 1.0;
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uintx4 a = *reinterpret_cast<const uintx4 *>(T1 + off + 16 * i);
            const uintx4 b = *reinterpret_cast<const uintx4 *>(T2 + off + 16 * i);
            tv1[4 * i] = a.x; tv1[4 * i + 1] = a.y; tv1[4 * i + 2] = a.z; tv1[4 * i + 3] = a.w;
            tv2[4 * i] = b.x; tv2[4 * i + 1] = b.y; tv2[4 * i + 2] = b.z; tv2[4 * i + 3] = b.w;
        }
        lam = lambda[u]; ap1 = alpha[2 * u]; ap2 = alpha[2 * u + 1];
    }

    // S'w in binary64 is exact in any order: every term t * w is a multiple of 2^-24 (w is binary16), and so
    // is every partial sum, which stays below 128 * 65504 < 2^23: at most 47 significant bits.
    int s11 = 0, s22 = 0, s12 = 0;
    double b1 = 0.0, b2 = 0.0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const uint32_t h = (wv[e >> 1] >> (16 * (e & 1))) & 0xffffu;
        int t1, t2;
        if (FIRST) {
            t1 = t2 = ((h & 0x8000u) && (h & 0x7fffu)) ? -1 : 1;     // sign(w) with 0 -> +1; -0.0 counts as zero
        } else {
            t1 = static_cast<int8_t>((tv1[e >> 2] >> (8 * (e & 3))) & 0xffu);
            t2 = static_cast<int8_t>((tv2[e >> 2] >> (8 * (e & 3))) & 0xffu);
        }
        const double w = half_to_double(h);
        s11 += t1 * t1; s22 += t2 * t2; s12 += t1 * t2;
        b1 = __builtin_fma(static_cast<double>(t1), w, b1);          // exact, fused or not
        b2 = __builtin_fma(static_cast<double>(t2), w, b2);
    }
    // S'S: three small integers in one word (unit sums are at most 128 in magnitude; s12 is signed)
    const int ps = quad_sum_i32(s11 | (s22 << 10) | ((s12 + 32) << 20));
    s11 = ps & 0x3ff; s22 = (ps >> 10) & 0x3ff; s12 = ((ps >> 20) & 0x3ff) - 128;
    b1 = quad_sum_f64(b1); b2 = quad_sum_f64(b2);

    // ridge normal equations, closed-form inverse A^-1 = (1/det) adj(A), kappa = ||A||_F ||A^-1||_F
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
    double rdet = __ddiv_rn(1.0, det);
    double i11 = A22 * rdet, i12 = -A12 * rdet, i22 = A11 * rdet;
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
        rdet = __ddiv_rn(1.0, det);
        i11 = A22 * rdet;
        i12 = -A12 * rdet;
        i22 = A11 * rdet;
    }
    const double m11 = i11 * b1, m12 = i12 * b2;
    const double m21 = i12 * b1, m22 = i22 * b2;
    const double a1 = m11 + m12, a2 = m21 + m22;

    // nine candidate values in the order c1 = -1,0,1 (outer), c2 = -1,0,1 (inner)
    // Candidate 8 - m is the exact negative of candidate m (negation commutes with every rounding), and
    // w - (-v) is the same operation as w + v: five values are kept, four of them used with either sign.
    double cand[5];
#pragma unroll
    for (int m = 0; m < 5; ++m) cand[m] = static_cast<double>(m / 3 - 1) * a1 + static_cast<double>(m % 3 - 1) * a2;
    // Per element: the first minimum of the nine errors.  The winner is tracked as the byte pair it will be
    // stored as (c1 in bits 0..7, c2 in bits 8..15); four elements' pairs are then split into one word per plane.
    uint32_t o1[8], o2[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        uint32_t pair[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = 4 * q + i;
            const double w = half_to_double((wv[e >> 1] >> (16 * (e & 1))) & 0xffffu);
            const double d0 = w - cand[0];
            double best = d0 * d0;
            uint32_t code = 0xffffu;                                   // (-1, -1)
#pragma unroll
            for (int m = 1; m < 9; ++m) {
                const double d = m < 5 ? w - cand[m] : w + cand[8 - m];
                const double err = d * d;
                const uint32_t cm = (static_cast<uint32_t>(m / 3 - 1) & 0xffu) | ((static_cast<uint32_t>(m % 3 - 1) & 0xffu) << 8);
                code = err < best ? cm : code;
                best = __builtin_fmin(best, err);
            }
            pair[i] = code;
        }
        const uint32_t p01 = pair[0] | (pair[1] << 16), p23 = pair[2] | (pair[3] << 16);
        o1[q] = __builtin_amdgcn_perm(p23, p01, 0x06040200u);          // bytes 0, 2 of each pair word
        o2[q] = __builtin_amdgcn_perm(p23, p01, 0x07050301u);          // bytes 1, 3
    }
    if (valid) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<uintx4 *>(T1 + off + 16 * i) = uintx4{o1[4 * i], o1[4 * i + 1], o1[4 * i + 2], o1[4 * i + 3]};
            *reinterpret_cast<uintx4 *>(T2 + off + 16 * i) = uintx4{o2[4 * i], o2[4 * i + 1], o2[4 * i + 2], o2[4 * i + 3]};
        }
        if (part == 0) {
            alpha[2 * u] = a1;
            alpha[2 * u + 1] = a2;
            lambda[u] = lam;
        }
    }
    // this workgroup's share of || alpha_t - alpha_(t-1) ||_F^2: its 64 units in a fixed order
    // (wave butterfly, then the four waves in turn)
    double dsum = 0.0;
    if (valid && part == 0) {
        const double d1 = a1 - ap1, d2 = a2 - ap2;
        const double q1 = d1 * d1, q2 = d2 * d2;
        dsum = q1 + q2;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t bits = __builtin_bit_cast(uint64_t, dsum);
        const int lo = __shfl_xor(static_cast<int>(bits & 0xffffffffu), o, 64);
        const int hi = __shfl_xor(static_cast<int>(bits >> 32), o, 64);
        dsum = dsum + __builtin_bit_cast(double, (static_cast<uint64_t>(static_cast<uint32_t>(hi)) << 32) | static_cast<uint32_t>(lo));
    }
    __shared__ double wsum[4];
    if (lane == 0) wsum[threadIdx.x >> 6] = dsum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wsum[0];
        t = t + wsum[1];
        t = t + wsum[2];
        t = t + wsum[3];
        delta2[blockIdx.x] = t;
    }
}

// Stopping rule: || alpha_t - alpha_(t-1) ||_F < eps over all units.  The unit kernel leaves one partial
// sum per workgroup; here one workgroup adds them in a fixed order: thread i takes partials i, i+1024, ...,
// then a binary tree in LDS.
__global__ void __launch_bounds__(1024)
quant_check_kernel(const double *__restrict__ delta2, int64_t nparts, double eps, QuantFlags *flags, int t)
{
    __shared__ double part[1024];
    if (flags->done) return;
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < nparts; i += 1024) s += delta2[i];
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

// Workspace of ptqtp_quantize_static: one array per device the library is loaded on, held until the process ends.
// In host code the array's name is only a stand-in for the symbol; the device address comes from
// hipGetSymbolAddress, once per device, and is the only thing host code hands to kernels.
__device__ __align__(256) unsigned char scratch[PTQTP_QUANTIZE_STATIC_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (nullptr on failure)
void *scratch_address() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

// N and K up to 2^30 each and N * K up to 2^37 (a binary16 matrix of 275 GB): unit and element counts,
// and the grids derived from them, then fit 32 bits
static bool quantize_shape_ok(int64_t N, int64_t K, int32_t group) {
    return N > 0 && K > 0 && K % group == 0 && N <= (1ll << 30) && K <= (1ll << 30) && N * K <= (1ll << 37);
}

size_t ptqtp_quantize_workspace_bytes(int64_t N, int64_t K, int32_t group) {
    if (group != kGroup || !quantize_shape_ok(N, K, group)) return 0;
    const size_t units = static_cast<size_t>(N) * static_cast<size_t>(K / group);
    return sizeof(QuantFlags) + units * 4 * sizeof(double);      // alpha (2), lambda, delta2
}

// The decomposition itself, enqueued on `stream_` with its state in `workspace` (validated by the callers).
static ptqtp_status quantize_enqueue(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                                     int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, int32_t *iters, void *workspace,
                                     void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int64_t NG = K / group, units = N * NG;
    QuantFlags *flags = static_cast<QuantFlags *>(workspace);
    double *alpha = reinterpret_cast<double *>(flags + 1);
    double *lambda = alpha + 2 * units;
    double *delta2 = lambda + units;
    const unsigned ublocks = static_cast<unsigned>((units + 63) / 64);     // 4 waves x 16 units per workgroup
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
        hipLaunchKernelGGL(quant_check_kernel, dim3(1), dim3(1024), 0, stream, delta2, static_cast<int64_t>(ublocks), eps, flags, t);
    }
    hipLaunchKernelGGL(quant_finish_kernel, dim3(static_cast<unsigned>((units + 255) / 256)), dim3(256), 0, stream, alpha,
                       a1, a2, flags, iters, units);
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

static ptqtp_status quantize_check_args(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                                        const int8_t *T1, const int8_t *T2, const uint16_t *a1, const uint16_t *a2)
{
    if (!W || !T1 || !T2 || !a1 || !a2) return PTQTP_ERR_NULL;
    if (group != kGroup) return PTQTP_ERR_GROUP;
    if (!quantize_shape_ok(N, K, group) || max_iters < 0 || max_iters > 10000 || !(eps >= 0.0))
        return PTQTP_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(T1, 16) || !aligned(T2, 16) || !aligned(a1, 2) || !aligned(a2, 2))
        return PTQTP_ERR_ALIGN;
    return PTQTP_OK;
}

ptqtp_status ptqtp_quantize(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                            int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, int32_t *iters, void *workspace,
                            size_t workspace_bytes, void *stream_)
{
    if (!workspace) return PTQTP_ERR_NULL;
    const ptqtp_status st = quantize_check_args(W, N, K, group, max_iters, eps, T1, T2, a1, a2);
    if (st != PTQTP_OK) return st;
    if (workspace_bytes < ptqtp_quantize_workspace_bytes(N, K, group)) return PTQTP_ERR_SIZE;
    if (!aligned(workspace, 256)) return PTQTP_ERR_ALIGN;
    return quantize_enqueue(W, N, K, group, max_iters, eps, T1, T2, a1, a2, iters, workspace, stream_);
}

ptqtp_status ptqtp_quantize_static(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                                   int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, int32_t *iters, void *stream_)
{
    const ptqtp_status st = quantize_check_args(W, N, K, group, max_iters, eps, T1, T2, a1, a2);
    if (st != PTQTP_OK) return st;
    if (ptqtp_quantize_workspace_bytes(N, K, group) > PTQTP_QUANTIZE_STATIC_BYTES) return PTQTP_ERR_SIZE;
    void *ws = scratch_address();
    if (!ws) return PTQTP_ERR_HIP;
    // the array keeps the previous call's contents: quant_begin_kernel clears the flags, the first iteration (or
    // quant_init_state_kernel) writes every scale, lambda and partial sum before anything reads them
    return quantize_enqueue(W, N, K, group, max_iters, eps, T1, T2, a1, a2, iters, ws, stream_);
}

}  // extern "C"
