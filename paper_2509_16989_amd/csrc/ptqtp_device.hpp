// Device-side pieces shared by the translation units of libptqtp: record geometry, vector types,
// the 2-bit -> fp16 expansion, the per-group MFMA sum and the global-memory load helpers.
// The record layout itself is described at the top of ptqtp.hip.
#ifndef PTQTP_DEVICE_HPP
#define PTQTP_DEVICE_HPP
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kHeaderBytes = 256;
constexpr int kTileRows = 16;
constexpr int kStepK = 256;
constexpr int kPlaneBytes = 1024;
constexpr int kRecordBytes = 2 * kPlaneBytes + 128;
constexpr uint64_t kMagic = 0x3130765054515450ull;  // "PTQTPv01" little-endian
constexpr uint32_t kLayoutId = 3;

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float half_bits_to_float(uint32_t bits16) {
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(bits16)));
}

// Field F of four packed words -> eight fp16 values in {0, +1, -1}: one lane's MFMA B operand.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
template <int F>
__device__ __forceinline__ half8 decode_field(uintx4 w) {
    const uint32_t word = (F >> 1) == 0 ? w.x : (F >> 1) == 1 ? w.y : (F >> 1) == 2 ? w.z : w.w;
    const uint32_t fp4 = ((F & 1) ? (word << 1) : word) & 0xAAAAAAAAu;
    const half2v h0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 0);
    const half2v h1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 1);
    const half2v h2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 2);
    const half2v h3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 3);
    return half8{h0.x, h0.y, h1.x, h1.y, h2.x, h2.y, h3.x, h3.y};
}

// One (plane, 128-column group): four MFMAs of 16 tokens x 16 rows x 32 columns each.
template <int MT, int G2>
__device__ __forceinline__ void group_sum(const uintx4 (&xa)[MT][8], uintx4 p, floatx4 (&acc)[MT]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    half8 b;
    b = decode_field<G2 * 4 + 0>(p);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[mt][G2 * 4 + 0]), b, acc[mt], 0, 0, 0);
    b = decode_field<G2 * 4 + 1>(p);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[mt][G2 * 4 + 1]), b, acc[mt], 0, 0, 0);
    b = decode_field<G2 * 4 + 2>(p);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[mt][G2 * 4 + 2]), b, acc[mt], 0, 0, 0);
    b = decode_field<G2 * 4 + 3>(p);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[mt][G2 * 4 + 3]), b, acc[mt], 0, 0, 0);
}

// Load through the global address space (descriptor pointers come out of memory and would
// otherwise be treated as generic: flat loads tie up the LDS counter as well).
template <class T>
__device__ __forceinline__ T load_global(const void *p) {
    return *(const __attribute__((address_space(1))) T *)(p);
}
// Same, marked non-temporal: the packed records are read exactly once per call and must not
// push the activations (re-read by every workgroup) out of L2.
template <class T>
__device__ __forceinline__ T load_stream(const void *p) {
    return __builtin_nontemporal_load((const __attribute__((address_space(1))) T *)(p));
}

struct StepRegs {             // one record + its activation slice
    uintx4 p1, p2;
    uintx2 sc, xr;
};

}  // namespace
#endif  // PTQTP_DEVICE_HPP
