// libptqtp: dual trit-plane linear layer for MI355X (gfx950, wave64, MFMA).
//
// y[m,n] = sum_g alpha1[n,g] * (T1[n,g,:] . x[m,g,:]) + alpha2[n,g] * (T2[n,g,:] . x[m,g,:])
// (paper, Eq. 1-2 with the group-wise scales of paragraph "Batch Processing").
//
// Device layout of the packed blob (layout id 3)
// ----------------------------------------------
//   [ 256-byte header ][ record(rt=0,ks=0) ][ record(rt=0,ks=1) ] ... [ record(rt=RT-1,ks=KS-1) ]
//   rt = 16-row tile (RT = ceil(N/16)), ks = 256-column step (KS = ceil(K/256)) = two scale groups.
//   One record = 2176 bytes = 17 cache lines of 128 B:
//     bytes    0..1023  plane 1, 64 lanes x 16 B   (one global_load_dwordx4 per wave)
//     bytes 1024..2047  plane 2, same shape
//     bytes 2048..2175  scales: row nl (0..15) -> {a1[g0], a1[g1], a2[g0], a2[g1]} fp16
//   Lane l = q*16 + nl holds 64 trits of row rt*16+nl in four 32-bit words.  Word i (0..3),
//   nibble j (0..7) holds two trits, A in bits (3,1) and B in bits (2,0) of the nibble, each as
//   (sign, nonzero): 0 -> 00, +1 -> 01, -1 -> 11.  With f = 2i for A and f = 2i+1 for B the trit
//   is column
//       k = ks*256 + (f/4)*128 + (f%4)*32 + q*8 + j
//   (the four quarter-lanes q of a row read 64 contiguous bytes of x per field)
//   `w & 0xAAAAAAAA` (A) and `(w << 1) & 0xAAAAAAAA` (B) are then eight FP4 (E2M1) numbers in
//   {0, +1, -1} (sign in bit 3, exponent LSB in bit 1), which v_cvt_scalef32_pk_f16_fp4 expands
//   two at a time into fp16: 11 VALU operations per 16 trits.  The eight fp16 values of a field
//   are exactly one lane's share of the 32-deep K dimension of v_mfma_f32_16x16x32_f16.  Fields
//   0..3 (words 0,1) belong to scale group g0 and 4..7 (words 2,3) to g1, so four MFMAs
//   accumulate one (row, group) trit sum for 16 rows x 16 tokens.
//
// Why MFMA for a GEMV: "multiplication-free" (Sec. "Inference Efficiency") is a statement about
// the mathematics.  On CDNA4 a product by +-1/0 in the matrix pipe is exact and is the cheapest
// way to add: it leaves the vector ALU only the expansion of the 2-bit codes, which is what
// keeps the kernel under the HBM roof instead of the VALU roof.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include <algorithm>
#include <atomic>
#include <type_traits>
#include <vector>

#include "ptqtp.h"
#include "ptqtp_device.hpp"

namespace ptqtp_detail {
extern int g_chain_waves, g_chain_depth, g_chain_table;       // ptqtp_chain.hip
}

namespace {

struct BlobHeader {
    uint64_t magic;
    uint32_t layout;
    int32_t group;
    int64_t N, K, RT, KS;
};

struct Shape {
    int64_t N, K, RT, KS, NG;
};

inline bool make_shape(int64_t M, int64_t N, int64_t K, int32_t group, Shape *s, ptqtp_status *st) {
    if (group != 128) { *st = PTQTP_ERR_GROUP; return false; }
    if (M <= 0 || N <= 0 || K <= 0 || K % group != 0 || N > (1ll << 30) || K > (1ll << 30)) {
        *st = PTQTP_ERR_SHAPE; return false;
    }
    s->N = N; s->K = K; s->NG = K / group;
    s->RT = (N + kTileRows - 1) / kTileRows;
    s->KS = (K + kStepK - 1) / kStepK;
    // at most 2^27 records (a blob of 292 GB, more than the device holds): record counts and the
    // grids derived from them then fit 32 bits
    if (s->RT * s->KS > (1ll << 27)) { *st = PTQTP_ERR_SHAPE; return false; }
    *st = PTQTP_OK;
    return true;
}

constexpr int64_t kMaxGrid = 0x7fffffff;      // workgroups of one launch (x dimension)

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ------------------------------------------------------------------------------------------
// pack / unpack
// ------------------------------------------------------------------------------------------
__global__ void clear_status_kernel(int32_t *st) { *st = 0; }

// Header of a blob against the shape the caller is about to use it with: a bit per field that differs.
__global__ void check_blob_kernel(const uint8_t *__restrict__ blob, int64_t N, int64_t K, int64_t RT, int64_t KS,
                                  int32_t *__restrict__ dev_status)
{
    const BlobHeader h = *reinterpret_cast<const BlobHeader *>(blob);
    int32_t bad = 0;
    if (h.magic != kMagic) bad |= PTQTP_BLOB_BAD_MAGIC;
    if (h.layout != kLayoutId) bad |= PTQTP_BLOB_BAD_LAYOUT;
    if (h.group != 128) bad |= PTQTP_BLOB_BAD_GROUP;
    if (h.N != N || h.RT != RT) bad |= PTQTP_BLOB_BAD_N;
    if (h.K != K || h.KS != KS) bad |= PTQTP_BLOB_BAD_K;
    *dev_status = bad;
}

// Four trits held as int8 bytes of x -> their 2-bit codes at nibble j of a 16-bit result, the nonzero bit at nibble
// bit 1 - par and the sign at 3 - par (the layout of one parity of a plane word).  For a valid byte (0x00, 0x01, 0xff)
// bit 0 says nonzero and bit 7 says negative.  `bad` collects, as nonzero bits, every byte that is none of the three.
__device__ __forceinline__ uint32_t code4(uint32_t x, int par, uint32_t &bad) {
    const uint32_t nz = x & 0x01010101u, sg = (x >> 7) & 0x01010101u;
    const uint32_t neg = (sg << 8) - sg;                   // 0xff in the bytes whose sign bit is set
    bad |= x ^ (nz | neg);                                 // a valid byte is rebuilt exactly
    uint32_t c = (nz << (1 - par)) | (sg << (3 - par));    // bits at 8j + {1 - par, 3 - par}
    c = (c | (c >> 4)) & 0x00ff00ffu;                      // byte 1 -> nibble 1, byte 3 -> nibble 5
    return (c | (c >> 8)) & 0xffffu;                       // nibbles 4, 5 -> 2, 3
}

// Eight 2-bit codes of one parity of a plane word (half = 0: nibbles 0..3, 1: nibbles 4..7) -> four int8 trits
__device__ __forceinline__ uint32_t trits4(uint32_t w, int par, int half) {
    uint32_t t = (w >> (16 * half + 1 - par)) & 0x5555u;   // per nibble: nonzero at bit 0, sign at bit 2
    t = (t | (t << 8)) & 0x00ff00ffu;
    t = (t | (t << 4)) & 0x0f0f0f0fu;                      // one nibble per byte
    const uint32_t nz = t & 0x01010101u, sg = (t >> 2) & 0x01010101u;
    const uint32_t neg = (sg << 8) - sg, any = (nz << 8) - nz;   // 0xff where negative / where nonzero
    return (neg & any) | nz;                               // 0xff, 0x01 or 0x00 per byte
}

// One workgroup of 256 threads per kPackRecs consecutive records of a row tile (a row's bytes for them are
// contiguous: up to 512 bytes).  Their 16 rows x 256 columns of both planes (8 KB of int8 per record) come in through
// LDS with 16-byte loads, all of a thread's loads in flight at once; then every thread builds one 32-bit word per
// plane and record from two 8-byte LDS reads, and threads 0..63 store one scale per record.
// VEC: both planes are 16-byte aligned (K is a multiple of 128, so every row segment then is).
constexpr int kPackRecs = 2;      // measured: 1 and 2 alike, 4 slower (LDS per workgroup limits the workgroups per CU)

template <bool VEC>
__global__ void __launch_bounds__(256)
pack_kernel(const int8_t *__restrict__ T1, const int8_t *__restrict__ T2,
            const uint16_t *__restrict__ a1, const uint16_t *__restrict__ a2,
            uint8_t *__restrict__ blob, int64_t N, int64_t K, int64_t RT, int64_t KS, int64_t NG,
            int32_t *__restrict__ dev_status)
{
    // LDS holds the 8-byte trit groups in the order their readers come: slot par*256 + u is what thread u reads for
    // parity par (consecutive threads, consecutive slots: no bank conflicts on the read side)
    __shared__ uintx2 slots[kPackRecs][2][512];
    const int64_t per_rt = (KS + kPackRecs - 1) / kPackRecs;
    const int64_t rt = blockIdx.x / per_rt, ks0 = (blockIdx.x % per_rt) * kPackRecs;
    const int t = threadIdx.x;
    if (blockIdx.x == 0 && t == 0) {
        BlobHeader h;
        h.magic = kMagic; h.layout = kLayoutId; h.group = 128; h.N = N; h.K = K; h.RT = RT; h.KS = KS;
        *reinterpret_cast<BlobHeader *>(blob) = h;
    }
    if (blockIdx.x == 0 && t >= 12 && t < 64) reinterpret_cast<uint32_t *>(blob)[t] = 0;  // header tail (48..255)

    // thread -> row t/16, 16-byte segment t%16 of both planes of every record; rows past N and columns past K read as zero
    const int row = t >> 4, seg = t & 15;
    const int64_t n = rt * kTileRows + row;
    uintx4 v[kPackRecs][2];
    uint16_t scale[kPackRecs];
#pragma unroll
    for (int r = 0; r < kPackRecs; ++r) {
        const int64_t k = (ks0 + r) * kStepK + seg * 16;
#pragma unroll
        for (int plane = 0; plane < 2; ++plane) {
            v[r][plane] = uintx4{0u, 0u, 0u, 0u};
            if (n < N && k < K) {
                const int8_t *src = (plane ? T2 : T1) + n * K + k;
                if (VEC) v[r][plane] = load_stream<uintx4>(src);      // read once: keep it out of the caches' way
                else {
                    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int b = 0; b < 16; ++b) w[b >> 2] |= static_cast<uint32_t>(static_cast<uint8_t>(src[b])) << (8 * (b & 3));
                    v[r][plane] = uintx4{w[0], w[1], w[2], w[3]};
                }
            }
        }
        scale[r] = 0;
        if (t < 64) {                    // row nl = t/4, slot j = t%4: {a1[g0], a1[g1], a2[g0], a2[g1]}
            const int64_t ns = rt * kTileRows + (t >> 2), g = (ks0 + r) * 2 + (t & 1);
            if (ns < N && g < NG) scale[r] = ((t >> 1) & 1) ? a2[ns * NG + g] : a1[ns * NG + g];
        }
    }
    {
        // the 16 bytes are field f = seg/2 of quarter-lanes q0 and q0 + 1: word f/2, parity f%2 of lanes q*16 + row
        const int f = seg >> 1, q0 = (seg & 1) * 2;
        const int sa = (f & 1) * 256 + (q0 * 16 + row) * 4 + (f >> 1), sb = sa + 64;
#pragma unroll
        for (int r = 0; r < kPackRecs; ++r)
#pragma unroll
            for (int plane = 0; plane < 2; ++plane) {
                slots[r][plane][sa] = uintx2{v[r][plane].x, v[r][plane].y};
                slots[r][plane][sb] = uintx2{v[r][plane].z, v[r][plane].w};
            }
    }
    __syncthreads();
    uint32_t bad = 0;
#pragma unroll
    for (int r = 0; r < kPackRecs; ++r) {
        if (ks0 + r >= KS) break;                                          // uniform
        uint8_t *rec = blob + kHeaderBytes + (rt * KS + ks0 + r) * kRecordBytes;
#pragma unroll
        for (int plane = 0; plane < 2; ++plane) {
            uint32_t word = 0;
#pragma unroll
            for (int par = 0; par < 2; ++par) {
                const uintx2 b8 = slots[r][plane][par * 256 + t];
                uint32_t wrong = 0;
                const uint32_t lo = code4(b8.x, par, wrong), hi = code4(b8.y, par, wrong);
                // a byte outside {-1, 0, +1} is flagged and packed as 0: drop the codes of its nibble
                if (wrong) {
                    uint32_t keep = 0;
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if ((((j < 4 ? b8.x : b8.y) >> (8 * (j & 3))) + 1u & 0xffu) < 3u) keep |= 0xfu << (4 * j);
                    word |= (lo | (hi << 16)) & keep;
                    bad = 1;
                } else {
                    word |= lo | (hi << 16);
                }
            }
            reinterpret_cast<uint32_t *>(rec + plane * kPlaneBytes)[t] = word;
        }
        if (t < 64) reinterpret_cast<uint16_t *>(rec + 2 * kPlaneBytes)[t] = scale[r];
    }
    if (bad && dev_status) atomicOr(dev_status, 1);
}

// The mirror of pack_kernel: one workgroup of 256 threads per kPackRecs consecutive records of a row tile.  The
// plane words come in through LDS (thread t: word t of each plane of each record, all loads in flight at once);
// then thread t writes 16 consecutive columns of row t/16 per record and plane with one 16-byte store: those columns
// are field f = (t%16)/2, quarter-lanes q and q+1, all eight nibbles of word f/2 at parity f%2.
// VEC: the output planes are 16-byte aligned; otherwise bytes.
template <bool VEC>
__global__ void __launch_bounds__(256)
unpack_trits_kernel(const uint8_t *__restrict__ blob, int8_t *__restrict__ T1, int8_t *__restrict__ T2,
                    int64_t N, int64_t K, int64_t KS)
{
    __shared__ uint32_t words[kPackRecs][2][256];
    const int64_t per_rt = (KS + kPackRecs - 1) / kPackRecs;
    const int64_t rt = blockIdx.x / per_rt, ks0 = (blockIdx.x % per_rt) * kPackRecs;
    const int t = threadIdx.x;
    uint32_t w[kPackRecs][2];
#pragma unroll
    for (int r = 0; r < kPackRecs; ++r) {
        const int64_t ks = ks0 + r < KS ? ks0 + r : KS - 1;               // past the end: a duplicate, never stored
        const uint8_t *rec = blob + kHeaderBytes + (rt * KS + ks) * kRecordBytes;
#pragma unroll
        for (int plane = 0; plane < 2; ++plane) w[r][plane] = load_global<uint32_t>(rec + plane * kPlaneBytes + 4 * t);
    }
#pragma unroll
    for (int r = 0; r < kPackRecs; ++r) {
        words[r][0][t] = w[r][0];
        words[r][1][t] = w[r][1];
    }
    __syncthreads();
    const int row = t >> 4, seg = t & 15;
    const int f = seg >> 1, q0 = (seg & 1) * 2, i = f >> 1, par = f & 1;
    const int64_t n = rt * kTileRows + row;
    if (n >= N) return;
#pragma unroll
    for (int r = 0; r < kPackRecs; ++r) {
        const int64_t k = (ks0 + r) * kStepK + seg * 16;
        if (k >= K) break;
#pragma unroll
        for (int plane = 0; plane < 2; ++plane) {
            int8_t *T = plane ? T2 : T1;
            if (!T) continue;
            const uint32_t wa = words[r][plane][(q0 * 16 + row) * 4 + i], wb = words[r][plane][((q0 + 1) * 16 + row) * 4 + i];
            const uint32_t out[4] = {trits4(wa, par, 0), trits4(wa, par, 1), trits4(wb, par, 0), trits4(wb, par, 1)};
            int8_t *dst = T + n * K + k;
            if (VEC) *reinterpret_cast<uintx4 *>(dst) = uintx4{out[0], out[1], out[2], out[3]};
            else {
#pragma unroll
                for (int b = 0; b < 16; ++b) dst[b] = static_cast<int8_t>((out[b >> 2] >> (8 * (b & 3))) & 0xffu);
            }
        }
    }
}

__global__ void __launch_bounds__(256)
unpack_scales_kernel(const uint8_t *__restrict__ blob, uint16_t *__restrict__ a1, uint16_t *__restrict__ a2,
                     int64_t N, int64_t NG, int64_t KS)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= N * NG) return;
    const int64_t n = idx / NG, g = idx % NG;
    const int64_t rt = n / kTileRows, ks = g / 2;
    const int nl = static_cast<int>(n % kTileRows), j = static_cast<int>(g & 1);
    const uint16_t *sc = reinterpret_cast<const uint16_t *>(
        blob + kHeaderBytes + (rt * KS + ks) * kRecordBytes + 2 * kPlaneBytes);
    if (a1) a1[idx] = sc[nl * 4 + j];
    if (a2) a2[idx] = sc[nl * 4 + 2 + j];
}

// ------------------------------------------------------------------------------------------
// streamed GEMV / small-batch GEMM on the matrix pipe
// ------------------------------------------------------------------------------------------
// ------------------------------------------------------------------------------------------
// One workgroup = one item = one 16-row tile of one linear over its whole K.  Its W waves split
// the item's 256-column steps (wave w: ks = w, w+W, ...).  A wave issues the loads of up to S
// steps at once (straight-line code, so every wait is an exact vmcnt), consumes them, and
// repeats; latency is hidden by the other workgroups resident on the CU.  Partial sums meet in
// LDS in fixed order.  A plan (table of linears + item -> linear map) lets one launch cover many
// linears, so the HBM stream does not drain between the layers of a stack.
struct LinearDesc {
    const uint8_t *records;   // blob + header
    const uint16_t *x;        // fp16 [K]
    void *y;                  // [N] f32 or f16
    int32_t N, K, RT, KS;
    int32_t first_item;       // index of this linear's row tile 0 in the item list
    int32_t pad;
};

struct PlanHeader {           // 64 bytes, followed by LinearDesc[count], then int32 item_lin[total_items]
    uint64_t magic;
    int32_t count, total_items, y_f16, group;
    int32_t reserved[10];
};
constexpr uint64_t kPlanMagic = 0x314e4c5050545150ull;  // "PQTPPLN1"
constexpr int kPlanChunk = 32;
constexpr int kPlanPad = 16;     // items per linear are rounded up to this: a workgroup of up to 16 row tiles never straddles two linears

struct DescChunk { LinearDesc d[kPlanChunk]; };

__global__ void plan_write_kernel(PlanHeader *plan, DescChunk chunk, int base, int n, int count, int total_items,
                                  int y_f16)
{
    const int t = threadIdx.x;
    if (base == 0 && t == 0) {
        PlanHeader h = {};
        h.magic = kPlanMagic; h.count = count; h.total_items = total_items; h.y_f16 = y_f16; h.group = 128;
        *plan = h;
    }
    if (t < n) reinterpret_cast<LinearDesc *>(plan + 1)[base + t] = chunk.d[t];
}

// item -> linear index, by bisection over first_item (one-time, after plan_write_kernel)
__global__ void __launch_bounds__(256) plan_map_kernel(PlanHeader *plan)
{
    const int count = plan->count, total = plan->total_items;
    LinearDesc *table = reinterpret_cast<LinearDesc *>(plan + 1);
    int32_t *map = reinterpret_cast<int32_t *>(table + count);
    for (int item = blockIdx.x * 256 + threadIdx.x; item < total; item += gridDim.x * 256) {
        int lo = 0, hi = count - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (table[mid].first_item <= item) lo = mid; else hi = mid - 1;
        }
        map[item] = lo;
    }
}

template <bool PLAN, int S>
__global__ void __launch_bounds__(1024)
gemv_items_kernel(const PlanHeader *__restrict__ plan, LinearDesc single, int single_f16)
{
    __shared__ float red[16][16];
    __shared__ uintx2 xs[16][64];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int W = blockDim.x >> 6;
    const int nl = lane & 15, q = lane >> 4;
    const uint32_t lane16 = lane * 16u, nl8 = nl * 8u;
    const int item = blockIdx.x;

    const LinearDesc *dp = &single;
    int y_f16 = single_f16;
    if (PLAN) {
        const LinearDesc *table = reinterpret_cast<const LinearDesc *>(plan + 1);
        const int32_t *map = reinterpret_cast<const int32_t *>(table + plan->count);
        if (item >= plan->total_items) return;      // whole workgroup leaves: no barrier is skipped
        dp = table + map[item];
        y_f16 = plan->y_f16;
    }
    const int K = dp->K, KS = dp->KS, N = dp->N;
    const int rt = item - dp->first_item;
    if (rt >= dp->RT) return;                       // padding item of a plan (whole workgroup leaves)
    const uint8_t *rec0 = dp->records + static_cast<size_t>(rt) * KS * kRecordBytes;
    const int rot = (rt * 5) % KS;
    const uint16_t *x = dp->x;

    uintx4 xa[1][8];
#pragma unroll
    for (int f = 0; f < 8; ++f) xa[0][f] = uintx4{0, 0, 0, 0};   // lanes of tokens 1..15 stay zero
    const char *xs_rd = reinterpret_cast<const char *>(&xs[w][0]) + q * 16;
    float yacc = 0.f;

    // tail: K is an odd number of 128-column groups, so the last record is half padding and the lanes of its second
    // half must not read x past its end.  The choice is made once per item, outside the loop (every LLaMA shape
    // takes the branch without the checks), so that each loop stays straight-line code.
    auto run = [&](auto tail_tag) {
        constexpr bool tail = decltype(tail_tag)::value;
        for (int ks0 = w; ks0 < KS; ks0 += S * W) {
            StepRegs r[S];
            // issue: S steps in flight.  Steps past the end re-read the wave's first step (address
            // stays valid, result unused) so that the number of outstanding loads is static.
    #pragma unroll
            for (int i = 0; i < S; ++i) {
                const int ks = ks0 + i * W;
                int kse = (ks < KS ? ks : ks0) + rot;       // rotated start: neighbours hit different x lines
                kse = kse >= KS ? kse - KS : kse;
                const uint8_t *rec = rec0 + static_cast<size_t>(kse) * kRecordBytes;
                // uniform base + 32-bit lane offset: the loads take the record address from scalar registers
                r[i].p1 = load_stream<uintx4>(rec + lane16);
                r[i].p2 = load_stream<uintx4>(rec + (kPlaneBytes + lane16));
                r[i].sc = load_stream<uintx2>(rec + (2 * kPlaneBytes + nl8));
                int k = kse * kStepK + lane * 4;
                if (tail) k = k < K ? k : 0;                         // odd number of groups: tail lanes
                r[i].xr = load_global<uintx2>(x + static_cast<uint32_t>(k));
            }
    #pragma unroll
            for (int i = 0; i < S; ++i) {
                const int ks = ks0 + i * W;
                if (ks < KS) {
                    uintx2 xr = r[i].xr;
                    int kr = ks + rot;
                    kr = kr >= KS ? kr - KS : kr;
                    if (tail && kr * kStepK + lane * 4 >= K) xr = uintx2{0, 0};
                    xs[w][lane] = xr;                                // wave-private bounce: no barrier
                    if (nl == 0) {
    #pragma unroll
                        for (int f = 0; f < 8; ++f)
                            xa[0][f] = *reinterpret_cast<const uintx4 *>(xs_rd + (f >> 2) * 256 + (f & 3) * 64);
                    }
                    const float a1g0 = half_bits_to_float(r[i].sc.x & 0xffffu), a1g1 = half_bits_to_float(r[i].sc.x >> 16);
                    const float a2g0 = half_bits_to_float(r[i].sc.y & 0xffffu), a2g1 = half_bits_to_float(r[i].sc.y >> 16);
                    floatx4 acc[1];
                    group_sum<1, 0>(xa, r[i].p1, acc); yacc = fmaf(a1g0, acc[0][0], yacc);
                    group_sum<1, 1>(xa, r[i].p1, acc); yacc = fmaf(a1g1, acc[0][0], yacc);
                    group_sum<1, 0>(xa, r[i].p2, acc); yacc = fmaf(a2g0, acc[0][0], yacc);
                    group_sum<1, 1>(xa, r[i].p2, acc); yacc = fmaf(a2g1, acc[0][0], yacc);
                }
            }
        }
    };
    if (K & (kStepK - 1)) run(std::true_type{}); else run(std::false_type{});

    if (q == 0) red[w][nl] = yacc;
    __syncthreads();
    if (threadIdx.x < 16) {
        float s = 0.f;
        for (int ww = 0; ww < W; ++ww) s += red[ww][threadIdx.x];
        const int n = rt * kTileRows + threadIdx.x;
        if (n < N) {
            if (y_f16) reinterpret_cast<_Float16 *>(dp->y)[n] = static_cast<_Float16>(s);
            else reinterpret_cast<float *>(dp->y)[n] = s;
        }
    }
}

int g_tune_stream_waves = 0, g_tune_stream_depth = 0;

template <bool PLAN>
hipError_t launch_items(const PlanHeader *plan, const LinearDesc &single, int y_f16, int64_t total_items,
                        int64_t min_ks, hipStream_t stream)
{
    // A batched launch has thousands of items in flight: 4 waves x 2 records each is enough.  A single
    // linear has few items, so more waves per item put the whole matrix in flight at once.
    int W = 4, S = 2;
    if (!PLAN || total_items < 2048) {
        S = 1;
        while (W < 16 && total_items * W * 2 <= 4096) W *= 2;
        while (W > 1 && W > min_ks) W /= 2;
        // one very tall layer (70B gate / up: 1792 row tiles over 32 steps): eight waves with two records each in
        // flight measured 22.3 us against 25.0 us for four waves with one (and 23.7-24.1 us for the shapes between)
        if (!PLAN && total_items >= 1536 && min_ks >= 16) { W = 8; S = 2; }
    }
    if (g_tune_stream_waves > 0) W = g_tune_stream_waves;
    if (g_tune_stream_depth > 0) S = g_tune_stream_depth;
    const dim3 grid(static_cast<unsigned>(total_items)), block(W * 64);
    if (S >= 4) hipLaunchKernelGGL((gemv_items_kernel<PLAN, 4>), grid, block, 0, stream, plan, single, y_f16);
    else if (S >= 2) hipLaunchKernelGGL((gemv_items_kernel<PLAN, 2>), grid, block, 0, stream, plan, single, y_f16);
    else hipLaunchKernelGGL((gemv_items_kernel<PLAN, 1>), grid, block, 0, stream, plan, single, y_f16);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// small-batch kernel (2 <= M <= 64): item = R consecutive 16-row tiles of one linear
// ------------------------------------------------------------------------------------------
// Same record stream as the batch-1 kernel; each decoded field feeds MT = ceil(M/16) MFMAs.
// Activations: a wave fetches the tokens' 256-column slices of its step with fully coalesced loads
// (32 lanes = the 512 contiguous bytes of one token, two tokens per load instruction, ML
// instructions for up to 2*ML tokens), parks them in a wave-private LDS slot with padded rows, and
// reads them back in the MFMA A-operand layout (lane = token + 16*quarter, 8 columns per field).
// LDS operations of a wave execute in order, so the slot needs no barrier and is reused every step.
// Token rows >= M re-load the last real token: their rows of D are garbage that is never stored
// (rows of A only influence the same rows of D).
// slot layout, token-major: row r at r*528, chunk c at c*16
constexpr int kSlotRowBytes = 528;                   // 512 B of one token + 16 B pad: conflict-free operand reads
constexpr int kSlotBytes = 16 * kSlotRowBytes;       // per wave
__device__ __forceinline__ int slot_wr_off(int row, int chunk) { return row * kSlotRowBytes + chunk * 16; }
__device__ __forceinline__ int slot_rd_off(int nl, int q, int f) { return nl * kSlotRowBytes + (f >> 2) * 256 + (f & 3) * 64 + q * 16; }

// PLAN: the item list of a batch plan (R must be 1): one launch over many linears, all with M tokens.
// ML = load instructions per 16-token tile (1, 2, 4 or 8): covers M <= 2*ML when MT == 1.
// (MT, R) whose registers fit two waves per SIMD (256 per lane): those run with up to eight waves per item
constexpr bool items_eight_waves(int MT, int R) { return MT * R < 6 || (MT == 2 && R == 4); }

template <int MT, int R, int S, bool PLAN, int ML>
__global__ void __launch_bounds__(items_eight_waves(MT, R) ? 512 : 256)
gemm_items_kernel(const PlanHeader *__restrict__ plan, const uint8_t *__restrict__ records_,
                  const uint16_t *__restrict__ x_, void *__restrict__ y_, int M, int N_, int K_, int RT_, int KS_,
                  int y_f16_, const uint16_t *__restrict__ residual, int gated)
{
    extern __shared__ float red[];                     // [W][R][MT][16 tokens][16 rows]; first used as bounce slots
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int W = blockDim.x >> 6;
    const int nl = lane & 15, q = lane >> 4;
    const uint8_t *records = records_;
    const uint16_t *x = x_;
    void *y = y_;
    // gated (decode chain, R == 2): the item's two row tiles are gate tile i and up tile i of a stacked
    // [gate; up] linear, RT/2 tiles apart; otherwise R consecutive tiles
    const int rstride = gated ? RT_ / 2 : 1;
    int N = N_, K = K_, RT = RT_, KS = KS_, y_f16 = y_f16_, rt0 = gated ? blockIdx.x : blockIdx.x * R;
    if (PLAN) {
        if (static_cast<int>(blockIdx.x) >= plan->total_items) return;   // whole workgroup, before any barrier
        const LinearDesc *table = reinterpret_cast<const LinearDesc *>(plan + 1);
        const int32_t *map = reinterpret_cast<const int32_t *>(table + plan->count);
        const LinearDesc *dp = table + map[blockIdx.x];
        records = dp->records; x = dp->x; y = dp->y;
        N = dp->N; K = dp->K; RT = dp->RT; KS = dp->KS; y_f16 = plan->y_f16;
        rt0 = blockIdx.x - dp->first_item;
        if (rt0 >= RT) return;                       // padding item
    }
    const int rot = (rt0 * 5) % KS;

    float yacc[R][MT][4];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j) yacc[r][mt][j] = 0.f;

    // loader role of this lane: 16-byte chunk lc (0..31) of token row 2*i + lh of load instruction i
    const int lh = lane >> 5, lc = lane & 31;
    char *slot = reinterpret_cast<char *>(red) + w * kSlotBytes;

    for (int ks0 = w; ks0 < KS; ks0 += S * W) {
        uintx4 p1[S][R], p2[S][R];
        uintx2 sc[S][R];
        uintx4 xa[S][MT][8];                          // first ML entries: raw loads; after the bounce: operands
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const int ks = ks0 + i * W;
            int kse = (ks < KS ? ks : ks0) + rot;        // past the end: re-read, result unused
            kse = kse >= KS ? kse - KS : kse;              // rotated start: neighbours hit different x lines
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int rt = rt0 + r * rstride < RT ? rt0 + r * rstride : rt0;
                const uint8_t *rec = records + (static_cast<size_t>(rt) * KS + kse) * kRecordBytes;
                p1[i][r] = load_stream<uintx4>(rec + lane * 16);
                p2[i][r] = load_stream<uintx4>(rec + kPlaneBytes + lane * 16);
                sc[i][r] = load_stream<uintx2>(rec + 2 * kPlaneBytes + nl * 8);
            }
            int kc = kse * kStepK + lc * 8;
            kc = kc < K ? kc : kc - 128;                 // padded half record: its trits are zero
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int l = 0; l < ML; ++l) {
                    int m = mt * 16 + 2 * l + lh;
                    m = m < M ? m : M - 1;
                    xa[i][mt][l] = load_global<uintx4>(x + static_cast<size_t>(m) * K + kc);
                }
        }
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const int ks = ks0 + i * W;
            if (ks < KS) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                    for (int l = 0; l < ML; ++l)
                        *reinterpret_cast<uintx4 *>(slot + slot_wr_off(2 * l + lh, lc)) = xa[i][mt][l];
#pragma unroll
                    for (int f = 0; f < 8; ++f)
                        xa[i][mt][f] = *reinterpret_cast<const uintx4 *>(slot + slot_rd_off(nl, q, f));
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const float a1g0 = half_bits_to_float(sc[i][r].x & 0xffffu), a1g1 = half_bits_to_float(sc[i][r].x >> 16);
                    const float a2g0 = half_bits_to_float(sc[i][r].y & 0xffffu), a2g1 = half_bits_to_float(sc[i][r].y >> 16);
                    floatx4 acc[MT];
                    group_sum<MT, 0>(xa[i], p1[i][r], acc);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a1g0, acc[mt][j], yacc[r][mt][j]);
                    group_sum<MT, 1>(xa[i], p1[i][r], acc);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a1g1, acc[mt][j], yacc[r][mt][j]);
                    group_sum<MT, 0>(xa[i], p2[i][r], acc);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a2g0, acc[mt][j], yacc[r][mt][j]);
                    group_sum<MT, 1>(xa[i], p2[i][r], acc);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a2g1, acc[mt][j], yacc[r][mt][j]);
                }
            }
        }
    }

    constexpr int OUT = R * MT * 256;
    __syncthreads();                                   // bounce slots are dead: the space becomes `red`
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                red[w * OUT + ((r * MT + mt) * 16 + 4 * q + j) * 16 + nl] = yacc[r][mt][j];
    __syncthreads();
    const int n_out = gated ? N / 2 : N;              // gated: silu(gate) * up, one output per (gate, up) row pair
    for (int o = threadIdx.x; o < (gated ? OUT / R : OUT); o += blockDim.x) {
        float s = 0.f;
        for (int ww = 0; ww < W; ++ww) s += red[ww * OUT + o];
        const int on = o & 15, t = o >> 4;
        const int m = (t / 16 % MT) * 16 + (t & 15), r = t / (16 * MT);
        const int n = (rt0 + r) * kTileRows + on;
        if (m < M && rt0 + r * rstride < RT && n < n_out) {
            if (gated) {
                float u = 0.f;
                for (int ww = 0; ww < W; ++ww) u += red[ww * OUT + o + MT * 256];
                s = (s / (1.0f + __expf(-s))) * u;
            }
            const size_t off = static_cast<size_t>(m) * n_out + n;
            if (residual != nullptr) s += half_bits_to_float(load_global<uint16_t>(residual + off));
            if (y_f16) reinterpret_cast<_Float16 *>(y)[off] = static_cast<_Float16>(s);
            else reinterpret_cast<float *>(y)[off] = s;
        }
    }
}

// ------------------------------------------------------------------------------------------
// MFMA tile for large batches / prefill: here the path is a dense contraction
// ------------------------------------------------------------------------------------------
// Workgroup = 4 waves along the rows, each owning 4 row tiles x MTW token tiles (64 rows x 64 or
// 128 tokens, 16 or 32 MFMA accumulators).  Per scale
// group (128 columns) the workgroup stages its tokens' activations in LDS (coalesced loads,
// padded rows, double-buffered, one barrier per group); every wave expands the trits of its own
// four row tiles in registers and multiplies them by the group scale -- alpha * {0,+-1} is exact
// in fp16, so alpha1*T1 and alpha2*T2 enter the matrix pipe directly and both planes share one
// fp32 accumulator -- then issues 8*MTW MFMAs per 32-column field against MTW LDS operand reads.
// Workgroups are numbered so that all token blocks of a row block run on the same XCD and
// share its L2 copy of the packed rows.
constexpr int kTileChunk = 1040;                    // 1 KiB chunk of four tokens + 16-byte skew (tiles with direct-to-LDS loads)

// One direct global -> LDS load of 16 bytes per lane (lane l lands at lds_base + 16*l), written as inline assembly.
// Through the compiler's builtin the same instruction makes the wait-count pass treat every later LDS wait of the wave
// as "counters may retire out of order" until both counters have been drained: each s_waitcnt for an operand read
// becomes lgkmcnt(0) and operand reads issued ahead of their use buy nothing.  Hidden from that pass, the loads are
// waited for by hand (s_waitcnt vmcnt(0) before the barrier that publishes the buffer); loads the pass does not know
// of can only make its own vmcnt waits stricter, never weaker, because the counter retires in issue order.
// M0 (the LDS base of the load) is a register the compiler reserves for the instructions that read it implicitly; the
// statement saves it in a scalar temporary and puts it back after the load has been issued, so nothing is assumed
// about what else the compiler keeps there.  One wait state separates the scalar write of M0 from the load that
// reads it.
__device__ __forceinline__ void lds_direct_load16(const void *gptr, const char *lds_base)
{
    const uint32_t lds_off = static_cast<uint32_t>(reinterpret_cast<size_t>(
        (const __attribute__((address_space(3))) char *)lds_base));
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "v"(gptr), "s"(lds_off) : "memory");
}
#pragma clang diagnostic pop

// Epilogues of the MFMA tiles (the decode chain at many tokens): `gated` = the layer stacks N/2 gate rows over N/2
// up rows and a wave's row tiles alternate gate, up of the same 16 outputs: out = silu(gate) * up; then, if
// residual != null, out += residual[m][n] (fp16, same shape as the output).
struct TileEpilogue {
    const uint16_t *residual;
    int gated;
};

// The r-th row tile of a wave whose first tile (or gate/up pair) index is `first`, out of RT row tiles
__device__ __forceinline__ int tile_row(int first, int r, int RT, int gated) {
    if (!gated) return first + r;
    const int P = RT >> 1;
    const int p = first + (r >> 1);
    return (p < P ? p : P - 1) + (r & 1) * P;
}

// Store one wave's accumulators: acc[r][mt] = rows of row tile r (lane nl) x tokens m_of(mt, j)
template <int RTW, int MTW, typename TokenOf>
__device__ __forceinline__ void tile_store(const floatx4 (&acc)[RTW][MTW], void *y, int y_f16, int first, int nl, int M, int N,
                                           const TileEpilogue &ep, TokenOf m_of)
{
    const int n_out = ep.gated ? N >> 1 : N;
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        if (ep.gated && (r & 1)) continue;
        const int t = ep.gated ? first + (r >> 1) : first + r;       // output tile
        const int n = t * kTileRows + nl;
        if (n < n_out) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int m = m_of(mt, j);
                    if (m < M) {
                        float out = acc[r][mt][j];
                        if (ep.gated) {
                            const float up = acc[r + 1 < RTW ? r + 1 : r][mt][j];
                            out = (out / (1.0f + __expf(-out))) * up;             // silu(gate) * up
                        }
                        const size_t off = static_cast<size_t>(m) * n_out + n;
                        if (ep.residual != nullptr) out += half_bits_to_float(load_global<uint16_t>(ep.residual + off));
                        if (y_f16) reinterpret_cast<_Float16 *>(y)[off] = static_cast<_Float16>(out);
                        else reinterpret_cast<float *>(y)[off] = out;
                    }
                }
        }
    }
}

__device__ __forceinline__ half8 decode8(uint32_t word, int parity) {
    const uint32_t fp4 = (parity ? (word << 1) : word) & 0xAAAAAAAAu;
    const half2v h0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 0);
    const half2v h1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 1);
    const half2v h2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 2);
    const half2v h3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(fp4, 1.0f, 3);
    return half8{h0.x, h0.y, h1.x, h1.y, h2.x, h2.y, h3.x, h3.y};
}

template <int RTW>
struct TileRecs {               // the records of a wave's RTW row tiles for one 256-column step
    uintx4 p1[RTW], p2[RTW];
    uintx2 sc[RTW];
};

// MTW = token tiles per wave (4 or 8), RTW = row tiles per wave (4, 2 or 1).  The four waves of a workgroup sit
// along the rows: workgroup tile = 64*RTW rows x 16*MTW tokens.  The smaller tiles are for problems that would
// otherwise leave most CUs without a workgroup (short prompts on 8B-sized layers).
// FUSE: the two planes are summed before the matrix pipe, w16 = fp16(alpha1*t1 + alpha2*t2): both
// products are exact in fp16, so this is ONE rounding per weight (the "dequantization" forward of
// Sec. "Inference Efficiency": the weight is rebuilt, here per 32-column field in registers) and
// half the MFMAs.
template <int MTW, bool FUSE, int RTW>
__global__ void __launch_bounds__(256)
gemm_tile_kernel(const uint8_t *__restrict__ records, const uint16_t *__restrict__ x, void *__restrict__ y,
                 int M, int N, int K, int RT, int KS, int y_f16, int MB, int NB, int nb0, TileEpilogue ep)
{
    extern __shared__ char xt[];                     // [2][TM/4 chunks][kTileChunk]
    constexpr int TM = 16 * MTW, NRT = 4 * RTW;      // tokens, row tiles per workgroup
    constexpr int kBuf = (TM / 4) * kTileChunk;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nl = lane & 15, q = lane >> 4;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int nb = nb0 + (slot / MB) * 8 + xcd, mb = slot % MB;   // this launch covers row blocks nb0 .. NB-1
    if (nb >= NB) return;                            // whole workgroup, before any barrier
    const int m0 = mb * TM;
    const int rt_base = ep.gated ? nb * (NRT / 2) + w * (RTW / 2) : nb * NRT + w * RTW;   // first tile, or first pair
    const int NG = K / 128;

    // staging (global -> LDS directly): wave w brings in chunks w, w+4, ... of the group; a chunk is the 256-byte group
    // slice of four tokens, lane t*16+p bringing 16-byte piece p of token c%16 + 16*t of 64-token block c/16
    const uint16_t *xcol = x + (lane & 15) * 8;
    auto stage = [&](int g, int buf) {
#pragma unroll
        for (int j = 0; j < TM / 16; ++j) {
            const int c = w + 4 * j;
            int m = m0 + (c >> 4) * 64 + (c & 15) + (lane >> 4) * 16;
            m = m < M ? m : M - 1;                   // rows past M: duplicates, never stored
            asm volatile("" : "+v"(m));              // recompute the row address here instead of keeping TM/16 of them
            lds_direct_load16(xcol + static_cast<size_t>(m) * K + g * 128, xt + buf * kBuf + c * kTileChunk);
        }
    };
    // operand of token tile mt: tokens (mt%4)*16 + nl of block mt/4 -> chunk nl, run mt%4
    const char *xop = xt + nl * kTileChunk + q * 16;

    const uint8_t *rec[RTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        int rt = tile_row(rt_base, r, RT, ep.gated);
        rt = rt < RT ? rt : RT - 1;
        rec[r] = records + static_cast<size_t>(rt) * KS * kRecordBytes;
    }

    floatx4 acc[RTW][MTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) acc[r][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto load_recs = [&](TileRecs<RTW> &t, int ks) {
#pragma unroll
        for (int r = 0; r < RTW; ++r) {
            const uint8_t *p = rec[r] + static_cast<size_t>(ks) * kRecordBytes;
            t.p1[r] = load_global<uintx4>(p + lane * 16);
            t.p2[r] = load_global<uintx4>(p + kPlaneBytes + lane * 16);
            t.sc[r] = load_global<uintx2>(p + 2 * kPlaneBytes + nl * 8);
        }
    };

    TileRecs<RTW> ra, rb;
    stage(0, 0);
    load_recs(ra, 0);
    rb = ra;
    __builtin_amdgcn_s_waitcnt(0);                   // this wave's chunks have landed in LDS
    __syncthreads();

    // one 256-column step: two scale groups from `cur`, while `nxt` is filled for step ks+1
    auto step = [&](const TileRecs<RTW> &cur, TileRecs<RTW> &nxt, int ks) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int g = ks * 2 + h;
            if (g < NG) {
                const bool more = g + 1 < NG;
                if (more) stage(g + 1, (g + 1) & 1);
                if (h == 0 && ks + 1 < KS) load_recs(nxt, ks + 1);
                const char *xb = xop + (g & 1) * kBuf;
                half8 al1[RTW], al2[RTW];
#pragma unroll
                for (int r = 0; r < RTW; ++r) {
                    const _Float16 a1 = __builtin_bit_cast(_Float16, static_cast<uint16_t>(h ? (cur.sc[r].x >> 16) : (cur.sc[r].x & 0xffffu)));
                    const _Float16 a2 = __builtin_bit_cast(_Float16, static_cast<uint16_t>(h ? (cur.sc[r].y >> 16) : (cur.sc[r].y & 0xffffu)));
                    al1[r] = half8{a1, a1, a1, a1, a1, a1, a1, a1};
                    al2[r] = half8{a2, a2, a2, a2, a2, a2, a2, a2};
                }
                // software pipeline over the four 32-column fields of the group: while the MFMAs of
                // field fm run, the operands of field fm+1 are read from LDS and its trits expanded
                constexpr int NPL = FUSE ? 1 : 2;
                half8 bq[2][NPL][RTW], aq[2][MTW];
                auto expand = [&](half8 (&b)[NPL][RTW], int fm) {
                    const int wi = 2 * h + (fm >> 1), par = fm & 1;
#pragma unroll
                    for (int r = 0; r < RTW; ++r) {
                        if constexpr (FUSE) {
                            b[0][r] = decode8(cur.p1[r][wi], par) * al1[r] + decode8(cur.p2[r][wi], par) * al2[r];
                        } else {
                            b[0][r] = decode8(cur.p1[r][wi], par) * al1[r];
                            b[NPL - 1][r] = decode8(cur.p2[r][wi], par) * al2[r];
                        }
                    }
                };
                auto operands = [&](half8 (&a)[MTW], int fm) {
#pragma unroll
                    for (int mt = 0; mt < MTW; ++mt)
                        a[mt] = __builtin_bit_cast(
                            half8, *reinterpret_cast<const uintx4 *>(xb + (mt >> 2) * (16 * kTileChunk) + (mt & 3) * 256 + fm * 64));
                };
                // (measured: pays with one MFMA set per field; with two the plain order is as fast)
                constexpr bool AHEAD = FUSE;
                if (AHEAD) { operands(aq[0], 0); expand(bq[0], 0); }
#pragma unroll
                for (int fm = 0; fm < 4; ++fm) {
                    if (!AHEAD) { operands(aq[fm & 1], fm); expand(bq[fm & 1], fm); }
                    else if (fm + 1 < 4) {
                        operands(aq[(fm + 1) & 1], fm + 1);
                        expand(bq[(fm + 1) & 1], fm + 1);
                    }
                    // consecutive MFMAs write different accumulators
#pragma unroll
                    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
                        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                            for (int r = 0; r < RTW; ++r)
                                acc[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aq[fm & 1][mt], bq[fm & 1][pl][r], acc[r][mt], 0, 0, 0);
                }
                __builtin_amdgcn_s_waitcnt(0);       // the next group's chunks (and records) have landed
                __syncthreads();
            }
        }
    };

    for (int ks = 0; ks < KS; ks += 2) {
        step(ra, rb, ks);
        if (ks + 1 < KS) step(rb, ra, ks + 1);
    }

    tile_store<RTW, MTW>(acc, y, y_f16, rt_base, nl, M, N, ep, [&](int mt, int j) { return m0 + mt * 16 + 4 * q + j; });
}

// Large prefill tile: 256 rows x 256 tokens, eight waves along the rows (two per SIMD), each 2 row tiles x all 16
// token tiles: every trit of the workgroup is expanded exactly once and used for 16 MFMAs (a 4 x 2 arrangement of
// waves with 4 row tiles x 8 token tiles each expands every trit twice and measured 3-9 % slower, although it reads
// half as many operands from LDS), and a second wave on every SIMD fills the issue slots the first one leaves.
// What makes it fit in 256 registers per lane:
//  - activations go from global memory straight into LDS (global_load_lds_dwordx4, no staging
//    registers).  One instruction moves a 1-KiB chunk = the 256 bytes (one 128-column group) of
//    four tokens, lane t*16+p bringing 16-byte piece p of token t -- four full 256-byte runs, the
//    pattern the L1 serves at full rate (16 tokens x 64 bytes per instruction runs 4x slower).
//    Chunk c of a 64-token block holds tokens c, c+16, c+32, c+48 and starts at c*1040 bytes, so
//    the 16 tokens of an MFMA token tile sit in 16 different chunks, each skewed by 16 bytes:
//    the A-operand read (token nl, pieces 4*field+q) is one conflict-free ds_read_b128;
//  - record words are fetched per scale group, 8 bytes per lane, plane and row tile.
// FUSE as in gemm_tile_kernel.
constexpr int kTile3Tokens = 256;
constexpr int kTile3BufBytes = 64 * kTileChunk;              // one 128-column group of 256 tokens

template <bool FUSE>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
gemm_tile3_kernel(const uint8_t *__restrict__ records, const uint16_t *__restrict__ x, void *__restrict__ y,
                  int M, int N, int K, int RT, int KS, int y_f16, int MB, int NB, int nb0, TileEpilogue ep)
{
    extern __shared__ char xt[];                     // [2][64 chunks][1040]
    constexpr int TM = kTile3Tokens, NRT = 16, RTW = 2, MTW = 16;   // row tiles, token tiles per wave
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nl = lane & 15, q = lane >> 4;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int nb = nb0 + (slot / MB) * 8 + xcd, mb = slot % MB;   // this launch covers row blocks nb0 .. NB-1
    if (nb >= NB) return;                            // whole workgroup, before any barrier
    const int m0 = mb * TM;
    const int rt_base = ep.gated ? nb * (NRT / 2) + w * (RTW / 2) : nb * NRT + w * RTW;   // first tile, or first pair
    const int NG = K / 128;

    // staging role: wave w brings in chunks 8*(w%2) .. +7 of 64-token block w/2; lane t*16+p: piece p of token c + 16*t
    const int tok0 = m0 + (w >> 1) * 64 + (w & 1) * 8 + (lane >> 4) * 16;
    const uint16_t *xcol = x + (lane & 15) * 8;
    auto stage = [&](int g, int buf) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            int m = tok0 + j;
            m = m < M ? m : M - 1;                   // rows past M: duplicates, never stored
            asm volatile("" : "+v"(m));              // recompute the row address here: eight hoisted 64-bit addresses would not fit
            lds_direct_load16(xcol + static_cast<size_t>(m) * K + g * 128,
                              xt + buf * kTile3BufBytes + ((w >> 1) * 16 + (w & 1) * 8 + j) * kTileChunk);
        }
    };

    const uint8_t *rec[RTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        int rt = tile_row(rt_base, r, RT, ep.gated);
        rt = rt < RT ? rt : RT - 1;
        rec[r] = records + static_cast<size_t>(rt) * KS * kRecordBytes + lane * 16;
    }

    floatx4 acc[RTW][MTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) acc[r][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    // words of group g: record g/2, half g%2 -> 8 bytes per lane, plane and row tile; scales: 4 fp16 per row
    auto load_group = [&](uintx2 (&pw)[RTW][2], uintx2 (&sc)[RTW], int g) {
        const size_t off = static_cast<size_t>(g >> 1) * kRecordBytes + (g & 1) * 8;
#pragma unroll
        for (int r = 0; r < RTW; ++r) {
            pw[r][0] = load_global<uintx2>(rec[r] + off);
            pw[r][1] = load_global<uintx2>(rec[r] + off + kPlaneBytes);
            sc[r] = load_global<uintx2>(rec[r] - lane * 16 + static_cast<size_t>(g >> 1) * kRecordBytes + 2 * kPlaneBytes + nl * 8);
        }
    };
    auto compute = [&](const uintx2 (&pw)[RTW][2], const uintx2 (&sc)[RTW], int g) {
        // token tile mt: 64-token block mt/4, tokens (mt%4)*16 + nl -> chunk nl, run mt%4
        const char *xb = xt + (g & 1) * kTile3BufBytes + nl * kTileChunk + q * 16;
        const int h = g & 1;
        constexpr int NPL = FUSE ? 1 : 2;
        half8 al[RTW][2];
#pragma unroll
        for (int r = 0; r < RTW; ++r) {
            const _Float16 a1 = __builtin_bit_cast(_Float16, static_cast<uint16_t>(h ? (sc[r].x >> 16) : (sc[r].x & 0xffffu)));
            const _Float16 a2 = __builtin_bit_cast(_Float16, static_cast<uint16_t>(h ? (sc[r].y >> 16) : (sc[r].y & 0xffffu)));
            al[r][0] = half8{a1, a1, a1, a1, a1, a1, a1, a1};
            al[r][1] = half8{a2, a2, a2, a2, a2, a2, a2, a2};
        }
#pragma unroll
        for (int fm = 0; fm < 4; ++fm) {
            half8 b[NPL][RTW];
#pragma unroll
            for (int r = 0; r < RTW; ++r) {
                const half8 t1 = decode8((fm >> 1) ? pw[r][0].y : pw[r][0].x, fm & 1) * al[r][0];
                const half8 t2 = decode8((fm >> 1) ? pw[r][1].y : pw[r][1].x, fm & 1) * al[r][1];
                if constexpr (FUSE) { b[0][r] = t1 + t2; } else { b[0][r] = t1; b[NPL - 1][r] = t2; }
            }
            // operand reads run one pair of token tiles ahead of the MFMAs that use them (the scheduling barriers keep
            // them there: left alone the compiler puts each read right before its wait)
            auto operand = [&](int mt) {
                return __builtin_bit_cast(
                    half8, *reinterpret_cast<const uintx4 *>(xb + (mt >> 2) * (16 * kTileChunk) + (mt & 3) * 256 + fm * 64));
            };
            half8 a[3][2];
            a[0][0] = operand(0);
            a[0][1] = operand(1);
            a[1][0] = operand(2);
            a[1][1] = operand(3);
#pragma unroll
            for (int mp = 0; mp < MTW / 2; ++mp) {
                if (mp + 2 < MTW / 2) {
                    a[(mp + 2) % 3][0] = operand(2 * mp + 4);
                    a[(mp + 2) % 3][1] = operand(2 * mp + 5);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
                        for (int r = 0; r < RTW; ++r)
                            acc[r][2 * mp + i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mp % 3][i], b[pl][r], acc[r][2 * mp + i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    uintx2 pa[RTW][2], pb[RTW][2], sa[RTW], sb[RTW];
    stage(0, 0);
    load_group(pa, sa, 0);
#pragma unroll
    for (int r = 0; r < RTW; ++r) { pb[r][0] = pa[r][0]; pb[r][1] = pa[r][1]; sb[r] = sa[r]; }
    __builtin_amdgcn_s_waitcnt(0);                   // this wave's chunks have landed in LDS
    __syncthreads();

    for (int g = 0; g < NG; g += 2) {
        const bool m1 = g + 1 < NG, m2 = g + 2 < NG;
        if (m1) { stage(g + 1, 1); load_group(pb, sb, g + 1); }
        compute(pa, sa, g);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (m1) {
            if (m2) { stage(g + 2, 0); load_group(pa, sa, g + 2); }
            compute(pb, sb, g + 1);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
    }

    tile_store<RTW, MTW>(acc, y, y_f16, rt_base, nl, M, N, ep, [&](int mt, int j) { return m0 + mt * 16 + 4 * q + j; });
}

template <bool FUSE>
hipError_t launch_gemm_tile3(const uint8_t *records, const uint16_t *x, void *y, int M, const Shape &s, int y_f16,
                             hipStream_t stream, int nb0 = 0, int nb1 = -1, TileEpilogue ep = {nullptr, 0})
{
    const int MB = (M + kTile3Tokens - 1) / kTile3Tokens;
    const int64_t units = ep.gated ? s.RT / 2 : s.RT, per = ep.gated ? 8 : 16;   // pairs per workgroup when gated
    const int NB = nb1 >= 0 ? nb1 : static_cast<int>((units + per - 1) / per);
    const int64_t grid = static_cast<int64_t>((NB - nb0 + 7) / 8) * 8 * MB;
    if (grid <= 0 || grid > kMaxGrid) return hipErrorInvalidValue;
    const size_t lds = 2 * static_cast<size_t>(kTile3BufBytes);
    static std::atomic<bool> configured{false};                  // raise the dynamic LDS limit once per process
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tile3_kernel<FUSE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((gemm_tile3_kernel<FUSE>), dim3(static_cast<unsigned>(grid)), dim3(512), lds, stream, records, x,
                       y, M, static_cast<int>(s.N), static_cast<int>(s.K), static_cast<int>(s.RT),
                       static_cast<int>(s.KS), y_f16, MB, NB, nb0, ep);
    return hipGetLastError();
}

// row blocks (of 64*RTW rows) nb0 .. nb1-1; nb1 < 0: to the end
template <int MTW, bool FUSE, int RTW = 4>
hipError_t launch_gemm_tile(const uint8_t *records, const uint16_t *x, void *y, int M, const Shape &s, int y_f16,
                            hipStream_t stream, int nb0 = 0, int nb1 = -1, TileEpilogue ep = {nullptr, 0})
{
    constexpr int TM = 16 * MTW, NRT = 4 * RTW;
    if (ep.gated && RTW < 2) return hipErrorInvalidValue;   // a wave needs a gate tile and its up tile
    const int MB = (M + TM - 1) / TM;
    const int64_t units = ep.gated ? s.RT / 2 : s.RT, per = ep.gated ? NRT / 2 : NRT;
    const int NB = nb1 >= 0 ? nb1 : static_cast<int>((units + per - 1) / per);
    const int64_t grid = static_cast<int64_t>((NB - nb0 + 7) / 8) * 8 * MB;
    if (grid <= 0 || grid > kMaxGrid) return hipErrorInvalidValue;
    const size_t lds = 2 * static_cast<size_t>(TM / 4) * kTileChunk;
    static std::atomic<bool> configured{false};                  // raise the dynamic LDS limit once per process
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tile_kernel<MTW, FUSE, RTW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((gemm_tile_kernel<MTW, FUSE, RTW>), dim3(static_cast<unsigned>(grid)), dim3(256), lds, stream, records, x,
                       y, M, static_cast<int>(s.N), static_cast<int>(s.K), static_cast<int>(s.RT),
                       static_cast<int>(s.KS), y_f16, MB, NB, nb0, ep);
    return hipGetLastError();
}

// The prefill tiles, largest first.  `units` = 16 x 16 output tiles per workgroup / 2 (one unit = the MFMA work of
// two row tiles x one token tile per field).  Times in microseconds per 32 scale groups, measured on 8B and 70B
// layer shapes: `lone` = a workgroup alone on its CU (the latency floor of the K loop), `rate` = per unit when the
// CU's matrix pipes are the limit; index 0 = both planes through the matrix pipe, 1 = planes summed first.
struct TileKind {
    int row_tiles, tokens, units;
    float lone[2], rate[2];
};
constexpr int kTileKindCount = 5;
constexpr TileKind kTileKinds[kTileKindCount] = {
    {16, 256, 256, {152.f, 104.f}, {0.68f, 0.46f}},   // gemm_tile3_kernel
    {16, 128, 128, {97.f, 66.f}, {0.77f, 0.53f}},     // gemm_tile_kernel<8, ., 4>
    {8, 128, 64, {55.f, 44.f}, {0.75f, 0.54f}},       // gemm_tile_kernel<8, ., 2>
    {8, 64, 32, {32.f, 28.f}, {0.83f, 0.65f}},        // gemm_tile_kernel<4, ., 2>
    {4, 64, 16, {24.f, 22.f}, {1.13f, 0.90f}},        // gemm_tile_kernel<4, ., 1>
};
constexpr double kTileLaunchCost = 3.0;               // a second launch, same scale

// Estimated time of one launch of tile kind k over `row_tiles` row tiles and M tokens: the busiest CU holds
// ceil(workgroups / 256) of them, and never finishes before one workgroup's K loop has run.
double tile_cost(int k, int fused, int row_tiles, int M)
{
    const TileKind &t = kTileKinds[k];
    const int64_t wgs = static_cast<int64_t>((row_tiles + t.row_tiles - 1) / t.row_tiles) * ((M + t.tokens - 1) / t.tokens);
    const double busy = static_cast<double>((wgs + 255) / 256) * t.units * t.rate[fused];
    return busy > t.lone[fused] ? busy : t.lone[fused];
}

double best_tile_cost(int row_tiles, int M)
{
    double c = 1e30;
    for (int k = 0; k < kTileKindCount; ++k) {
        const double ck = tile_cost(k, 0, row_tiles, M);
        c = ck < c ? ck : c;
    }
    return c;
}

// The small-batch kernel on chunks of 64 tokens, in microseconds: a full chunk streams the packed rows once (0.037 per
// row tile and 32 groups, at least 11 for the launch and its ramp); a last chunk of up to 16 / 32 / 48 tokens uses the narrower kernels.
double small_cost(int row_tiles, int groups, int M)
{
    const double stream = 0.037 * row_tiles * groups / 32.0;
    const double full = stream > 11.0 ? stream : 11.0;
    const int rest = M % 64;
    return (M / 64) * full + (rest == 0 ? 0.0 : rest > 48 ? full : rest > 32 ? 0.8 * full : rest > 16 ? 0.6 * full : 0.4 * full);
}

// Launch tile kind k over row tiles rt0 .. rt1-1 (rt0 a multiple of 16; rt1 < 0: to the end, else a multiple of 16).
hipError_t launch_tile_kind(int k, bool fuse, const uint8_t *records, const uint16_t *x, void *y, int M, const Shape &s,
                            int y_f16, hipStream_t stream, int rt0, int rt1, TileEpilogue ep = {nullptr, 0})
{
    const int per = kTileKinds[k].row_tiles;
    const int nb0 = rt0 / per, nb1 = rt1 < 0 ? -1 : rt1 / per;
#define PTQTP_TILE(MTW_, RTW_)                                                                         \
    (fuse ? launch_gemm_tile<MTW_, true, RTW_>(records, x, y, M, s, y_f16, stream, nb0, nb1, ep)       \
          : launch_gemm_tile<MTW_, false, RTW_>(records, x, y, M, s, y_f16, stream, nb0, nb1, ep))
    switch (k) {
        case 0: return fuse ? launch_gemm_tile3<true>(records, x, y, M, s, y_f16, stream, nb0, nb1, ep)
                            : launch_gemm_tile3<false>(records, x, y, M, s, y_f16, stream, nb0, nb1, ep);
        case 1: return PTQTP_TILE(8, 4);
        case 2: return PTQTP_TILE(8, 2);
        case 3: return PTQTP_TILE(4, 2);
        default: return PTQTP_TILE(4, 1);
    }
#undef PTQTP_TILE
}

// ptqtp_tune("tile_variant", v): the tile kind that value v forces (0 = the cost model chooses)
constexpr int kVariantKind[6] = {0, 1, 2, 0, 3, 4};

int g_tune_small_waves = 0, g_tune_tile = 0, g_tune_small_rows = 0, g_tune_small_rows_kernel = -1, g_tune_tile_variant = 0, g_tune_small_fold = -1;

template <int MT, int R, int S, bool PLAN, int ML>
hipError_t launch_gemm_items_impl(const PlanHeader *plan, const uint8_t *records, const uint16_t *x, void *y, int M,
                                  int N, int K, int RT, int KS, int y_f16, int64_t grid, int W, hipStream_t stream,
                                  const uint16_t *residual = nullptr, int gated = 0)
{
    size_t lds = static_cast<size_t>(W) * R * MT * 256 * sizeof(float);
    if (lds < static_cast<size_t>(W) * kSlotBytes) lds = static_cast<size_t>(W) * kSlotBytes;
    static std::atomic<bool> configured{false};                  // the slots of 8 waves exceed the default 64 KB limit
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_items_kernel<MT, R, S, PLAN, ML>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 8 * kSlotBytes);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((gemm_items_kernel<MT, R, S, PLAN, ML>), dim3(static_cast<unsigned>(grid)), dim3(W * 64), lds,
                       stream, plan, records, x, y, M, N, K, RT, KS, y_f16, residual, gated);
    return hipGetLastError();
}

// load instructions per 16-token tile needed for M tokens
template <int MT, int R, int S, bool PLAN>
hipError_t launch_gemm_items_ml(const PlanHeader *plan, const uint8_t *records, const uint16_t *x, void *y, int M,
                                int N, int K, int RT, int KS, int y_f16, int64_t grid, int W, hipStream_t stream,
                                const uint16_t *residual = nullptr, int gated = 0)
{
    if constexpr (MT == 1) {
        if (M <= 2)
            return launch_gemm_items_impl<MT, R, S, PLAN, 1>(plan, records, x, y, M, N, K, RT, KS, y_f16, grid, W, stream, residual, gated);
        if (M <= 4)
            return launch_gemm_items_impl<MT, R, S, PLAN, 2>(plan, records, x, y, M, N, K, RT, KS, y_f16, grid, W, stream, residual, gated);
        if (M <= 8)
            return launch_gemm_items_impl<MT, R, S, PLAN, 4>(plan, records, x, y, M, N, K, RT, KS, y_f16, grid, W, stream, residual, gated);
    }
    return launch_gemm_items_impl<MT, R, S, PLAN, 8>(plan, records, x, y, M, N, K, RT, KS, y_f16, grid, W, stream, residual, gated);
}

template <int MT, int R, int S>
hipError_t launch_gemm_items(const uint8_t *records, const uint16_t *x, void *y, int M, const Shape &s, int y_f16,
                             hipStream_t stream, const uint16_t *residual = nullptr, int gated = 0, int waves = 0)
{
    // measured: 8 waves per item, except for the register-heavy 64-token x 2-tile case: 2 waves there on 8B shapes
    // (K = 4096), 4 on longer rows (70B down, K = 28672, at 64 tokens: 166 -> 105 us)
    int W = g_tune_small_waves > 0 ? g_tune_small_waves : waves > 0 ? waves : (MT * R >= 6 ? (s.KS > 16 ? 4 : 2) : 8);
    if (W > (items_eight_waves(MT, R) ? 8 : 4)) W = items_eight_waves(MT, R) ? 8 : 4;
    while (W > 1 && W > s.KS) W /= 2;
    const int64_t grid = gated ? s.RT / 2 : (s.RT + R - 1) / R;
    return launch_gemm_items_ml<MT, R, S, false>(nullptr, records, x, y, M, static_cast<int>(s.N), static_cast<int>(s.K),
                                                 static_cast<int>(s.RT), static_cast<int>(s.KS), y_f16, grid, W, stream,
                                                 residual, gated);
}

// batched: every item of a plan, all linears with the same M (2..64)
hipError_t launch_gemm_items_plan(const PlanHeader *plan, int64_t items, int M, hipStream_t stream)
{
    const int W = g_tune_small_waves > 0 ? (g_tune_small_waves > 8 ? 8 : g_tune_small_waves) : 4;
    if (M <= 16) return launch_gemm_items_ml<1, 1, 2, true>(plan, nullptr, nullptr, nullptr, M, 0, 0, 0, 0, 0, items, W, stream);
    if (M <= 32) return launch_gemm_items_ml<2, 1, 1, true>(plan, nullptr, nullptr, nullptr, M, 0, 0, 0, 0, 0, items, W, stream);
    if (M <= 48) return launch_gemm_items_ml<3, 1, 1, true>(plan, nullptr, nullptr, nullptr, M, 0, 0, 0, 0, 0, items, W, stream);
    return launch_gemm_items_ml<4, 1, 1, true>(plan, nullptr, nullptr, nullptr, M, 0, 0, 0, 0, 0, items, W, stream);
}

// ------------------------------------------------------------------------------------------
// small-batch kernel for batched launches: workgroup = NW waves x RTW row tiles sharing one activation tile
// ------------------------------------------------------------------------------------------
// Wave w owns the RTW consecutive row tiles from NW*RTW*group + w*RTW over the whole K; per 256-column
// step the workgroup loads the step's activations once (MT*16 tokens x 512 B into a double-buffered LDS
// tile; one barrier per step) and every wave reads its MFMA A operands from there, so a linear's
// activations cross from L2 into the CU once per NW*RTW row tiles (with per-item loads that traffic
// exceeds the weight bytes from 8 tokens on) and no cross-wave reduction is needed: each wave stores its
// own rows.  Needs NW*RTW <= 16 row tiles of the same linear per workgroup, which batch plans guarantee
// (items are padded to a multiple of sixteen per linear).
//
// FOLD: the group scale is multiplied into the expanded trits before the matrix pipe
// (alpha * {0,+-1} is exact in fp16 and alpha*t*x is exact in fp32), so both planes and all
// groups accumulate into one set of MFMA accumulators that lives across the whole K loop:
// no per-group accumulator reset and rescale.  Pays once a decoded operand is reused by
// more than two token tiles: measured on the 8B stack, 17..32 tokens run 6-8 % faster
// without the fold, 33..64 tokens 5 % faster with it.
// At least two waves per SIMD (at most 256 registers per lane) wherever the accumulators allow:
// the compiler then keeps MFMA results in ordinary VGPRs and the rescale reads them in place.
// The activation tile goes from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers, no address arithmetic per row).  One instruction moves a 1-KiB chunk = the 512 bytes (one 256-column
// step) of TWO tokens, lane t*32+p bringing 16-byte piece p of token t.  Chunk c of a 32-token block holds tokens c
// and c+16 and starts at c*1040 bytes, so the 16 tokens of an MFMA token tile sit in 16 chunks skewed by 16 bytes
// each and the operand read stays one conflict-free ds_read_b128.
// (With 16 tokens or fewer a chunk holds one token and 528 bytes suffice.)
template <int MT>
constexpr int kRowsChunk = MT == 1 ? 528 : 1040;
template <int MT>
__device__ __forceinline__ constexpr int rows_operand_offset(int mt, int f) {
    return (mt >> 1) * (16 * kRowsChunk<MT>) + (mt & 1) * 512 + f * 64;
}

template <int MT, int RTW, bool FOLD, int NW = 4, bool FUSE = false>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu((!FOLD && MT * RTW >= 8) ? 1 : 2)))
gemm_rows_kernel(const PlanHeader *__restrict__ plan, int M)
{
    extern __shared__ char xtile[];                  // [2][(MT+1)/2 blocks of 32 tokens][16 chunks]
    constexpr int kBuf = ((MT + 1) / 2) * 16 * kRowsChunk<MT>;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nl = lane & 15, q = lane >> 4;
    const int item0 = blockIdx.x * (NW * RTW);
    if (item0 >= plan->total_items) return;
    const LinearDesc *table = reinterpret_cast<const LinearDesc *>(plan + 1);
    const int32_t *map = reinterpret_cast<const int32_t *>(table + plan->count);
    const LinearDesc *dp = table + map[item0];
    const int N = dp->N, K = dp->K, RT = dp->RT, KS = dp->KS, y_f16 = plan->y_f16;
    const int rt_first = item0 - dp->first_item + w * RTW;      // this wave's RTW consecutive row tiles
    const uint8_t *rec0[RTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        const int rt = rt_first + r < RT ? rt_first + r : RT - 1;    // past the end: shadow the last tile, store nothing
        rec0[r] = dp->records + static_cast<size_t>(rt) * KS * kRecordBytes;
    }
    const uint16_t *x = dp->x;
    const int rot = (blockIdx.x * 5) % KS;

    const char *xop = xtile + nl * kRowsChunk<MT> + q * 16;

    floatx4 yacc[RTW][MT];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) yacc[r][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto step_of = [&](int i) { int ks = i + rot; return ks >= KS ? ks - KS : ks; };
    auto load_rec = [&](StepRegs (&r)[RTW], int ks) {
#pragma unroll
        for (int t = 0; t < RTW; ++t) {
            const uint8_t *rec = rec0[t] + static_cast<size_t>(ks) * kRecordBytes;
            r[t].p1 = load_stream<uintx4>(rec + lane * 16);
            r[t].p2 = load_stream<uintx4>(rec + kPlaneBytes + lane * 16);
            r[t].sc = load_stream<uintx2>(rec + 2 * kPlaneBytes + nl * 8);
        }
    };
    auto compute = [&](const StepRegs (&r)[RTW], int buf) {
        const char *xb = xop + buf * kBuf;
        if constexpr (FOLD) {
            // operand reads run one 32-column field ahead of the MFMAs that use them
            half8 a[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                a[0][mt] = __builtin_bit_cast(half8, *reinterpret_cast<const uintx4 *>(xb + rows_operand_offset<MT>(mt, 0)));
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                const int g2 = f >> 2, fm = f & 3;
                const int wi = 2 * g2 + (fm >> 1), par = fm & 1;
                if (f + 1 < 8) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        a[(f + 1) & 1][mt] = __builtin_bit_cast(
                            half8, *reinterpret_cast<const uintx4 *>(xb + rows_operand_offset<MT>(mt, f + 1)));
                }
                constexpr int NPL = FUSE ? 1 : 2;
                half8 b[NPL][RTW];
#pragma unroll
                for (int t = 0; t < RTW; ++t) {
                    const _Float16 a1 = __builtin_bit_cast(_Float16, static_cast<uint16_t>(g2 ? (r[t].sc.x >> 16) : (r[t].sc.x & 0xffffu)));
                    const _Float16 a2 = __builtin_bit_cast(_Float16, static_cast<uint16_t>(g2 ? (r[t].sc.y >> 16) : (r[t].sc.y & 0xffffu)));
                    const half8 w1 = decode8(r[t].p1[wi], par) * half8{a1, a1, a1, a1, a1, a1, a1, a1};
                    const half8 w2 = decode8(r[t].p2[wi], par) * half8{a2, a2, a2, a2, a2, a2, a2, a2};
                    if constexpr (FUSE) { b[0][t] = w1 + w2; } else { b[0][t] = w1; b[NPL - 1][t] = w2; }
                }
                // consecutive MFMAs write different accumulators
#pragma unroll
                for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int t = 0; t < RTW; ++t)
                            yacc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[f & 1][mt], b[pl][t], yacc[t][mt], 0, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int g2 = 0; g2 < 2; ++g2) {
            {
            floatx4 acc1[RTW][MT], acc2[RTW][MT];
#pragma unroll
            for (int t = 0; t < RTW; ++t)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) { acc1[t][mt] = floatx4{0.f, 0.f, 0.f, 0.f}; acc2[t][mt] = floatx4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) {
                const int wi = 2 * g2 + (fm >> 1), par = fm & 1;
                half8 b1[RTW], b2[RTW];
#pragma unroll
                for (int t = 0; t < RTW; ++t) { b1[t] = decode8(r[t].p1[wi], par); b2[t] = decode8(r[t].p2[wi], par); }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const half8 a = __builtin_bit_cast(
                        half8, *reinterpret_cast<const uintx4 *>(xb + rows_operand_offset<MT>(mt, g2 * 4 + fm)));
#pragma unroll
                    for (int t = 0; t < RTW; ++t) {
                        acc1[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b1[t], acc1[t][mt], 0, 0, 0);
                        acc2[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b2[t], acc2[t][mt], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < RTW; ++t) {
                const float a1 = half_bits_to_float(g2 ? (r[t].sc.x >> 16) : (r[t].sc.x & 0xffffu));
                const float a2 = half_bits_to_float(g2 ? (r[t].sc.y >> 16) : (r[t].sc.y & 0xffffu));
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        yacc[t][mt][j] = fmaf(a1, acc1[t][mt][j], yacc[t][mt][j]);
                        yacc[t][mt][j] = fmaf(a2, acc2[t][mt][j], yacc[t][mt][j]);
                    }
            }
            }
        }
    };
    // staging role: wave w brings in chunks w, w+NW, ... of the step; lane t*32+p: piece p of token c + 16*t
    auto stage_direct = [&](int ks, int buf) {
        constexpr int NCH = 16 * ((MT + 1) / 2);
        static_assert(NCH % NW == 0, "the chunks of a step divide among the waves");
        int kc = ks * kStepK + (lane & 31) * 8;
        kc = kc < K ? kc : kc - 128;                 // padded half record: its trits are zero
        if (MT > 1 || lane < 32) {                   // 16 tokens or fewer: the second token of a chunk does not exist
#pragma unroll
            for (int j = 0; j < NCH / NW; ++j) {
                const int c = w + NW * j;            // chunk of the step
                int m = (c >> 4) * 32 + (c & 15) + (lane >> 5) * 16;
                m = m < M ? m : M - 1;               // rows past M: duplicates, never stored
                asm volatile("" : "+v"(m));          // keep the row address out of loop-invariant registers
                lds_direct_load16(x + static_cast<size_t>(m) * K + kc, xtile + buf * kBuf + c * kRowsChunk<MT>);
            }
        }
    };

    StepRegs ra[RTW], rb[RTW];
    stage_direct(step_of(0), 0);
    load_rec(ra, step_of(0));
#pragma unroll
    for (int t = 0; t < RTW; ++t) rb[t] = ra[t];
    __builtin_amdgcn_s_waitcnt(0);               // this wave's chunks have landed in LDS
    __syncthreads();
    for (int i = 0; i < KS; i += 2) {
        const bool m1 = i + 1 < KS, m2 = i + 2 < KS;
        if (m1) { stage_direct(step_of(i + 1), 1); load_rec(rb, step_of(i + 1)); }
        compute(ra, 0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (m1) {
            if (m2) { stage_direct(step_of(i + 2), 0); load_rec(ra, step_of(i + 2)); }
            compute(rb, 1);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
    }

#pragma unroll
    for (int t = 0; t < RTW; ++t) {
        const int rt = rt_first + t;
        const int n = rt * kTileRows + nl;
        if (rt < RT && n < N) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int m = mt * 16 + 4 * q + j;
                    if (m < M) {
                        const size_t off = static_cast<size_t>(m) * N + n;
                        if (y_f16) reinterpret_cast<_Float16 *>(dp->y)[off] = static_cast<_Float16>(yacc[t][mt][j]);
                        else reinterpret_cast<float *>(dp->y)[off] = yacc[t][mt][j];
                    }
                }
        }
    }
}

template <int MT, int RTW, bool FOLD, int NW = 4, bool FUSE = false>
hipError_t launch_gemm_rows(const PlanHeader *plan, int64_t items, int M, hipStream_t stream)
{
    static_assert(NW * RTW <= kPlanPad, "a workgroup's row tiles belong to one linear");
    const size_t lds = 2 * static_cast<size_t>((MT + 1) / 2) * 16 * kRowsChunk<MT>;
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_rows_kernel<MT, RTW, FOLD, NW, FUSE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((gemm_rows_kernel<MT, RTW, FOLD, NW, FUSE>), dim3(static_cast<unsigned>((items + NW * RTW - 1) / (NW * RTW))),
                       dim3(64 * NW), lds, stream, plan, M);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// small-batch item kernel with its loads one step ahead of the arithmetic
// ------------------------------------------------------------------------------------------
// One linear per launch has too few items to hide a DRAM round trip behind other workgroups (70B gate at 32
// tokens: 1.75 waves per SIMD), so here a wave hides it behind its own arithmetic.  Item, wave roles, rotated
// start, final reduction and epilogue are those of gemm_items_kernel; what differs is the K loop: the step's
// activations go from global memory straight into the wave's LDS slot (global_load_lds_dwordx4 in the chunk
// layout of gemm_rows_kernel: no staging registers), and as soon as the wave has read its MFMA operands out of
// the slot it issues the next step's activation loads into the same slot and the next step's records into a
// second register set; both are in flight while the MFMAs of the present step run.
// A wave's LDS reads are not ordered against its own later direct-to-LDS loads (the data comes back on another
// path), hence the wait for the operand reads before the next loads are issued.
template <int MT, int R>
__global__ void __launch_bounds__(items_eight_waves(MT, R) ? 512 : 256)
gemm_items_ahead_kernel(const uint8_t *__restrict__ records, const uint16_t *__restrict__ x, void *__restrict__ y,
                        int M, int N, int K, int RT, int KS, int y_f16, const uint16_t *__restrict__ residual, int gated)
{
    extern __shared__ float red[];                     // [W][R][MT][16 tokens][16 rows]; first used as activation slots
    constexpr int kChunk = kRowsChunk<MT>;
    constexpr int kSlot = ((MT + 1) / 2) * 16 * kChunk;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int W = blockDim.x >> 6;
    const int nl = lane & 15, q = lane >> 4;
    const int rstride = gated ? RT / 2 : 1;
    const int rt0 = gated ? blockIdx.x : blockIdx.x * R;
    const int rot = (rt0 * 5) % KS;

    float yacc[R][MT][4];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j) yacc[r][mt][j] = 0.f;

    char *slot = reinterpret_cast<char *>(red) + w * kSlot;
    const char *xop = slot + nl * kChunk + q * 16;

    struct Recs { uintx4 p1[R], p2[R]; uintx2 sc[R]; };
    auto step_of = [&](int ks) { const int kse = ks + rot; return kse >= KS ? kse - KS : kse; };
    auto load_recs = [&](Recs &c, int kse) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int rt = rt0 + r * rstride < RT ? rt0 + r * rstride : rt0;
            const uint8_t *rec = records + (static_cast<size_t>(rt) * KS + kse) * kRecordBytes;
            c.p1[r] = load_stream<uintx4>(rec + lane * 16);
            c.p2[r] = load_stream<uintx4>(rec + kPlaneBytes + lane * 16);
            c.sc[r] = load_stream<uintx2>(rec + 2 * kPlaneBytes + nl * 8);
        }
    };
    // chunk c = 1 KiB = 512 B of token t0(c) and of token t0(c) + 16 (one token with up to 16 tokens)
    auto stage = [&](int kse) {
        constexpr int NCH = 16 * ((MT + 1) / 2);
        int kc = kse * kStepK + (lane & 31) * 8;
        kc = kc < K ? kc : kc - 128;                 // padded half record: its trits are zero
        if (MT > 1 || lane < 32) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int t0 = (c >> 4) * 32 + (c & 15);
                if (t0 < M) {                        // uniform: chunks of tokens that do not exist are not loaded
                    int m = t0 + (lane >> 5) * 16;
                    m = m < M ? m : M - 1;           // second token past M: a duplicate, never stored
                    asm volatile("" : "+v"(m));      // keep the row address out of loop-invariant registers
                    lds_direct_load16(x + static_cast<size_t>(m) * K + kc, slot + c * kChunk);
                }
            }
        }
    };
    uintx4 xa[MT][8];
    auto operands = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the step's activations are in the slot, its records in registers
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int f = 0; f < 8; ++f)
                xa[mt][f] = *reinterpret_cast<const uintx4 *>(xop + rows_operand_offset<MT>(mt, f));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");    // the slot may be overwritten from here on
    };
    auto compute = [&](const Recs &c) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float a1g0 = half_bits_to_float(c.sc[r].x & 0xffffu), a1g1 = half_bits_to_float(c.sc[r].x >> 16);
            const float a2g0 = half_bits_to_float(c.sc[r].y & 0xffffu), a2g1 = half_bits_to_float(c.sc[r].y >> 16);
            floatx4 acc[MT];
            group_sum<MT, 0>(xa, c.p1[r], acc);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a1g0, acc[mt][j], yacc[r][mt][j]);
            group_sum<MT, 1>(xa, c.p1[r], acc);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a1g1, acc[mt][j], yacc[r][mt][j]);
            group_sum<MT, 0>(xa, c.p2[r], acc);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a2g0, acc[mt][j], yacc[r][mt][j]);
            group_sum<MT, 1>(xa, c.p2[r], acc);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) yacc[r][mt][j] = fmaf(a2g1, acc[mt][j], yacc[r][mt][j]);
        }
    };

    Recs ra, rb;
    int ks = w;                                        // this wave's steps: w, w + W, ...
    if (ks < KS) { stage(step_of(ks)); load_recs(ra, step_of(ks)); }
    while (ks < KS) {
        operands();
        if (ks + W < KS) { stage(step_of(ks + W)); load_recs(rb, step_of(ks + W)); }
        compute(ra);
        ks += W;
        if (ks >= KS) break;
        operands();
        if (ks + W < KS) { stage(step_of(ks + W)); load_recs(ra, step_of(ks + W)); }
        compute(rb);
        ks += W;
    }

    constexpr int OUT = R * MT * 256;
    __syncthreads();                                   // the slots are dead: the space becomes `red`
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                red[w * OUT + ((r * MT + mt) * 16 + 4 * q + j) * 16 + nl] = yacc[r][mt][j];
    __syncthreads();
    const int n_out = gated ? N / 2 : N;              // gated: silu(gate) * up, one output per (gate, up) row pair
    for (int o = threadIdx.x; o < (gated ? OUT / R : OUT); o += blockDim.x) {
        float s = 0.f;
        for (int ww = 0; ww < W; ++ww) s += red[ww * OUT + o];
        const int on = o & 15, t = o >> 4;
        const int m = (t / 16 % MT) * 16 + (t & 15), r = t / (16 * MT);
        const int n = (rt0 + r) * kTileRows + on;
        if (m < M && rt0 + r * rstride < RT && n < n_out) {
            if (gated) {
                float u = 0.f;
                for (int ww = 0; ww < W; ++ww) u += red[ww * OUT + o + MT * 256];
                s = (s / (1.0f + __expf(-s))) * u;
            }
            const size_t off = static_cast<size_t>(m) * n_out + n;
            if (residual != nullptr) s += half_bits_to_float(load_global<uint16_t>(residual + off));
            if (y_f16) reinterpret_cast<_Float16 *>(y)[off] = static_cast<_Float16>(s);
            else reinterpret_cast<float *>(y)[off] = s;
        }
    }
}

int g_tune_small_ahead = -1;

template <int MT, int R>
hipError_t launch_gemm_items_ahead(const uint8_t *records, const uint16_t *x, void *y, int M, const Shape &s, int y_f16,
                                   hipStream_t stream, const uint16_t *residual, int gated, int waves)
{
    constexpr int kSlot = ((MT + 1) / 2) * 16 * kRowsChunk<MT>;
    constexpr int kMaxLds = 8 * 16 * kRowsChunk<2>;             // eight slots of 32 tokens = four of 64
    constexpr int kMaxW = (!items_eight_waves(MT, R) || MT > 2) ? 4 : 8;
    int W = g_tune_small_waves > 0 ? g_tune_small_waves : waves > 0 ? waves : (MT * R >= 6 ? (s.KS > 16 ? 4 : 2) : 8);
    if (W > kMaxW) W = kMaxW;
    while (W > 1 && W > s.KS) W /= 2;
    size_t lds = static_cast<size_t>(W) * R * MT * 256 * sizeof(float);
    if (lds < static_cast<size_t>(W) * kSlot) lds = static_cast<size_t>(W) * kSlot;
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_items_ahead_kernel<MT, R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    const int64_t grid = gated ? s.RT / 2 : (s.RT + R - 1) / R;
    hipLaunchKernelGGL((gemm_items_ahead_kernel<MT, R>), dim3(static_cast<unsigned>(grid)), dim3(W * 64), lds, stream,
                       records, x, y, M, static_cast<int>(s.N), static_cast<int>(s.K), static_cast<int>(s.RT),
                       static_cast<int>(s.KS), y_f16, residual, gated);
    return hipGetLastError();
}

// 2..64 tokens: the small-batch item kernel in the shape that measured best
hipError_t launch_small(const uint8_t *records, const uint16_t *x, void *y, int M, const Shape &s, int f16,
                        hipStream_t stream, const uint16_t *residual = nullptr, int gated = 0)
{
    // measured on 8B shapes: two row tiles per item (sharing one set of activation operands) when the layer has
    // many row tiles, and always for 17..32 tokens; one otherwise (R = 4 exists for up to 32 tokens)
    int R = s.RT >= 512 ? 2 : 1;
    if (M > 16 && M <= 32) R = 2;
    // four on wide layers, where items are plentiful and the activations re-read per item weigh most (70B gate,
    // 28672 rows: 16 tokens 31.8 -> 29.7 us, 32 tokens 53 -> 44 us; 8B gate, 14336 rows, 17..32 tokens as eight
    // waves: 17.1 -> 14.5 us; slower on every narrower layer)
    if (s.RT >= 1536 && M >= 16 && M <= 32) R = 4;
    int waves = 0;                                     // 0: the launcher's own rule
    if (s.RT >= 768 && s.RT < 1536 && M > 16 && M <= 32) { R = 4; waves = 8; }
    // the kernel with its loads one step ahead, where it measured faster: 17..32 tokens on layers of few row tiles
    // as one tile per item and eight waves (8B q 9.1 -> 7.6 us, 8B down 23.2 -> 18.0 us, 70B k 14.3 -> 10.9 us),
    // 33..64 tokens on layers of 512..1024 row tiles with long rows (70B q at 64 tokens 33.7 -> 30.8 us, 70B down
    // 105 -> 91 us); equal or slower elsewhere (everything up to 16 tokens, 8B shapes above 32)
    bool ahead = false;
    if (g_tune_small_ahead != 0 && !gated) {
        if (M > 16 && M <= 32 && s.RT < 512) { ahead = true; R = 1; waves = 8; }
        if (M > 32 && s.RT >= 512 && s.RT <= 1024 && s.KS >= 32) { ahead = true; R = 2; }
    }
    if (g_tune_small_rows > 0) { R = g_tune_small_rows; waves = 0; }
    if (gated) { R = 2; waves = 0; }                   // a (gate tile, up tile) pair per item
    if (g_tune_small_ahead >= 0) ahead = g_tune_small_ahead == 1;
    if (ahead && M > 16 && R <= 2) {
        if (M <= 32) return R == 2 ? launch_gemm_items_ahead<2, 2>(records, x, y, M, s, f16, stream, residual, gated, waves)
                                   : launch_gemm_items_ahead<2, 1>(records, x, y, M, s, f16, stream, residual, gated, waves);
        if (M <= 48) return R == 2 ? launch_gemm_items_ahead<3, 2>(records, x, y, M, s, f16, stream, residual, gated, waves)
                                   : launch_gemm_items_ahead<3, 1>(records, x, y, M, s, f16, stream, residual, gated, waves);
        return R == 2 ? launch_gemm_items_ahead<4, 2>(records, x, y, M, s, f16, stream, residual, gated, waves)
                      : launch_gemm_items_ahead<4, 1>(records, x, y, M, s, f16, stream, residual, gated, waves);
    }
    if (M <= 16) return R == 4 ? launch_gemm_items<1, 4, 1>(records, x, y, M, s, f16, stream, residual, gated)
                      : R == 2 ? launch_gemm_items<1, 2, 1>(records, x, y, M, s, f16, stream, residual, gated)
                               : launch_gemm_items<1, 1, 2>(records, x, y, M, s, f16, stream, residual, gated);
    if (M <= 32) return R == 4 ? launch_gemm_items<2, 4, 1>(records, x, y, M, s, f16, stream, residual, gated, waves)
                      : R == 2 ? launch_gemm_items<2, 2, 1>(records, x, y, M, s, f16, stream, residual, gated)
                               : launch_gemm_items<2, 1, 1>(records, x, y, M, s, f16, stream, residual, gated);
    if (M <= 48) return R == 2 ? launch_gemm_items<3, 2, 1>(records, x, y, M, s, f16, stream, residual, gated)
                               : launch_gemm_items<3, 1, 1>(records, x, y, M, s, f16, stream, residual, gated);
    return R == 2 ? launch_gemm_items<4, 2, 1>(records, x, y, M, s, f16, stream, residual, gated)
                  : launch_gemm_items<4, 1, 1>(records, x, y, M, s, f16, stream, residual, gated);
}

}  // namespace

// one stage of a decode chain at 1..64 tokens (called from ptqtp_chain.hip): the small-batch item kernel with the
// stage's epilogue in its final reduction
namespace ptqtp_detail {
// One chain stage at many tokens on the cheapest single MFMA tile launch (a gated stage needs two row tiles per wave)
hipError_t tile_stage(const uint8_t *records, const uint16_t *x, void *y, const uint16_t *residual, int M, int64_t N,
                      int64_t K, int y_f16, int gated, bool fuse_planes, hipStream_t stream)
{
    Shape s;
    s.N = N; s.K = K; s.NG = K / 128;
    s.RT = (N + kTileRows - 1) / kTileRows;
    s.KS = (K + kStepK - 1) / kStepK;
    const int kinds = gated ? kTileKindCount - 1 : kTileKindCount;
    int best = 1;
    double cost = 1e30;
    for (int k = 0; k < kinds; ++k) {
        const double c = tile_cost(k, fuse_planes ? 1 : 0, static_cast<int>(s.RT), M);
        if (c < cost) { cost = c; best = k; }
    }
    if (g_tune_tile_variant != 0) {                  // ptqtp_tune("tile_variant"), where the stage allows that tile
        if (kVariantKind[g_tune_tile_variant] < kinds) best = kVariantKind[g_tune_tile_variant];
    }
    return launch_tile_kind(best, fuse_planes, records, x, y, M, s, y_f16, stream, 0, -1, TileEpilogue{residual, gated});
}

hipError_t small_batch_stage(const uint8_t *records, const uint16_t *x, void *y, const uint16_t *residual, int M,
                             int64_t N, int64_t K, int y_f16, int gated, hipStream_t stream)
{
    Shape s;
    s.N = N; s.K = K; s.NG = K / 128;
    s.RT = (N + kTileRows - 1) / kTileRows;
    s.KS = (K + kStepK - 1) / kStepK;
    return launch_small(records, x, y, M, s, y_f16, stream, residual, gated);
}
}

namespace {


// Which kernels a forward of M > 1 tokens runs (host logic only; ptqtp_gemm_route reports it).
struct Route {
    int path;                   // PTQTP_ROUTE_*
    int kind;                   // tile kind of the (first) launch, index into kTileKinds
    int split_row_tile;         // two launches: the first covers row tiles below this multiple of 16
    int second_kind;            // tile kind of the second launch, or -1
};

Route choose_route(const Shape &s, int M, bool fuse_planes)
{
    Route r = {PTQTP_ROUTE_SMALL, -1, 0, -1};
    const int RT = static_cast<int>(s.RT), NG = static_cast<int>(s.NG);
    const bool tile = M >= 256 || g_tune_tile == 1 ||
                      (g_tune_tile == 0 && M > 32 && best_tile_cost(RT, M) * NG / 32.0 < small_cost(RT, NG, M));
    if (!tile) {
        // 65..255 tokens without a tile: chunks of 64 tokens
        r.path = M > PTQTP_GEMM_SMALL_MAX_M ? PTQTP_ROUTE_SMALL_CHUNKS : PTQTP_ROUTE_SMALL;
        return r;
    }
    r.path = PTQTP_ROUTE_TILE;
    if (g_tune_tile_variant != 0) {
        r.kind = kVariantKind[g_tune_tile_variant];
        return r;
    }
    const int fz = fuse_planes ? 1 : 0;
    // one launch of the cheapest tile ...
    double cost = 1e30;
    for (int k = 0; k < kTileKindCount; ++k) {
        const double c = tile_cost(k, fz, RT, M);
        if (c < cost) { cost = c; r.kind = k; }
    }
    // ... or whole rounds of 256 x 256 tiles for the first row blocks, then the cheapest smaller tile for the rest,
    // when the last round of big tiles would leave most CUs idle
    const int MB3 = (M + 255) / 256, NB16 = (RT + 15) / 16;
    const int64_t t3 = static_cast<int64_t>(NB16) * MB3;
    const int nb3 = static_cast<int>(t3 / 256 * 256 / MB3);
    if (nb3 > 0 && nb3 < NB16) {
        const double head = tile_cost(0, fz, nb3 * 16, M);
        for (int k = 1; k < kTileKindCount; ++k) {
            const double c = head + tile_cost(k, fz, RT - nb3 * 16, M) + kTileLaunchCost;
            if (c < cost) { cost = c; r.kind = 0; r.second_kind = k; r.split_row_tile = nb3 * 16; }
        }
    }
    return r;
}

ptqtp_status run_forward(const void *packed, const uint16_t *x, void *y, int32_t y_dtype, int64_t M,
                         int64_t N, int64_t K, int32_t group, void *stream_, int64_t max_m, bool fuse_planes = false)
{
    Shape s;
    ptqtp_status st;
    if (!packed || !x || !y) return PTQTP_ERR_NULL;
    if (!make_shape(M, N, K, group, &s, &st)) return st;
    if (M > max_m) return PTQTP_ERR_SHAPE;
    if (y_dtype != PTQTP_F32 && y_dtype != PTQTP_F16) return PTQTP_ERR_DTYPE;
    if (!aligned(packed, 256) || !aligned(x, 16) || !aligned(y, y_dtype == PTQTP_F16 ? 2 : 4)) return PTQTP_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const uint8_t *records = static_cast<const uint8_t *>(packed) + kHeaderBytes;
    const int Mi = static_cast<int>(M), f16 = (y_dtype == PTQTP_F16);
    hipError_t e;
    if (M == 1) {
        LinearDesc d;
        d.records = records; d.x = x; d.y = y;
        d.N = static_cast<int32_t>(s.N); d.K = static_cast<int32_t>(s.K);
        d.RT = static_cast<int32_t>(s.RT); d.KS = static_cast<int32_t>(s.KS);
        d.first_item = 0; d.pad = 0;
        e = launch_items<false>(nullptr, d, f16, s.RT, s.KS, stream);
    } else {
        const Route r = choose_route(s, Mi, fuse_planes);
        if (r.path == PTQTP_ROUTE_TILE) {
            if (r.second_kind < 0) {
                e = launch_tile_kind(r.kind, fuse_planes, records, x, y, Mi, s, f16, stream, 0, -1);
            } else {
                e = launch_tile_kind(r.kind, fuse_planes, records, x, y, Mi, s, f16, stream, 0, r.split_row_tile);
                if (e == hipSuccess)
                    e = launch_tile_kind(r.second_kind, fuse_planes, records, x, y, Mi, s, f16, stream, r.split_row_tile, -1);
            }
        } else if (r.path == PTQTP_ROUTE_SMALL_CHUNKS) {
            // the small-batch kernel on chunks of 64 tokens
            e = hipSuccess;
            for (int m0 = 0; m0 < Mi && e == hipSuccess; m0 += 64) {
                const int mc = Mi - m0 < 64 ? Mi - m0 : 64;
                const uint16_t *xc = x + static_cast<size_t>(m0) * s.K;
                void *yc = static_cast<char *>(y) + static_cast<size_t>(m0) * s.N * (f16 ? 2 : 4);
                e = launch_small(records, xc, yc, mc, s, f16, stream);
            }
        } else {
            e = launch_small(records, x, y, Mi, s, f16, stream);
        }
    }
    return e == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

}  // namespace

extern "C" {

int32_t ptqtp_version(void) { return 100; }

const char *ptqtp_status_string(ptqtp_status s) {
    switch (s) {
        case PTQTP_OK: return "ok";
        case PTQTP_ERR_NULL: return "null pointer";
        case PTQTP_ERR_SHAPE: return "invalid shape";
        case PTQTP_ERR_GROUP: return "unsupported group size";
        case PTQTP_ERR_SIZE: return "buffer too small";
        case PTQTP_ERR_DTYPE: return "unsupported output dtype";
        case PTQTP_ERR_ALIGN: return "misaligned pointer";
        case PTQTP_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

size_t ptqtp_packed_bytes(int64_t M, int64_t N, int64_t K, int32_t group) {
    Shape s;
    ptqtp_status st;
    if (!make_shape(M, N, K, group, &s, &st)) return 0;
    return static_cast<size_t>(kHeaderBytes) + static_cast<size_t>(s.RT) * s.KS * kRecordBytes;
}

size_t ptqtp_workspace_bytes(int64_t, int64_t, int64_t, int32_t) { return 0; }

ptqtp_status ptqtp_check_blob(const void *packed, size_t packed_bytes, int64_t N, int64_t K, int32_t group,
                              int32_t *dev_status, void *stream_) {
    if (!packed || !dev_status) return PTQTP_ERR_NULL;
    Shape s;
    ptqtp_status st;
    if (!make_shape(1, N, K, group, &s, &st)) return st;
    if (packed_bytes < ptqtp_packed_bytes(1, N, K, group)) return PTQTP_ERR_SIZE;
    if (!aligned(packed, 256) || !aligned(dev_status, 4)) return PTQTP_ERR_ALIGN;
    hipLaunchKernelGGL(check_blob_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream_),
                       static_cast<const uint8_t *>(packed), s.N, s.K, s.RT, s.KS, dev_status);
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_pack(const int8_t *T1, const int8_t *T2, const uint16_t *a1, const uint16_t *a2,
                        int64_t M, int64_t N, int64_t K, int32_t group, void *packed, size_t packed_bytes,
                        int32_t *dev_status, void *stream_)
{
    Shape s;
    ptqtp_status st;
    if (!T1 || !T2 || !a1 || !a2 || !packed) return PTQTP_ERR_NULL;
    if (!make_shape(M, N, K, group, &s, &st)) return st;
    if (packed_bytes < ptqtp_packed_bytes(M, N, K, group)) return PTQTP_ERR_SIZE;
    if (!aligned(packed, 256) || !aligned(T1, 2) || !aligned(T2, 2) || !aligned(a1, 2) || !aligned(a2, 2))
        return PTQTP_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dev_status) hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, stream, dev_status);
    const dim3 grid(static_cast<unsigned>(s.RT * ((s.KS + kPackRecs - 1) / kPackRecs)));
    if (aligned(T1, 16) && aligned(T2, 16))
        hipLaunchKernelGGL(pack_kernel<true>, grid, dim3(256), 0, stream, T1, T2, a1, a2,
                           static_cast<uint8_t *>(packed), s.N, s.K, s.RT, s.KS, s.NG, dev_status);
    else
        hipLaunchKernelGGL(pack_kernel<false>, grid, dim3(256), 0, stream, T1, T2, a1, a2,
                           static_cast<uint8_t *>(packed), s.N, s.K, s.RT, s.KS, s.NG, dev_status);
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_unpack(const void *packed, int64_t M, int64_t N, int64_t K, int32_t group, int8_t *T1,
                          int8_t *T2, uint16_t *a1, uint16_t *a2, void *stream_)
{
    Shape s;
    ptqtp_status st;
    if (!packed) return PTQTP_ERR_NULL;
    if (!make_shape(M, N, K, group, &s, &st)) return st;
    if (!aligned(packed, 256)) return PTQTP_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const uint8_t *blob = static_cast<const uint8_t *>(packed);
    if (T1 || T2) {
        const int64_t blocks = s.RT * ((s.KS + kPackRecs - 1) / kPackRecs);
        if (aligned(T1, 16) && aligned(T2, 16))
            hipLaunchKernelGGL(unpack_trits_kernel<true>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                               blob, T1, T2, s.N, s.K, s.KS);
        else
            hipLaunchKernelGGL(unpack_trits_kernel<false>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                               blob, T1, T2, s.N, s.K, s.KS);
    }
    if (a1 || a2) {
        const int64_t blocks = (s.N * s.NG + 255) / 256;
        hipLaunchKernelGGL(unpack_scales_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, blob, a1,
                           a2, s.N, s.NG, s.KS);
    }
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_gemv(const void *packed, const uint16_t *x, void *y, int32_t y_dtype, int64_t M, int64_t N,
                        int64_t K, int32_t group, void *, size_t, void *stream)
{
    if (M != 1) return PTQTP_ERR_SHAPE;
    return run_forward(packed, x, y, y_dtype, M, N, K, group, stream, 1);
}

ptqtp_status ptqtp_gemm_small(const void *packed, const uint16_t *x, void *y, int32_t y_dtype, int64_t M, int64_t N,
                              int64_t K, int32_t group, void *, size_t, void *stream)
{
    return run_forward(packed, x, y, y_dtype, M, N, K, group, stream, PTQTP_GEMM_SMALL_MAX_M);
}

ptqtp_status ptqtp_gemm(const void *packed, const uint16_t *x, void *y, int32_t y_dtype, int64_t M, int64_t N,
                        int64_t K, int32_t group, void *, size_t, void *stream)
{
    const bool fuse = (y_dtype & PTQTP_FUSED_PLANES) != 0 && M >= 256;
    return run_forward(packed, x, y, y_dtype & ~PTQTP_FUSED_PLANES, M, N, K, group, stream, PTQTP_GEMM_MAX_M, fuse);
}

ptqtp_status ptqtp_gemm_route(int64_t M, int64_t N, int64_t K, int32_t group, int32_t y_dtype, int32_t *route)
{
    Shape s;
    ptqtp_status st;
    if (!route) return PTQTP_ERR_NULL;
    if (!make_shape(M, N, K, group, &s, &st)) return st;
    if (M > PTQTP_GEMM_MAX_M) return PTQTP_ERR_SHAPE;
    if (M == 1) { route[0] = PTQTP_ROUTE_STREAM; route[1] = -1; route[2] = 0; route[3] = -1; return PTQTP_OK; }
    const Route r = choose_route(s, static_cast<int>(M), (y_dtype & PTQTP_FUSED_PLANES) != 0 && M >= 256);
    route[0] = r.path; route[1] = r.kind; route[2] = r.split_row_tile; route[3] = r.second_kind;
    return PTQTP_OK;
}

static ptqtp_status plan_items(const ptqtp_linear *linears, int32_t count, int32_t group, int64_t *total) {
    if (!linears) return PTQTP_ERR_NULL;
    if (count <= 0 || count > PTQTP_BATCH_MAX_LINEARS) return PTQTP_ERR_SHAPE;
    *total = 0;
    for (int i = 0; i < count; ++i) {
        Shape s;
        ptqtp_status st;
        if (!make_shape(1, linears[i].N, linears[i].K, group, &s, &st)) return st;
        *total += (s.RT + kPlanPad - 1) / kPlanPad * kPlanPad;   // every linear starts a new group of kPlanPad items
    }
    return *total > (1ll << 30) ? PTQTP_ERR_SHAPE : PTQTP_OK;
}

size_t ptqtp_batch_plan_bytes(const ptqtp_linear *linears, int32_t count, int32_t group) {
    int64_t total;
    if (plan_items(linears, count, group, &total) != PTQTP_OK) return 0;
    return sizeof(PlanHeader) + static_cast<size_t>(count) * sizeof(LinearDesc) + static_cast<size_t>(total) * 4;
}

ptqtp_status ptqtp_gemv_batch_plan(const ptqtp_linear *linears, int32_t count, int32_t y_dtype, int32_t group,
                                   void *plan, size_t plan_bytes, void *stream_)
{
    int64_t total = 0;
    if (!plan) return PTQTP_ERR_NULL;
    ptqtp_status st = plan_items(linears, count, group, &total);
    if (st != PTQTP_OK) return st;
    if (y_dtype != PTQTP_F32 && y_dtype != PTQTP_F16) return PTQTP_ERR_DTYPE;
    if (plan_bytes < ptqtp_batch_plan_bytes(linears, count, group)) return PTQTP_ERR_SIZE;
    if (!aligned(plan, 256)) return PTQTP_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {
        if (!linears[i].packed || !linears[i].x || !linears[i].y) return PTQTP_ERR_NULL;
        if (!aligned(linears[i].packed, 256) || !aligned(linears[i].x, 16) ||
            !aligned(linears[i].y, y_dtype == PTQTP_F16 ? 2 : 4))
            return PTQTP_ERR_ALIGN;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    // The table lists the linears with the longest rows first (stable otherwise): a workgroup's work grows with K,
    // and the launch ends sooner when the items handed out last are the short ones.
    std::vector<int> order(count);
    for (int i = 0; i < count; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return linears[a].K > linears[b].K; });
    int64_t first = 0;
    for (int base = 0; base < count; base += kPlanChunk) {
        DescChunk chunk = {};
        const int n = count - base < kPlanChunk ? count - base : kPlanChunk;
        for (int i = 0; i < n; ++i) {
            const ptqtp_linear &lin = linears[order[base + i]];
            Shape s;
            make_shape(1, lin.N, lin.K, group, &s, &st);
            LinearDesc &d = chunk.d[i];
            d.records = static_cast<const uint8_t *>(lin.packed) + kHeaderBytes;
            d.x = lin.x; d.y = lin.y;
            d.N = static_cast<int32_t>(s.N); d.K = static_cast<int32_t>(s.K);
            d.RT = static_cast<int32_t>(s.RT); d.KS = static_cast<int32_t>(s.KS);
            d.first_item = static_cast<int32_t>(first); d.pad = 0;
            first += (s.RT + kPlanPad - 1) / kPlanPad * kPlanPad;
        }
        hipLaunchKernelGGL(plan_write_kernel, dim3(1), dim3(64), 0, stream, static_cast<PlanHeader *>(plan), chunk,
                           base, n, count, static_cast<int>(total), y_dtype == PTQTP_F16 ? 1 : 0);
    }
    const unsigned blocks = static_cast<unsigned>(total + 255) / 256;
    hipLaunchKernelGGL(plan_map_kernel, dim3(blocks > 1024 ? 1024 : blocks), dim3(256), 0, stream,
                       static_cast<PlanHeader *>(plan));
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

int64_t ptqtp_batch_items(const ptqtp_linear *linears, int32_t count, int32_t group) {
    int64_t total;
    return plan_items(linears, count, group, &total) == PTQTP_OK ? total : 0;
}

ptqtp_status ptqtp_gemv_batch(const void *plan, int64_t items, void *stream_) {
    if (!plan) return PTQTP_ERR_NULL;
    if (!aligned(plan, 256)) return PTQTP_ERR_ALIGN;
    if (items <= 0 || items > (1ll << 30)) return PTQTP_ERR_SHAPE;
    LinearDesc none = {};
    const hipError_t e = launch_items<true>(static_cast<const PlanHeader *>(plan), none, 0, items, 16,
                                            static_cast<hipStream_t>(stream_));
    return e == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

static ptqtp_status run_gemm_batch(const void *plan, int64_t items, int64_t M, void *stream_, bool fuse_planes) {
    if (!plan) return PTQTP_ERR_NULL;
    if (!aligned(plan, 256)) return PTQTP_ERR_ALIGN;
    if (items <= 0 || items > (1ll << 30) || M < 1 || M > PTQTP_GEMM_SMALL_MAX_M) return PTQTP_ERR_SHAPE;
    if (M == 1) return ptqtp_gemv_batch(plan, items, stream_);
    const PlanHeader *ph = static_cast<const PlanHeader *>(plan);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int Mi = static_cast<int>(M);
    hipError_t e;
    if (g_tune_small_rows_kernel == 0) e = launch_gemm_items_plan(ph, items, Mi, stream);
    else {
        // 16 row tiles per workgroup share one activation tile.  Measured on the 8B stack: as four waves x four
        // row tiles up to 16 tokens (M = 16: 727 us with 8 per workgroup -> 677 us), as eight waves x two above
        // (M = 32: 950 -> 925 us, M = 64: 1665 us with 8 per workgroup -> 1536 us as 4 x 4 -> 1450 us as 8 x 2).
        // `rows`: 1, 2, 4 = row tiles per wave of a four-wave workgroup; 8 = two per wave, eight waves.
        const int rows = g_tune_small_rows ? g_tune_small_rows : (M <= 16 ? 4 : 8);
        const bool fold = g_tune_small_fold < 0 ? M > 32 : g_tune_small_fold != 0;   // measured on the 8B stack
        if (fuse_planes && M > 32) {
            // the weight rebuilt in fp16 per 32-column field, one MFMA pass instead of one per plane (8B stack,
            // 64 tokens: 1433 -> 1131 us; 48: 1198 -> 993 us); up to 32 tokens the matrix pipe is not what binds
            e = M <= 48 ? launch_gemm_rows<3, 2, true, 8, true>(ph, items, Mi, stream)
                        : launch_gemm_rows<4, 2, true, 8, true>(ph, items, Mi, stream);
        }
        else if (rows == 8) {
            if (M <= 16) e = launch_gemm_rows<1, 2, false, 8>(ph, items, Mi, stream);
            else if (M <= 32) e = fold ? launch_gemm_rows<2, 2, true, 8>(ph, items, Mi, stream)
                                       : launch_gemm_rows<2, 2, false, 8>(ph, items, Mi, stream);
            else if (M <= 48) e = launch_gemm_rows<3, 2, true, 8>(ph, items, Mi, stream);
            else e = launch_gemm_rows<4, 2, true, 8>(ph, items, Mi, stream);
        }
        else if (M <= 16 && rows == 4) e = launch_gemm_rows<1, 4, false>(ph, items, Mi, stream);
        else if (M <= 32 && rows == 4) e = fold ? launch_gemm_rows<2, 4, true>(ph, items, Mi, stream)
                                                : launch_gemm_rows<2, 4, false>(ph, items, Mi, stream);
        else if (M <= 48 && rows == 4) e = launch_gemm_rows<3, 4, true>(ph, items, Mi, stream);
        else if (rows == 4) e = launch_gemm_rows<4, 4, true>(ph, items, Mi, stream);
        else if (M <= 16) e = rows == 1 ? launch_gemm_rows<1, 1, false>(ph, items, Mi, stream)
                       : fold ? launch_gemm_rows<1, 2, true>(ph, items, Mi, stream)
                              : launch_gemm_rows<1, 2, false>(ph, items, Mi, stream);
        else if (M <= 32) e = rows == 1 ? launch_gemm_rows<2, 1, false>(ph, items, Mi, stream)
                            : fold ? launch_gemm_rows<2, 2, true>(ph, items, Mi, stream)
                                   : launch_gemm_rows<2, 2, false>(ph, items, Mi, stream);
        else if (M <= 48) e = rows == 1 ? launch_gemm_rows<3, 1, false>(ph, items, Mi, stream)
                            : fold ? launch_gemm_rows<3, 2, true>(ph, items, Mi, stream)
                                   : launch_gemm_rows<3, 2, false>(ph, items, Mi, stream);
        else e = rows == 1 ? launch_gemm_rows<4, 1, false>(ph, items, Mi, stream)
                 : fold ? launch_gemm_rows<4, 2, true>(ph, items, Mi, stream)
                        : launch_gemm_rows<4, 2, false>(ph, items, Mi, stream);
    }
    return e == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_gemm_batch(const void *plan, int64_t items, int64_t M, void *stream) {
    return run_gemm_batch(plan, items, M, stream, false);
}

ptqtp_status ptqtp_gemm_batch_fused(const void *plan, int64_t items, int64_t M, void *stream) {
    return run_gemm_batch(plan, items, M, stream, true);
}

ptqtp_status ptqtp_tune(const char *key, int32_t value) {
    if (!key) return PTQTP_ERR_NULL;
    if (!strcmp(key, "chain_waves")) {
        if (value < 0 || value > 16 || (value & 1)) return PTQTP_ERR_SHAPE;
        ptqtp_detail::g_chain_waves = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "chain_depth")) {
        if (value != 0 && value != 1 && value != 2 && value != 4) return PTQTP_ERR_SHAPE;
        ptqtp_detail::g_chain_depth = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "chain_table")) {
        if (value < 0 || value > 1) return PTQTP_ERR_SHAPE;
        ptqtp_detail::g_chain_table = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "small_ahead")) {
        if (value < -1 || value > 1) return PTQTP_ERR_SHAPE;
        g_tune_small_ahead = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "small_fold")) {
        if (value < -1 || value > 1) return PTQTP_ERR_SHAPE;
        g_tune_small_fold = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "stream_waves")) {
        if (value < 0 || value > 16) return PTQTP_ERR_SHAPE;
        g_tune_stream_waves = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "tile_variant")) {
        if (value < 0 || value > 5) return PTQTP_ERR_SHAPE;
        g_tune_tile_variant = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "tile")) {
        if (value < -1 || value > 1) return PTQTP_ERR_SHAPE;
        g_tune_tile = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "batch_rows_kernel")) {
        if (value < -1 || value > 1) return PTQTP_ERR_SHAPE;
        g_tune_small_rows_kernel = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "small_rows")) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return PTQTP_ERR_SHAPE;
        g_tune_small_rows = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "small_waves")) {
        if (value < 0 || value > 8) return PTQTP_ERR_SHAPE;
        g_tune_small_waves = value;
        return PTQTP_OK;
    }
    if (!strcmp(key, "stream_depth")) {
        if (value != 0 && value != 1 && value != 2 && value != 4) return PTQTP_ERR_SHAPE;
        g_tune_stream_depth = value;
        return PTQTP_OK;
    }
    return PTQTP_ERR_SHAPE;
}

}  // extern "C"
