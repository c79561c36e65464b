// libptqtp: decode chain -- dependent batch-1 linears with fused epilogues (gated-MLP product,
// residual add, fp16 activations), one launch per level of the chain.
//
// Work item = one 16-row tile of a stage (for a gated-MLP stage: the pair of tiles that holds
// gate rows i..i+15 and up rows i..i+15) over the stage's whole K, handled by one workgroup
// exactly like the batch-1 item kernel: its waves split the item's 256-column steps, stream
// their records with non-temporal loads, expand the 2-bit codes to fp16 and add in the matrix
// pipe; partial sums meet in LDS in a fixed order and lanes 0..15 of wave 0 apply the epilogue.
// Items are numbered level by level; a level with few items gets more waves per item so that
// every record of the level is requested in one round trip.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

#include "ptqtp.h"
#include "ptqtp_device.hpp"

namespace ptqtp_detail {
int g_chain_waves = 0, g_chain_depth = 0;      // ptqtp_tune("chain_waves" / "chain_depth"): 0 = heuristic
int g_chain_table = 0;                         // ptqtp_tune("chain_table"): 1 = every level finds its stages through the plan table
// ptqtp.hip: the small-batch item kernel with a stage's epilogue in its final reduction
hipError_t small_batch_stage(const uint8_t *records, const uint16_t *x, void *y, const uint16_t *residual, int M,
                             int64_t N, int64_t K, int y_f16, int gated, hipStream_t stream);
// ptqtp.hip: one MFMA tile launch with the epilogue in its store (more than 64 tokens)
hipError_t tile_stage(const uint8_t *records, const uint16_t *x, void *y, const uint16_t *residual, int M,
                      int64_t N, int64_t K, int y_f16, int gated, bool fuse_planes, hipStream_t stream);
}

namespace {

constexpr int kChainMaxWaves = 16;
constexpr uint64_t kChainMagic = 0x314e484350545150ull;  // "PQTPCHN1"

struct StageDesc {              // 72 bytes
    const uint8_t *records;     // blob + header
    const uint16_t *x;          // fp16 [K]
    void *y;                    // [N] or [N/2]
    const uint16_t *residual;   // fp16 or null
    int32_t N, K, RT, KS;
    int32_t first_item, items;  // items = RT, or RT/2 for a gated-MLP stage
    int32_t epilogue, y_f16;
    int32_t level, pad;         // dense level index
};
static_assert(sizeof(StageDesc) == 72, "StageDesc layout");

struct ChainHeader {            // 256 bytes; then StageDesc[count], int32 item_stage[total_items]
    uint64_t magic;
    int32_t count, total_items, levels, pad;
    int32_t reserved[58];
};
static_assert(sizeof(ChainHeader) == 256, "ChainHeader layout");

constexpr int kChainChunk = 32;
struct StageChunk { StageDesc d[kChainChunk]; };

__device__ __forceinline__ const StageDesc *chain_table(const ChainHeader *h) {
    return reinterpret_cast<const StageDesc *>(h + 1);
}

__global__ void chain_write_kernel(ChainHeader *plan, StageChunk chunk, int base, int n, int count, int total_items,
                                   int levels)
{
    const int t = threadIdx.x;
    if (base == 0 && t == 0) {
        ChainHeader h = {};
        h.magic = kChainMagic; h.count = count; h.total_items = total_items; h.levels = levels;
        *plan = h;
    }
    if (t < n) reinterpret_cast<StageDesc *>(plan + 1)[base + t] = chunk.d[t];
}

// item -> stage index, by bisection over first_item (one-time, after chain_write_kernel)
__global__ void __launch_bounds__(256) chain_map_kernel(ChainHeader *plan)
{
    const int count = plan->count, total = plan->total_items;
    const StageDesc *table = chain_table(plan);
    int32_t *map = const_cast<int32_t *>(reinterpret_cast<const int32_t *>(table + count));
    for (int item = blockIdx.x * 256 + threadIdx.x; item < total; item += gridDim.x * 256) {
        int lo = 0, hi = count - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (table[mid].first_item <= item) lo = mid; else hi = mid - 1;
        }
        map[item] = lo;
    }
}

// One work item: S = records a wave requests at once; the workgroup has blockDim.x / 64 <= 16 waves (an even
// number, so that a gated-MLP item gives each of its two row tiles half of them).  Every argument is uniform over
// the workgroup (it comes from kernel arguments or from the plan table through scalar loads).
template <int S>
__device__ __forceinline__ void chain_item(const uint8_t *records, const uint16_t *x, void *y, const uint16_t *residual,
                                           int N, int K, int KS, int RT, int it, bool pair, int y_f16,
                                           float (*red)[16], uintx2 (*xs)[64])
{
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int W = blockDim.x >> 6;
    const int nl = lane & 15, q = lane >> 4;
    const int Wh = pair ? W / 2 : W;                    // waves that share one row tile
    const int half = w / Wh, part = w - half * Wh;
    const int rt = it + (half ? RT / 2 : 0);
    const uint8_t *rec0 = records + static_cast<size_t>(rt) * KS * kRecordBytes;
    const int rot = (it * 5) % KS;

    uintx4 xa[1][8];
#pragma unroll
    for (int f = 0; f < 8; ++f) xa[0][f] = uintx4{0, 0, 0, 0};   // lanes of tokens 1..15 stay zero
    const char *xs_rd = reinterpret_cast<const char *>(&xs[w][0]) + q * 16;
    float yacc = 0.f;

    for (int ks0 = part; ks0 < KS; ks0 += S * Wh) {
        uintx4 p1[S], p2[S];
        uintx2 sc[S], xr[S];
        // issue: S steps in flight.  Steps past the end re-read the batch's first step (address
        // stays valid, result unused) so that the number of outstanding loads is static.
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const int ks = ks0 + i * Wh;
            int kse = (ks < KS ? ks : ks0) + rot;       // rotated start: neighbours hit different x lines
            kse = kse >= KS ? kse - KS : kse;
            const uint8_t *rec = rec0 + static_cast<size_t>(kse) * kRecordBytes;
            p1[i] = load_stream<uintx4>(rec + lane * 16);
            p2[i] = load_stream<uintx4>(rec + kPlaneBytes + lane * 16);
            sc[i] = load_stream<uintx2>(rec + 2 * kPlaneBytes + nl * 8);
            int k = kse * kStepK + lane * 4;
            k = k < K ? k : 0;                          // odd number of groups: tail lanes
            xr[i] = load_global<uintx2>(x + k);
        }
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const int ks = ks0 + i * Wh;
            if (ks < KS) {
                uintx2 xv = xr[i];
                int kr = ks + rot;
                kr = kr >= KS ? kr - KS : kr;
                if (kr * kStepK + lane * 4 >= K) xv = uintx2{0, 0};
                xs[w][lane] = xv;                                // wave-private bounce: no barrier
                if (nl == 0) {
#pragma unroll
                    for (int f = 0; f < 8; ++f)
                        xa[0][f] = *reinterpret_cast<const uintx4 *>(xs_rd + (f >> 2) * 256 + (f & 3) * 64);
                }
                const float a1g0 = half_bits_to_float(sc[i].x & 0xffffu), a1g1 = half_bits_to_float(sc[i].x >> 16);
                const float a2g0 = half_bits_to_float(sc[i].y & 0xffffu), a2g1 = half_bits_to_float(sc[i].y >> 16);
                floatx4 acc[1];
                group_sum<1, 0>(xa, p1[i], acc); yacc = fmaf(a1g0, acc[0][0], yacc);
                group_sum<1, 1>(xa, p1[i], acc); yacc = fmaf(a1g1, acc[0][0], yacc);
                group_sum<1, 0>(xa, p2[i], acc); yacc = fmaf(a2g0, acc[0][0], yacc);
                group_sum<1, 1>(xa, p2[i], acc); yacc = fmaf(a2g1, acc[0][0], yacc);
            }
        }
    }

    if (q == 0) red[w][nl] = yacc;
    __syncthreads();
    if (w == 0) {
        // lanes 0..15: one output each (fixed summation order); fp16 outputs leave as 32-bit pairs
        float out = 0.f;
        const int n_out = pair ? N / 2 : N;
        const int n = it * kTileRows + nl;
        if (lane < 16) {
            float lo = 0.f, hi = 0.f;                    // sums over the first and the second half of the waves
            for (int ww = 0; ww < W / 2; ++ww) { lo += red[ww][nl]; hi += red[W / 2 + ww][nl]; }
            if (pair) out = (lo / (1.0f + __expf(-lo))) * hi;     // silu(gate) * up
            else out = lo + hi;
            if (residual != nullptr && n < n_out) out += half_bits_to_float(load_global<uint16_t>(residual + n));
        }
        if (y_f16) {
            const uint32_t hb = __builtin_bit_cast(uint16_t, static_cast<_Float16>(out));
            const uint32_t nb = __shfl_down(hb, 1);                 // the odd neighbour's half
            if (lane < 16 && (lane & 1) == 0 && n < n_out) {
                uint16_t *yp = reinterpret_cast<uint16_t *>(y) + n;
                if (n + 1 < n_out) *reinterpret_cast<uint32_t *>(yp) = hb | (nb << 16);
                else *yp = static_cast<uint16_t>(hb);             // last element of an odd-length output
            }
        } else if (lane < 16 && n < n_out) {
            reinterpret_cast<float *>(y)[n] = out;
        }
    }
}

// A level of up to kLevelStages stages: the stage descriptors travel as kernel arguments, so a workgroup knows its
// records' address without a single load from memory (a level's launch is short: two or three dependent loads from
// a device-side table before the first record request were a third of it).  The grid is exactly the level's items;
// first_item counts from the launch's first item.
constexpr int kLevelStages = 4;
struct LevelArgs { StageDesc d[kLevelStages]; };

template <int S, bool MULTI>
__global__ void __launch_bounds__(kChainMaxWaves * 64)
chain_level_kernel(const LevelArgs args, int n_stages)
{
    __shared__ float red[kChainMaxWaves][16];
    __shared__ uintx2 xs[kChainMaxWaves][64];
    const int item = static_cast<int>(blockIdx.x);
    int idx = 0;
    if (MULTI) {
#pragma unroll
        for (int i = 1; i < kLevelStages; ++i)
            if (i < n_stages && item >= args.d[i].first_item) idx = i;
    }
    const StageDesc &sd = args.d[idx];
    chain_item<S>(sd.records, sd.x, sd.y, sd.residual, sd.N, sd.K, sd.KS, sd.RT, item - sd.first_item,
                  sd.epilogue == PTQTP_EPI_SWIGLU, sd.y_f16, red, xs);
}

// The same items found through the device-side plan (item -> stage map): for levels of more than kLevelStages stages.
template <int S>
__global__ void __launch_bounds__(kChainMaxWaves * 64)
chain_items_kernel(const ChainHeader *__restrict__ plan, int item_base)
{
    __shared__ float red[kChainMaxWaves][16];
    __shared__ uintx2 xs[kChainMaxWaves][64];
    const int item = item_base + static_cast<int>(blockIdx.x);     // the grid is exactly the level's items
    const StageDesc *table = chain_table(plan);
    const int32_t *map = reinterpret_cast<const int32_t *>(table + plan->count);
    const StageDesc *sd = table + map[item];
    chain_item<S>(sd->records, sd->x, sd->y, sd->residual, sd->N, sd->K, sd->KS, sd->RT, item - sd->first_item,
                  sd->epilogue == PTQTP_EPI_SWIGLU, sd->y_f16, red, xs);
}

// first_stage / stages: the level's slice of the stage array; min_steps / max_steps: fewest and most 256-column steps
// of a stage of the level; gated: it has a gated stage
struct LevelRange { int first_item, items, min_steps, max_steps, gated, first_stage, stages; };

// host-side geometry of a chain; returns false (and a status) on invalid input
bool chain_geometry(const ptqtp_stage *stages, int32_t count, int32_t group, StageDesc *descs /* count or null */,
                    LevelRange *levels /* count or null */, int *n_levels, int64_t *total_items, ptqtp_status *st)
{
    *st = PTQTP_OK;
    if (!stages) { *st = PTQTP_ERR_NULL; return false; }
    if (count <= 0 || count > PTQTP_CHAIN_MAX_STAGES) { *st = PTQTP_ERR_SHAPE; return false; }
    if (group != 128) { *st = PTQTP_ERR_GROUP; return false; }
    int64_t item = 0;
    int lv = -1, prev_level = -1, cur_level_items = 0;
    for (int i = 0; i < count; ++i) {
        const ptqtp_stage &s = stages[i];
        if (!s.packed || !s.x || !s.y) { *st = PTQTP_ERR_NULL; return false; }
        if (s.N <= 0 || s.K <= 0 || s.K % group != 0 || s.N > (1ll << 30) || s.K > (1ll << 30)) { *st = PTQTP_ERR_SHAPE; return false; }
        if (s.epilogue != PTQTP_EPI_NONE && s.epilogue != PTQTP_EPI_SWIGLU) { *st = PTQTP_ERR_SHAPE; return false; }
        if (s.epilogue == PTQTP_EPI_SWIGLU && s.N % 32 != 0) { *st = PTQTP_ERR_SHAPE; return false; }
        const int32_t ydt = s.y_dtype & ~PTQTP_FUSED_PLANES;      // the flag only counts in ptqtp_chain_run_batch
        if (ydt != PTQTP_F32 && ydt != PTQTP_F16) { *st = PTQTP_ERR_DTYPE; return false; }
        if (s.level < 0 || s.level < prev_level || s.reserved != 0) { *st = PTQTP_ERR_SHAPE; return false; }
        if ((reinterpret_cast<uintptr_t>(s.packed) & 255) || (reinterpret_cast<uintptr_t>(s.x) & 15) ||
            (reinterpret_cast<uintptr_t>(s.y) & 15) || (reinterpret_cast<uintptr_t>(s.residual) & 15)) {
            *st = PTQTP_ERR_ALIGN; return false;
        }
        if (s.level != prev_level) {
            if (lv >= 0 && levels) levels[lv].items = cur_level_items;
            ++lv;
            cur_level_items = 0;
            if (levels) {
                levels[lv].first_item = static_cast<int>(item); levels[lv].min_steps = 1 << 30; levels[lv].max_steps = 0;
                levels[lv].gated = 0; levels[lv].first_stage = i; levels[lv].stages = 0;
            }
            prev_level = s.level;
        }
        const int64_t RT = (s.N + kTileRows - 1) / kTileRows;
        const int64_t KS = (s.K + kStepK - 1) / kStepK;
        const int64_t items = s.epilogue == PTQTP_EPI_SWIGLU ? RT / 2 : RT;
        if (descs) {
            StageDesc d = {};
            d.records = static_cast<const uint8_t *>(s.packed) + kHeaderBytes;
            d.x = s.x; d.y = s.y; d.residual = s.residual;
            d.N = static_cast<int32_t>(s.N); d.K = static_cast<int32_t>(s.K);
            d.RT = static_cast<int32_t>(RT); d.KS = static_cast<int32_t>(KS);
            d.first_item = static_cast<int32_t>(item); d.items = static_cast<int32_t>(items);
            d.epilogue = s.epilogue; d.y_f16 = ydt == PTQTP_F16;
            d.level = lv;
            descs[i] = d;
        }
        if (levels && KS < levels[lv].min_steps) levels[lv].min_steps = static_cast<int>(KS);
        if (levels && KS > levels[lv].max_steps) levels[lv].max_steps = static_cast<int>(KS);
        if (levels) ++levels[lv].stages;
        if (levels && s.epilogue == PTQTP_EPI_SWIGLU) levels[lv].gated = 1;
        item += items;
        cur_level_items += static_cast<int>(items);
        if (item > (1ll << 30)) { *st = PTQTP_ERR_SHAPE; return false; }
    }
    if (levels) levels[lv].items = cur_level_items;
    *n_levels = lv + 1;
    *total_items = item;
    return true;
}

// launch shape of a level: W waves per item, S records in flight per wave
void level_shape(const LevelRange &lr, int *W_, int *S_) {
    // thousands of items: 4 waves x 2 records each keep the stream full.  Few items: more waves per
    // item and one record each put the whole level in flight in one round trip.
    int W = 4, S = 2;
    if (lr.items < 2048) {
        S = 1;
        while (W < kChainMaxWaves && lr.items * W * 2 <= 4096) W *= 2;
        if (lr.gated) {
            // a gated item gives each of its two row tiles half of the waves: double them, and let a wave that still
            // has four or more steps request two at a time (measured on the 8B gate|up stage: 16.3 -> 14.4 us)
            if (W < kChainMaxWaves) W *= 2;
            if ((lr.min_steps + W / 2 - 1) / (W / 2) >= 4) S = 2;
        }
        while (W > 2 && W / 2 > lr.min_steps) W /= 2;
    }
    if (ptqtp_detail::g_chain_waves > 0) W = ptqtp_detail::g_chain_waves;
    if (ptqtp_detail::g_chain_depth > 0) S = ptqtp_detail::g_chain_depth;
    *W_ = W; *S_ = S >= 4 ? 4 : S == 2 ? 2 : 1;
}

template <bool MULTI>
void launch_level(const LevelArgs &args, int n, int items, int W, int S, hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>(items)), block(W * 64);
    if (S == 4) hipLaunchKernelGGL((chain_level_kernel<4, MULTI>), grid, block, 0, stream, args, n);
    else if (S == 2) hipLaunchKernelGGL((chain_level_kernel<2, MULTI>), grid, block, 0, stream, args, n);
    else hipLaunchKernelGGL((chain_level_kernel<1, MULTI>), grid, block, 0, stream, args, n);
}

}  // namespace

extern "C" {

size_t ptqtp_chain_plan_bytes(const ptqtp_stage *stages, int32_t count, int32_t group) {
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, nullptr, nullptr, &n_levels, &total, &st)) return 0;
    const size_t bytes = sizeof(ChainHeader) + static_cast<size_t>(count) * sizeof(StageDesc) + static_cast<size_t>(total) * 4;
    return (bytes + 255) & ~static_cast<size_t>(255);
}

ptqtp_status ptqtp_chain_plan(const ptqtp_stage *stages, int32_t count, int32_t group,
                              void *plan, size_t plan_bytes, void *stream_) {
    if (!plan) return PTQTP_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(plan) & 255) return PTQTP_ERR_ALIGN;
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, nullptr, nullptr, &n_levels, &total, &st)) return st;
    std::vector<StageDesc> descs(static_cast<size_t>(count));       // host memory only
    chain_geometry(stages, count, group, descs.data(), nullptr, &n_levels, &total, &st);
    if (plan_bytes < ptqtp_chain_plan_bytes(stages, count, group)) return PTQTP_ERR_SIZE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ChainHeader *ph = static_cast<ChainHeader *>(plan);
    for (int base = 0; base < count; base += kChainChunk) {
        StageChunk chunk;
        const int n = count - base < kChainChunk ? count - base : kChainChunk;
        for (int i = 0; i < n; ++i) chunk.d[i] = descs[base + i];
        hipLaunchKernelGGL(chain_write_kernel, dim3(1), dim3(64), 0, stream, ph, chunk, base, n, count,
                           static_cast<int>(total), n_levels);
    }
    const int blocks = static_cast<int>((total + 255) / 256) < 1024 ? static_cast<int>((total + 255) / 256) : 1024;
    hipLaunchKernelGGL(chain_map_kernel, dim3(blocks), dim3(256), 0, stream, ph);
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_chain_run(const ptqtp_stage *stages, int32_t count, int32_t group, const void *plan, void *stream_) {
    if (!plan) return PTQTP_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(plan) & 255) return PTQTP_ERR_ALIGN;
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, nullptr, nullptr, &n_levels, &total, &st)) return st;
    std::vector<StageDesc> descs(static_cast<size_t>(count));       // host memory only
    std::vector<LevelRange> lr(static_cast<size_t>(count));
    chain_geometry(stages, count, group, descs.data(), lr.data(), &n_levels, &total, &st);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const ChainHeader *ph = static_cast<const ChainHeader *>(plan);
    for (int l = 0; l < n_levels; ++l) {
        int W, S;
        level_shape(lr[l], &W, &S);
        if (lr[l].stages <= kLevelStages && ptqtp_detail::g_chain_table <= 0) {
            // the usual case: the level's descriptors fit the kernel arguments
            LevelArgs args = {};
            for (int i = 0; i < lr[l].stages; ++i) {
                args.d[i] = descs[static_cast<size_t>(lr[l].first_stage + i)];
                args.d[i].first_item -= lr[l].first_item;
            }
            if (lr[l].stages == 1) launch_level<false>(args, 1, lr[l].items, W, S, stream);
            else launch_level<true>(args, lr[l].stages, lr[l].items, W, S, stream);
        } else {
            // a wide level: items find their stage through the device-side plan
            const dim3 grid(static_cast<unsigned>(lr[l].items)), block(W * 64);
            if (S == 4) hipLaunchKernelGGL((chain_items_kernel<4>), grid, block, 0, stream, ph, lr[l].first_item);
            else if (S == 2) hipLaunchKernelGGL((chain_items_kernel<2>), grid, block, 0, stream, ph, lr[l].first_item);
            else hipLaunchKernelGGL((chain_items_kernel<1>), grid, block, 0, stream, ph, lr[l].first_item);
        }
    }
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_chain_run_batch(const ptqtp_stage *stages, int32_t count, int32_t group, int64_t M, void *stream_) {
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, nullptr, nullptr, &n_levels, &total, &st)) return st;
    if (M < 1 || M > PTQTP_GEMM_MAX_M) return PTQTP_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    for (int i = 0; i < count; ++i) {
        const ptqtp_stage &s = stages[i];
        // up to 64 tokens: the small-batch kernel; above: one MFMA tile launch with the epilogue in its store
        const uint8_t *records = static_cast<const uint8_t *>(s.packed) + kHeaderBytes;
        const int f16 = (s.y_dtype & ~PTQTP_FUSED_PLANES) == PTQTP_F16, gated = s.epilogue == PTQTP_EPI_SWIGLU;
        const bool fuse = (s.y_dtype & PTQTP_FUSED_PLANES) != 0 && M >= 256;
        const hipError_t e =
            M <= PTQTP_GEMM_SMALL_MAX_M
                ? ptqtp_detail::small_batch_stage(records, s.x, s.y, s.residual, static_cast<int>(M), s.N, s.K, f16, gated, stream)
                : ptqtp_detail::tile_stage(records, s.x, s.y, s.residual, static_cast<int>(M), s.N, s.K, f16, gated, fuse, stream);
        if (e != hipSuccess) return PTQTP_ERR_HIP;
    }
    return PTQTP_OK;
}

}  // extern "C"
