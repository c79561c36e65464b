// libptqtp: decode chain -- dependent batch-1 linears with fused epilogues (gated-MLP product,
// residual add, fp16 activations), run as one launch per level or as ONE persistent launch whose
// workgroups order themselves with device-side completion counters.
//
// Work item = one 16-row tile of a stage (for a gated-MLP stage: the pair of tiles that holds
// gate rows i..i+15 and up rows i..i+15) over the stage's whole K, handled by one workgroup of
// four waves exactly like the batch-1 item kernel: the waves split the item's 256-column steps,
// stream their records with non-temporal loads, expand the 2-bit codes to fp16 and add in the
// matrix pipe; partial sums meet in LDS in a fixed order.  Items are numbered level by level.
//
// Persistent mode.  A workgroup draws its item number from a device counter when it starts, so
// item numbers follow the order in which workgroups actually began to run: the unfinished item
// with the smallest number is always held by a running workgroup whose inputs are complete, and
// waiting on items with smaller numbers can never deadlock, whatever the dispatch order.  The
// workgroup issues the loads of its first records (weights do not depend on activations), then
// polls the completion counter of the previous level, then reads x.  Waits are bounded
// (spin_limit polls); a wait that runs out, or a status word already set by another workgroup,
// ends the wait: the workgroup finishes normally with whatever x holds and the status word
// says the run is invalid.  Activations cross XCDs, whose L2s do not snoop each other:
//   sync 0: the producer's stores are followed by an agent-scope release fence (L2 write-back)
//           before its counter increment, the consumer's poll by an agent-scope acquire fence
//           (L2 invalidate) -- the textbook pattern;
//   sync 1: activations are written with agent-scope (write-through) stores and read with
//           agent-scope (L2-bypassing) loads, ordered against the counter by waiting for the
//           stores' acknowledgement; no cache-wide operation.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ptqtp.h"
#include "ptqtp_device.hpp"

namespace ptqtp_detail {
int g_chain_spin_limit = 0;   // 0 = default
int g_chain_sync = -1;        // -1 = default
}

namespace {

constexpr int kChainWaves = 4;
constexpr int kChainDepth = 2;                       // records in flight per wave
constexpr int kDefaultSpinLimit = 1 << 18;           // polls of ~1 us each
constexpr uint64_t kChainMagic = 0x314e484350545150ull;  // "PQTPCHN1"

struct StageDesc {              // 72 bytes
    const uint8_t *records;     // blob + header
    const uint16_t *x;          // fp16 [K]
    void *y;                    // [N] or [N/2]
    const uint16_t *residual;   // fp16 or null
    int32_t N, K, RT, KS;
    int32_t first_item, items;  // items = RT, or RT/2 for a gated-MLP stage
    int32_t epilogue, y_f16;
    int32_t level, wait_count;  // dense level index; items of the previous level (0 for level 0)
};
static_assert(sizeof(StageDesc) == 72, "StageDesc layout");

struct ChainHeader {            // 256 bytes; then int32 done[levels_padded], StageDesc[count], int32 item_stage[total_items]
    uint64_t magic;
    int32_t count, total_items, levels, levels_padded;
    int32_t next_item;          // persistent mode: next item number to hand out
    int32_t status;             // PTQTP_OK or PTQTP_ERR_WAIT
    int32_t reserved[56];
};
static_assert(sizeof(ChainHeader) == 256, "ChainHeader layout");

constexpr int kChainChunk = 32;
struct StageChunk { StageDesc d[kChainChunk]; };

__device__ __forceinline__ int32_t *chain_done(ChainHeader *h) { return reinterpret_cast<int32_t *>(h + 1); }
__device__ __forceinline__ const StageDesc *chain_table(const ChainHeader *h) {
    return reinterpret_cast<const StageDesc *>(reinterpret_cast<const int32_t *>(h + 1) + h->levels_padded);
}

__global__ void chain_write_kernel(ChainHeader *plan, StageChunk chunk, int base, int n, int count, int total_items,
                                   int levels, int levels_padded)
{
    const int t = threadIdx.x;
    if (base == 0 && t == 0) {
        ChainHeader h = {};
        h.magic = kChainMagic; h.count = count; h.total_items = total_items;
        h.levels = levels; h.levels_padded = levels_padded;
        *plan = h;
    }
    if (base == 0) {
        for (int i = t; i < levels_padded; i += blockDim.x) reinterpret_cast<int32_t *>(plan + 1)[i] = 0;
    }
    if (t < n) {
        StageDesc *table = reinterpret_cast<StageDesc *>(reinterpret_cast<int32_t *>(plan + 1) + levels_padded);
        table[base + t] = chunk.d[t];
    }
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

// start of a persistent run: counters and status back to zero (a kernel, not a memset, so that a
// captured run replays correctly)
__global__ void chain_reset_kernel(ChainHeader *plan)
{
    int32_t *done = chain_done(plan);
    for (int i = threadIdx.x; i < plan->levels_padded; i += blockDim.x) done[i] = 0;
    if (threadIdx.x == 0) { plan->next_item = 0; plan->status = PTQTP_OK; }
}

typedef const __attribute__((address_space(1))) uint64_t *gptr64;
typedef __attribute__((address_space(1))) uint32_t *gptr32w;

// 8 bytes of activations.  COHERENT: an agent-scope load, served from the level of the memory
// hierarchy all XCDs share.
template <bool COHERENT>
__device__ __forceinline__ uintx2 load_x8(const uint16_t *p) {
    if constexpr (COHERENT) {
        const uint64_t v = __hip_atomic_load((gptr64)(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return uintx2{static_cast<uint32_t>(v), static_cast<uint32_t>(v >> 32)};
    } else {
        return load_global<uintx2>(p);
    }
}

// PERSIST: dynamic item numbers + bounded waits on the previous level.  SYNC (persistent only): 0 = fences, 1 = coherent accesses.
template <bool PERSIST, int SYNC>
__global__ void __launch_bounds__(kChainWaves * 64) __attribute__((amdgpu_waves_per_eu(4)))
chain_items_kernel(ChainHeader *__restrict__ plan, int item_base, int item_count, int spin_limit)
{
    constexpr int S = kChainDepth, W = kChainWaves;
    constexpr bool COH = PERSIST && SYNC == 1;
    __shared__ float red[W][16];
    __shared__ uintx2 xs[W][64];
    __shared__ int s_item;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nl = lane & 15, q = lane >> 4;

    int item;
    if constexpr (PERSIST) {
        if (threadIdx.x == 0)
            s_item = __hip_atomic_fetch_add(&plan->next_item, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        item = s_item;
    } else {
        item = item_base + static_cast<int>(blockIdx.x);
    }
    if (item >= item_base + item_count) return;         // whole workgroup leaves: no later barrier is skipped

    const StageDesc *table = chain_table(plan);
    const int32_t *map = reinterpret_cast<const int32_t *>(table + plan->count);
    const StageDesc *sd = table + map[item];
    const int K = sd->K, KS = sd->KS, N = sd->N;
    const bool pair = sd->epilogue == PTQTP_EPI_SWIGLU;
    const int Wh = pair ? W / 2 : W;                    // waves that share one row tile
    const int half = w / Wh, part = w - half * Wh;
    const int it = item - sd->first_item;
    const int rt = it + (half ? sd->RT / 2 : 0);
    const uint8_t *rec0 = sd->records + static_cast<size_t>(rt) * KS * kRecordBytes;
    const int rot = (it * 5) % KS;
    const uint16_t *x = sd->x;

    uintx4 xa[1][8];
#pragma unroll
    for (int f = 0; f < 8; ++f) xa[0][f] = uintx4{0, 0, 0, 0};   // lanes of tokens 1..15 stay zero
    const char *xs_rd = reinterpret_cast<const char *>(&xs[w][0]) + q * 16;
    float yacc = 0.f;
    bool first = true;

    for (int ks0 = part; ks0 < KS; ks0 += S * Wh) {
        uintx4 p1[S], p2[S];
        uintx2 sc[S], xr[S];
        int kx[S];
        // issue: S steps in flight.  Steps past the end re-read the wave's first step (address
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
            kx[i] = k < K ? k : 0;                      // odd number of groups: tail lanes
        }
        if constexpr (PERSIST) {
            if (first && sd->wait_count > 0) {
                // the records above are in flight; now wait for the level that writes x
                const __attribute__((address_space(1))) int32_t *done =
                    (const __attribute__((address_space(1))) int32_t *)(chain_done(plan) + (sd->level - 1));
                const __attribute__((address_space(1))) int32_t *stp =
                    (const __attribute__((address_space(1))) int32_t *)(&plan->status);
                const int need = sd->wait_count;
                int tries = 0;
                while (true) {
                    const int v = __hip_atomic_load(done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const int st = __hip_atomic_load(stp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (v >= need || st != PTQTP_OK) break;
                    if (++tries >= spin_limit) {
                        __hip_atomic_store(&plan->status, static_cast<int32_t>(PTQTP_ERR_WAIT), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(16);
                }
                if constexpr (SYNC == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            }
            first = false;
        }
#pragma unroll
        for (int i = 0; i < S; ++i) xr[i] = load_x8<COH>(x + kx[i]);
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
            if (pair) {
                const float g = red[0][nl] + red[1][nl];
                const float u = red[2][nl] + red[3][nl];
                out = (g / (1.0f + __expf(-g))) * u;
            } else {
                out = (red[0][nl] + red[1][nl]) + (red[2][nl] + red[3][nl]);
            }
            if (sd->residual != nullptr && n < n_out) {
                uint16_t rb;
                const uint16_t *rp = sd->residual + n;
                if constexpr (COH) rb = __hip_atomic_load((const __attribute__((address_space(1))) uint16_t *)(rp),
                                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else rb = load_global<uint16_t>(rp);
                out += half_bits_to_float(rb);
            }
        }
        if (sd->y_f16) {
            const uint32_t hb = __builtin_bit_cast(uint16_t, static_cast<_Float16>(out));
            const uint32_t nb = __shfl_down(hb, 1);                 // neighbour's half (n_out is even or the tail lane stores alone)
            if (lane < 16 && (lane & 1) == 0 && n < n_out) {
                uint16_t *yp = reinterpret_cast<uint16_t *>(sd->y) + n;
                if (n + 1 < n_out) {
                    const uint32_t word = hb | (nb << 16);
                    if constexpr (COH) __hip_atomic_store((gptr32w)(yp), word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else *reinterpret_cast<uint32_t *>(yp) = word;
                } else {                                          // last element of an odd-length output
                    if constexpr (COH) __hip_atomic_store((__attribute__((address_space(1))) uint16_t *)(yp),
                                                          static_cast<uint16_t>(hb), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else *yp = static_cast<uint16_t>(hb);
                }
            }
        } else if (lane < 16 && n < n_out) {
            uint32_t *yp = reinterpret_cast<uint32_t *>(sd->y) + n;
            const uint32_t fb = __builtin_bit_cast(uint32_t, out);
            if constexpr (COH) __hip_atomic_store((gptr32w)(yp), fb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else *yp = fb;
        }
        if constexpr (PERSIST) {
            // publish: stores first, then the level's completion counter (same wave, program order)
            if constexpr (SYNC == 0) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            } else {
                __builtin_amdgcn_s_waitcnt(0);                     // all counters to zero: stores acknowledged
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            }
            if (lane == 0)
                __hip_atomic_fetch_add(chain_done(plan) + sd->level, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

struct LevelRange { int first_item, items; };

// host-side geometry of a chain; returns false (and a status) on invalid input
bool chain_geometry(const ptqtp_stage *stages, int32_t count, int32_t group, StageDesc *descs /* count or null */,
                    LevelRange *levels /* count or null */, int *n_levels, int64_t *total_items, ptqtp_status *st)
{
    *st = PTQTP_OK;
    if (!stages) { *st = PTQTP_ERR_NULL; return false; }
    if (count <= 0 || count > PTQTP_CHAIN_MAX_STAGES) { *st = PTQTP_ERR_SHAPE; return false; }
    if (group != 128) { *st = PTQTP_ERR_GROUP; return false; }
    int64_t item = 0;
    int lv = -1, prev_level = -1, prev_level_items = 0, cur_level_items = 0;
    for (int i = 0; i < count; ++i) {
        const ptqtp_stage &s = stages[i];
        if (!s.packed || !s.x || !s.y) { *st = PTQTP_ERR_NULL; return false; }
        if (s.N <= 0 || s.K <= 0 || s.K % group != 0 || s.N > (1ll << 30) || s.K > (1ll << 30)) { *st = PTQTP_ERR_SHAPE; return false; }
        if (s.epilogue != PTQTP_EPI_NONE && s.epilogue != PTQTP_EPI_SWIGLU) { *st = PTQTP_ERR_SHAPE; return false; }
        if (s.epilogue == PTQTP_EPI_SWIGLU && s.N % 32 != 0) { *st = PTQTP_ERR_SHAPE; return false; }
        if (s.y_dtype != PTQTP_F32 && s.y_dtype != PTQTP_F16) { *st = PTQTP_ERR_DTYPE; return false; }
        if (s.level < 0 || s.level < prev_level || s.reserved != 0) { *st = PTQTP_ERR_SHAPE; return false; }
        if ((reinterpret_cast<uintptr_t>(s.packed) & 255) || (reinterpret_cast<uintptr_t>(s.x) & 15) ||
            (reinterpret_cast<uintptr_t>(s.y) & 15) || (reinterpret_cast<uintptr_t>(s.residual) & 15)) {
            *st = PTQTP_ERR_ALIGN; return false;
        }
        if (s.level != prev_level) {
            if (lv >= 0 && levels) levels[lv].items = cur_level_items;
            ++lv;
            prev_level_items = cur_level_items;
            cur_level_items = 0;
            if (levels) levels[lv].first_item = static_cast<int>(item);
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
            d.epilogue = s.epilogue; d.y_f16 = s.y_dtype == PTQTP_F16;
            d.level = lv; d.wait_count = lv == 0 ? 0 : prev_level_items;
            descs[i] = d;
        }
        item += items;
        cur_level_items += static_cast<int>(items);
        if (item > (1ll << 30)) { *st = PTQTP_ERR_SHAPE; return false; }
    }
    if (levels) levels[lv].items = cur_level_items;
    *n_levels = lv + 1;
    *total_items = item;
    return true;
}

inline int pad64(int v) { return (v + 63) & ~63; }

}  // namespace

extern "C" {

size_t ptqtp_chain_plan_bytes(const ptqtp_stage *stages, int32_t count, int32_t group) {
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, nullptr, nullptr, &n_levels, &total, &st)) return 0;
    const size_t bytes = sizeof(ChainHeader) + static_cast<size_t>(pad64(n_levels)) * 4 +
                         static_cast<size_t>(count) * sizeof(StageDesc) + static_cast<size_t>(total) * 4;
    return (bytes + 255) & ~static_cast<size_t>(255);
}

ptqtp_status ptqtp_chain_plan(const ptqtp_stage *stages, int32_t count, int32_t group,
                              void *plan, size_t plan_bytes, void *stream_) {
    if (!plan) return PTQTP_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(plan) & 255) return PTQTP_ERR_ALIGN;
    static thread_local StageDesc descs[PTQTP_CHAIN_MAX_STAGES];
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, descs, nullptr, &n_levels, &total, &st)) return st;
    if (plan_bytes < ptqtp_chain_plan_bytes(stages, count, group)) return PTQTP_ERR_SIZE;
    // a wait_count of a later level refers to the complete previous level: fix up stages that were
    // described before their level's item count was known (levels are contiguous runs)
    {
        static thread_local LevelRange lr[PTQTP_CHAIN_MAX_STAGES];
        chain_geometry(stages, count, group, nullptr, lr, &n_levels, &total, &st);
        for (int i = 0; i < count; ++i) descs[i].wait_count = descs[i].level == 0 ? 0 : lr[descs[i].level - 1].items;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ChainHeader *ph = static_cast<ChainHeader *>(plan);
    for (int base = 0; base < count; base += kChainChunk) {
        StageChunk chunk;
        const int n = count - base < kChainChunk ? count - base : kChainChunk;
        for (int i = 0; i < n; ++i) chunk.d[i] = descs[base + i];
        hipLaunchKernelGGL(chain_write_kernel, dim3(1), dim3(64), 0, stream, ph, chunk, base, n, count,
                           static_cast<int>(total), n_levels, pad64(n_levels));
    }
    const int blocks = static_cast<int>((total + 255) / 256) < 1024 ? static_cast<int>((total + 255) / 256) : 1024;
    hipLaunchKernelGGL(chain_map_kernel, dim3(blocks), dim3(256), 0, stream, ph);
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_chain_run(const ptqtp_stage *stages, int32_t count, int32_t group,
                             void *plan, int32_t mode, void *stream_) {
    if (!plan) return PTQTP_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(plan) & 255) return PTQTP_ERR_ALIGN;
    if (mode != PTQTP_CHAIN_LAUNCHES && mode != PTQTP_CHAIN_PERSISTENT) return PTQTP_ERR_SHAPE;
    static thread_local LevelRange lr[PTQTP_CHAIN_MAX_STAGES];
    int n_levels; int64_t total; ptqtp_status st;
    if (!chain_geometry(stages, count, group, nullptr, lr, &n_levels, &total, &st)) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ChainHeader *ph = static_cast<ChainHeader *>(plan);
    const dim3 block(kChainWaves * 64);
    if (mode == PTQTP_CHAIN_LAUNCHES) {
        for (int l = 0; l < n_levels; ++l)
            hipLaunchKernelGGL((chain_items_kernel<false, 0>), dim3(lr[l].items), block, 0, stream, ph,
                               lr[l].first_item, lr[l].items, 0);
    } else {
        const int limit = ptqtp_detail::g_chain_spin_limit > 0 ? ptqtp_detail::g_chain_spin_limit : kDefaultSpinLimit;
        const int sync = ptqtp_detail::g_chain_sync < 0 ? 0 : ptqtp_detail::g_chain_sync;
        hipLaunchKernelGGL(chain_reset_kernel, dim3(1), dim3(256), 0, stream, ph);
        if (sync == 0)
            hipLaunchKernelGGL((chain_items_kernel<true, 0>), dim3(static_cast<unsigned>(total)), block, 0, stream, ph,
                               0, static_cast<int>(total), limit);
        else
            hipLaunchKernelGGL((chain_items_kernel<true, 1>), dim3(static_cast<unsigned>(total)), block, 0, stream, ph,
                               0, static_cast<int>(total), limit);
    }
    return hipGetLastError() == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

ptqtp_status ptqtp_chain_status(const void *plan, int32_t *status_host, void *stream_) {
    if (!plan || !status_host) return PTQTP_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const ChainHeader *ph = static_cast<const ChainHeader *>(plan);
    if (hipMemcpyAsync(status_host, &ph->status, sizeof(int32_t), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return PTQTP_ERR_HIP;
    return hipStreamSynchronize(stream) == hipSuccess ? PTQTP_OK : PTQTP_ERR_HIP;
}

}  // extern "C"
