/*
 * libptqtp -- the decode-time hot path of PTQTP on AMD MI355X (gfx950).
 *
 * The layer (paper, Sec. "Magnitude-Topology Decoupling", Eq. 1-2; scales made
 * group-wise along the input dimension by paragraph "Batch Processing", G = 128):
 *
 *   y[m,n] = sum_g ( alpha1[n,g] * sum_{k in g} T1[n,k] x[m,k]
 *                  + alpha2[n,g] * sum_{k in g} T2[n,k] x[m,k] )
 *
 *   T1, T2 in {-1,0,+1}^{N x K}   two trit planes  (N = out features, K = in features)
 *   alpha1, alpha2  fp16 [N, K/G] one scale per (output row, group of G inputs)
 *   x  fp16 [M, K]  activations,  y  [M, N]  (no bias: the decomposition is bias-free)
 *
 * Sec. "Inference Efficiency" observes that a product with a trit is a sign
 * flip, a copy or a zero, so the plane products need additions only and the
 * two planes are independent; the only true multiplies are the 2 per
 * (row, group) scale applications.  Storage follows the appendix memory model:
 * 2 bits per trit per plane + two fp16 scales per (row, group) = 4 + 32/G bits
 * per weight (4.25 at G = 128).
 *
 * Conventions for every entry point
 *   - Pointers named "device" are HIP device pointers, 16-byte aligned (the packed
 *     blob and workspace 256-byte aligned); the caller owns every buffer.  The
 *     library never allocates or frees device memory and never synchronises: work
 *     is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and runs asynchronously.  (The plan-writing and chain calls use a few
 *     KB of host heap for their tables while they run.)
 *   - Threads: every entry point except ptqtp_tune may be called from several host
 *     threads at once (the one-time kernel attribute set-up behind the first launch
 *     of each kernel is an idempotent call guarded by an atomic flag).
 *   - Arguments are validated on the host before anything is launched; a
 *     non-zero status means nothing was enqueued and no memory was touched.
 *   - Outputs are overwritten, never accumulated into.  Results are
 *     deterministic: no atomics on floating-point data, fixed reduction order.
 *   - `group` must be 128.  K must be a multiple of `group`.  N is arbitrary
 *     (rows are padded to a multiple of 16 inside the blob; padding is never
 *     written to y).
 */
#ifndef PTQTP_H
#define PTQTP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t ptqtp_status;
enum {
    PTQTP_OK         = 0,
    PTQTP_ERR_NULL   = 1,  /* a required pointer is NULL                                   */
    PTQTP_ERR_SHAPE  = 2,  /* M, N or K not positive, K % group != 0, M out of range, N or K
                              above 2^30, or ceil(N/16) * ceil(K/256) above 2^27 (a packed
                              layer of 292 GB)                                             */
    PTQTP_ERR_GROUP  = 3,  /* group size not supported (only 128)                          */
    PTQTP_ERR_SIZE   = 4,  /* packed_bytes / workspace_bytes smaller than required         */
    PTQTP_ERR_DTYPE  = 5,  /* y_dtype is neither PTQTP_F32 nor PTQTP_F16                   */
    PTQTP_ERR_ALIGN  = 6,  /* a device pointer is not aligned as required                  */
    PTQTP_ERR_HIP    = 7   /* the HIP runtime reported an error at launch                  */
};

enum { PTQTP_F32 = 0, PTQTP_F16 = 1 };   /* y_dtype */

/* Largest batch ptqtp_gemm_small accepts on its streamed path. */
#define PTQTP_GEMM_SMALL_MAX_M 64

/* Library version: major*10000 + minor*100 + patch. */
int32_t ptqtp_version(void);

/* Static string for a status code (never NULL). */
const char *ptqtp_status_string(ptqtp_status s);

/*
 * Size in bytes of the packed blob for an N x K layer (appendix memory model:
 * N*K/2 bytes of planes + 4*N*K/group bytes of scales, after padding N to a
 * multiple of 16 and K to a multiple of 256, plus a 256-byte header).
 * Returns 0 for invalid arguments.  `M` is a batch hint and is currently ignored.
 */
size_t ptqtp_packed_bytes(int64_t M, int64_t N, int64_t K, int32_t group);

/* Workspace the compute calls need for this shape (currently always 0: the
 * cross-wave reduction lives in LDS).  Returns 0 for invalid arguments too. */
size_t ptqtp_workspace_bytes(int64_t M, int64_t N, int64_t K, int32_t group);

/*
 * Pack two trit planes and their scales into the device layout the compute
 * kernels stream (appendix memory model: 2-bit trits, fp16 scales).
 *
 *   T1, T2      device, int8 [N, K] row-major, entries in {-1,0,+1}; 2-byte alignment is
 *               enough, planes that are both 16-byte aligned are read 16 bytes at a time
 *   a1, a2      device, fp16 bit patterns [N, K/group] row-major
 *   packed      device, receives ptqtp_packed_bytes(M,N,K,group) bytes; opaque
 *   dev_status  device int32 or NULL; set to 0, then to 1 by the kernel if any
 *               entry of T1/T2 lies outside {-1,0,+1} (such an entry is stored as 0)
 * One-time, stream-ordered; not part of the timed decode step.
 */
ptqtp_status ptqtp_pack(const int8_t *T1, const int8_t *T2,
                        const uint16_t *a1, const uint16_t *a2,
                        int64_t M, int64_t N, int64_t K, int32_t group,
                        void *packed, size_t packed_bytes,
                        int32_t *dev_status, void *stream);

/*
 * Check that a blob is what the compute calls are about to take it for.  The compute kernels
 * trust the caller's N and K (they never read the header on the hot path): a blob packed for
 * another shape, or bytes that are not a blob at all, would be streamed as they are.  This call
 * compares the blob's header -- magic, layout id, group, N, K and the tile counts derived from
 * them (appendix memory model: what a packed layer consists of) -- with the arguments, on the
 * device, stream-ordered, without synchronising:
 *   packed, packed_bytes   device blob and its size; must hold ptqtp_packed_bytes(1,N,K,group)
 *   dev_status             device int32: receives 0 if everything matches, else an OR of
 *                          PTQTP_BLOB_BAD_* (read it after the stream has reached this point)
 * One thread, one 48-byte read: meant to be called once per blob when it is loaded or first used.
 * Host-side errors (nothing launched): PTQTP_ERR_NULL, _SHAPE, _GROUP, _SIZE, _ALIGN as elsewhere.
 */
enum {
    PTQTP_BLOB_BAD_MAGIC  = 1,   /* not a blob of this library                        */
    PTQTP_BLOB_BAD_LAYOUT = 2,   /* a record layout this build does not stream         */
    PTQTP_BLOB_BAD_GROUP  = 4,   /* packed with another group size                     */
    PTQTP_BLOB_BAD_N      = 8,   /* packed for another number of rows                  */
    PTQTP_BLOB_BAD_K      = 16   /* packed for another number of columns               */
};
ptqtp_status ptqtp_check_blob(const void *packed, size_t packed_bytes, int64_t N, int64_t K, int32_t group,
                              int32_t *dev_status, void *stream);

/*
 * Inverse of ptqtp_pack (bit-exact): recovers T1, T2 (int8 [N,K]) and a1, a2
 * (fp16 bits [N,K/group]) from a blob.  All pointers device.  Any of the four
 * outputs may be NULL to skip it.  Planes that are both 16-byte aligned are written 16
 * bytes at a time, others byte by byte.
 */
ptqtp_status ptqtp_unpack(const void *packed, int64_t M, int64_t N, int64_t K, int32_t group,
                          int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, void *stream);

/*
 * Batch-1 forward of the dual trit-plane layer (Eq. 1-2, group-wise scales):
 *   y[n] = sum_g alpha1[n,g]*(T1[n,g,:] . x[g,:]) + alpha2[n,g]*(T2[n,g,:] . x[g,:])
 *
 *   packed   device, blob from ptqtp_pack for the same N, K, group
 *   x        device, fp16 bits [K]
 *   y        device, [N] of float (PTQTP_F32) or fp16 bits (PTQTP_F16)
 *   M        must be 1
 *   workspace, workspace_bytes   device scratch of >= ptqtp_workspace_bytes(...)
 *            bytes; may be NULL when that is 0
 * fp32 accumulation of exact +-x terms; one fp32 multiply per (row, group, plane).
 */
ptqtp_status ptqtp_gemv(const void *packed, const uint16_t *x, void *y, int32_t y_dtype,
                        int64_t M, int64_t N, int64_t K, int32_t group,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Small-batch forward, 1 <= M <= PTQTP_GEMM_SMALL_MAX_M: the same sum for every
 * token m, each decoded trit reused for all M tokens.
 *   x  device fp16 bits [M, K] row-major;  y  device [M, N] row-major.
 */
ptqtp_status ptqtp_gemm_small(const void *packed, const uint16_t *x, void *y, int32_t y_dtype,
                              int64_t M, int64_t N, int64_t K, int32_t group,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Any batch, 1 <= M <= PTQTP_GEMM_MAX_M: dispatches to the batch-1 kernel, the small-batch
 * kernel (in chunks of 64 tokens up to 255), or -- from 256 tokens (prefill), where the
 * layer is a dense contraction -- an MFMA tile that stages activations in LDS and feeds
 * alpha*T (exact in fp16) to the matrix pipe.  Arguments as in ptqtp_gemm_small.
 */
/*
 * PTQTP_FUSED_PLANES, OR-ed into y_dtype of ptqtp_gemm (and of a ptqtp_stage, where it counts in
 * ptqtp_chain_run_batch) only: from 256 tokens on, rebuild the weight
 * before the matrix pipe, w16 = fp16(alpha1*t1 + alpha2*t2) -- ONE rounding per weight, both
 * products being exact in fp16 -- and run one MFMA pass over w16 instead of one per plane (the
 * "dequantization" forward Sec. "Inference Efficiency" names beside the dequantization-free one).
 * The result is the exact layer of the rounded weights: |y - y_unfused| <= 2^-11 * B with B the
 * L1 bound sum_k (|alpha1 t1| + |alpha2 t2|) |x_k|.  Below 256 tokens the flag has no effect.
 */
#define PTQTP_FUSED_PLANES 16
#define PTQTP_GEMM_MAX_M 65536
ptqtp_status ptqtp_gemm(const void *packed, const uint16_t *x, void *y, int32_t y_dtype,
                        int64_t M, int64_t N, int64_t K, int32_t group,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Many independent batch-1 layers in ONE launch (fused q/k/v, gate/up, or a whole
 * stack of layers whose inputs are all known): the same sum as ptqtp_gemv for each
 * entry.  One launch covers every 16-row tile of every entry, so the HBM stream does
 * not drain between layers and small layers share the chip with their neighbours.
 *
 * ptqtp_gemv_batch_plan writes a small device-side table (one-time, stream-ordered):
 *   linears     HOST array of `count` entries; every pointer inside is a device
 *               pointer with the meaning and alignment it has in ptqtp_gemv; the
 *               entries' y buffers must not overlap each other or any x
 *   plan        device, receives ptqtp_batch_plan_bytes(linears,count,group) bytes,
 *               256-byte aligned
 * ptqtp_gemv_batch runs the plan: `items` must be ptqtp_batch_items(...) of the same
 * list (= sum over entries of ceil(N/16) rounded up to a multiple of 16).  The plan may be
 * re-run any number of times and stays valid while the buffers it names are alive.
 * ptqtp_batch_plan_bytes and ptqtp_batch_items return 0 for invalid arguments.
 */
#define PTQTP_BATCH_MAX_LINEARS 4096
typedef struct ptqtp_linear {
    const void *packed;     /* device, blob from ptqtp_pack for this N, K */
    const uint16_t *x;      /* device, fp16 bits [K] */
    void *y;                /* device, [N] of the plan's y_dtype */
    int64_t N, K;
} ptqtp_linear;

size_t ptqtp_batch_plan_bytes(const ptqtp_linear *linears, int32_t count, int32_t group);
int64_t ptqtp_batch_items(const ptqtp_linear *linears, int32_t count, int32_t group);
ptqtp_status ptqtp_gemv_batch_plan(const ptqtp_linear *linears, int32_t count, int32_t y_dtype, int32_t group,
                                   void *plan, size_t plan_bytes, void *stream);
ptqtp_status ptqtp_gemv_batch(const void *plan, int64_t items, void *stream);

/*
 * The same plan run with M tokens per entry, 1 <= M <= PTQTP_GEMM_SMALL_MAX_M: every entry's x is
 * then fp16 [M, K] row-major and its y [M, N] row-major (the plan only stores the pointers; M is
 * given here and must be the same for all entries).  One launch of the small-batch kernel over
 * every 16-row tile of every entry.
 */
ptqtp_status ptqtp_gemm_batch(const void *plan, int64_t items, int64_t M, void *stream);

/*
 * ptqtp_gemm_batch with the arithmetic of PTQTP_FUSED_PLANES where that pays: from 33 tokens on, each weight is
 * rebuilt before the matrix pipe, w16 = fp16(alpha1*t1 + alpha2*t2) (one rounding, both products exact in fp16:
 * the "dequantization" forward of Sec. "Inference Efficiency"), and one MFMA pass runs over w16 instead of one per
 * plane; the result is the exact layer of the rounded weights, |y - y_unfused| <= 2^-11 * B as for ptqtp_gemm.
 * Up to 32 tokens, where the matrix pipe is not what binds, the call is ptqtp_gemm_batch bit for bit.
 * Arguments and errors as in ptqtp_gemm_batch.
 */
ptqtp_status ptqtp_gemm_batch_fused(const void *plan, int64_t items, int64_t M, void *stream);

/*
 * Decode chain: the dependent linears of a decoder block (and of a whole stack of blocks) at
 * batch 1, with the steps either side of them fused into the producing kernel.  The paper
 * replaces every linear projection of LLaMA-family blocks (Sec. "Experiments", setup) and
 * times token generation (Sec. "Inference Efficiency"); around the linears such a block has
 * a gated MLP, down(silu(gate x) * up x) with silu(z) = z / (1 + exp(-z)), and a residual
 * stream that adds each sublayer's output to its input.
 *
 * A chain is an array of stages.  Stage s computes its linear y = W^ x (the sum at the top of
 * this header, M = 1) and then its epilogue:
 *   PTQTP_EPI_NONE     out[n] = y[n]                         n < N
 *   PTQTP_EPI_SWIGLU   out[i] = silu(y[i]) * y[N/2 + i]      i < N/2; the blob stacks the N/2
 *                      gate rows over the N/2 up rows; N must be a multiple of 32
 *   then, if residual != NULL, out += residual (fp16), and out is stored as y_dtype.
 * `level` orders the stages: levels are non-decreasing along the array, stages of one level
 * are independent of each other, and a stage may read (as x or residual) what stages of
 * lower levels wrote as fp16.  A stage's y may be its own residual buffer (in-place residual
 * stream) but must not overlap anything else a stage of the same or the previous level reads.
 *
 *   ptqtp_chain_plan   writes the device-side table (one-time, stream-ordered): plan receives
 *                      ptqtp_chain_plan_bytes(...) bytes, 256-byte aligned
 *   ptqtp_chain_run    runs the chain: one launch per level, in stream order (capture it in a
 *                      HIP graph to replay a decode step); a level with few work items gets more
 *                      waves per item.  `stages`, `count` must be the ones the plan was written from.
 *   ptqtp_chain_run_batch  the same chain at M tokens, 1 <= M <= PTQTP_GEMM_MAX_M: every x is then
 *                      fp16 [M, K] row-major, every y and residual [M, N] (or [M, N/2]) row-major.  One
 *                      launch per stage, in array order: the small-batch kernel up to
 *                      PTQTP_GEMM_SMALL_MAX_M tokens, an MFMA tile with the epilogue in its store above
 *                      (a prompt through the same chain); needs no plan.
 * ptqtp_chain_plan_bytes returns 0 for invalid arguments.
 */
enum { PTQTP_EPI_NONE = 0, PTQTP_EPI_SWIGLU = 1 };
#define PTQTP_CHAIN_MAX_STAGES 4096
typedef struct ptqtp_stage {
    const void *packed;        /* device, blob from ptqtp_pack for this N, K */
    const uint16_t *x;         /* device, fp16 bits [K] */
    void *y;                   /* device, [N] (PTQTP_EPI_NONE) or [N/2] (PTQTP_EPI_SWIGLU) of y_dtype */
    const uint16_t *residual;  /* device, fp16 bits, as long as y, or NULL */
    int64_t N, K;
    int32_t epilogue;          /* PTQTP_EPI_* */
    int32_t y_dtype;           /* PTQTP_F32 or PTQTP_F16 */
    int32_t level;             /* >= 0, non-decreasing along the array */
    int32_t reserved;          /* 0 */
} ptqtp_stage;

size_t ptqtp_chain_plan_bytes(const ptqtp_stage *stages, int32_t count, int32_t group);
ptqtp_status ptqtp_chain_plan(const ptqtp_stage *stages, int32_t count, int32_t group,
                              void *plan, size_t plan_bytes, void *stream);
ptqtp_status ptqtp_chain_run(const ptqtp_stage *stages, int32_t count, int32_t group,
                             const void *plan, void *stream);
ptqtp_status ptqtp_chain_run_batch(const ptqtp_stage *stages, int32_t count, int32_t group, int64_t M, void *stream);

/*
 * The step before the path: PTQTP decomposition of an fp16 weight matrix into the two trit
 * planes and scales that ptqtp_pack takes (paper, Sec. "Dual Trit-planes Approximation" and
 * "Progressive Optimization", both algorithm listings): per (row, group) unit, initialise
 * T1 = T2 = sign(w) (0 -> +1), alpha = [1,1], lambda = 1e-8; then up to max_iters times solve the
 * 2x2 ridge system alpha = (S'S + lambda I)^-1 S'w (lambda raised to min(1, lambda*sqrt(kappa/1e6))
 * first when kappa = ||A||_F ||A^-1||_F >= 1e6) and re-pick every trit pair as the first minimiser of
 * (w - alpha1 c1 - alpha2 c2)^2 over the nine pairs in the order c1 = -1,0,1 (outer), c2 = -1,0,1
 * (inner); stop when the Frobenius norm of the change of all scales of the matrix is below eps.
 * The paper's settings are max_iters = 50, eps = 1e-4.  All arithmetic that decides a trit is
 * binary64 and reproducible; the scales are stored as their binary16 rounding.
 *
 *   W           device, fp16 bits [N, K] row-major (finite values)
 *   T1, T2      device, int8 [N, K], overwritten (also used as state between iterations)
 *   a1, a2      device, fp16 bits [N, K/group], overwritten
 *   iters       device int32 or NULL: receives the number of iterations performed
 *   workspace   device, >= ptqtp_quantize_workspace_bytes(N, K, group) bytes, 256-byte aligned
 * Stream-ordered, never synchronises: 2 launches per iteration; once the stopping rule has fired
 * the remaining launches return immediately.
 * Errors: PTQTP_ERR_SHAPE for N or K above 2^30, N * K above 2^37, K % group != 0, max_iters outside
 * 0..10000 or eps negative or NaN (the workspace size is 0 for such a shape); the others as above.
 */
size_t ptqtp_quantize_workspace_bytes(int64_t N, int64_t K, int32_t group);
ptqtp_status ptqtp_quantize(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                            int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, int32_t *iters,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * ptqtp_quantize for callers that cannot allocate device memory or pass a workspace along (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same decomposition, the same kernels and
 * bit-identical results, with the workspace in a file-scope device array of PTQTP_QUANTIZE_STATIC_BYTES (16 MiB + 256
 * bytes, present once on every device the library runs on until the process ends).  The call allocates and frees
 * nothing.  Layers whose workspace would be larger -- ptqtp_quantize_workspace_bytes(N, K, group) >
 * PTQTP_QUANTIZE_STATIC_BYTES, i.e. more than 524,288 (row, group) units, e.g. above 16384 x 4096 -- are refused with
 * PTQTP_ERR_SIZE; PTQTP_ERR_HIP if the array's address cannot be obtained on the current device.  Every call on a
 * device shares that device's array: calls that overlap on one device (two streams, two threads) race; calls on
 * one stream are ordered.  Other arguments and errors as for ptqtp_quantize.
 */
#define PTQTP_QUANTIZE_STATIC_BYTES (16u * 1024u * 1024u + 256u)
ptqtp_status ptqtp_quantize_static(const uint16_t *W, int64_t N, int64_t K, int32_t group, int32_t max_iters, double eps,
                                   int8_t *T1, int8_t *T2, uint16_t *a1, uint16_t *a2, int32_t *iters, void *stream);

/*
 * Which kernels ptqtp_gemm would run for a shape (host logic only, no GPU needed; for tests and sweeps).
 * route[0] = PTQTP_ROUTE_*; for PTQTP_ROUTE_TILE route[1] = workgroup tile of the (first) launch
 * (0 = 256 rows x 256 tokens, 1 = 256 x 128, 2 = 128 x 128, 3 = 128 x 64, 4 = 64 x 64), route[2] = the
 * row (a multiple of 256) at which a second launch takes over, divided by 16, or 0, route[3] = that second
 * launch's tile or -1.  The choice never changes what is computed per accumulator within the tile path
 * (all tiles add the groups in the same order); it follows ptqtp_tune.  y_dtype as for ptqtp_gemm.
 */
#define PTQTP_ROUTE_STREAM 0        /* batch 1: streamed rows */
#define PTQTP_ROUTE_SMALL 1         /* small-batch kernel, one launch */
#define PTQTP_ROUTE_SMALL_CHUNKS 2  /* small-batch kernel on chunks of 64 tokens */
#define PTQTP_ROUTE_TILE 3          /* MFMA tile(s) */
ptqtp_status ptqtp_gemm_route(int64_t M, int64_t N, int64_t K, int32_t group, int32_t y_dtype, int32_t *route);

/*
 * Tuning hook for benchmarks and sweeps (not needed for correct use): override
 * the launch shape the compute calls pick.  key = "stream_waves" (batch 1: waves per item, 1..16),
 * "stream_depth" (batch 1: records in flight per wave: 1, 2 or 4), "small_waves" (one linear at batch > 1:
 * waves per item, 1..8), "small_rows" (row tiles per item / per wave of the small-batch kernels: 1 or 2, for ptqtp_gemm_batch also 4, and 8 = two per wave in a workgroup of eight waves),
 * "chain_waves" (ptqtp_chain_run: waves per item, an even number up to 16), "chain_depth" (ptqtp_chain_run:
 * records in flight per wave: 1, 2 or 4), "chain_table" (ptqtp_chain_run: 1 = every level looks its stages up in the
 * device-side plan, 0 = default: levels of up to four stages carry their descriptors as kernel arguments), "batch_rows_kernel" (ptqtp_gemm_batch: 0 = per-wave activation loads, -1/1 = shared activation tile),
 * "small_fold" (ptqtp_gemm_batch with two row tiles per wave: 1 = multiply the group scales into the
 * expanded trits before the matrix pipe, 0 = rescale the per-group sums after it, -1 = default: before for
 * more than 32 tokens), "small_ahead" (one linear at 17..64 tokens, up to two row tiles per item: 1 = the item
 * kernel whose loads run one step ahead of its arithmetic, 0 = the plain one, -1 = default: by shape),
 * "tile" (1 = use an MFMA tile for every batch > 1, -1 = never below 256 tokens,
 * 0 = default: by cost model from 33 tokens on), "tile_variant" (workgroup tile, rows x tokens: 1 = 256 x 128, 2 = 128 x 128, 3 = 256 x 256, 4 = 128 x 64, 5 = 64 x 64,
 * 0 = default: the cheapest by a cost model of the problem size; also honoured by ptqtp_chain_run_batch
 * above PTQTP_GEMM_SMALL_MAX_M tokens where the stage allows the tile);
 * value 0 restores the built-in heuristic.  Returns PTQTP_ERR_SHAPE for an
 * unknown key or out-of-range value.  Not thread-safe: the overrides are process-wide globals, to be set while no
 * other thread is inside the library.
 */
ptqtp_status ptqtp_tune(const char *key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* PTQTP_H */
