/*
 * flashkm.h — C ABI of the MI355X (gfx950) exact Lloyd k-means iteration.
 *
 * One Lloyd iteration (Flash-KMeans paper, Section 3.1, Eq. 2-3) is
 *     assignment  a_i = argmin_k || x_i - c_k ||^2
 *     update      n_k = #{i : a_i = k},  s_k = sum_{a_i = k} x_i,  c_k <- s_k / n_k
 * computed here as the paper's two kernels: a fused distance + online-argmin pass that
 * never stores the N x K distance matrix (Section 4.1, Algorithm 2), and a sort-inverse
 * update that argsorts the assignment vector and reduces contiguous cluster segments of
 * gathered rows (Section 4.2, Algorithm 3), plus the chunked host-streamed variant of
 * Section 4.3.
 *
 * Conventions shared by every entry point
 *   - Row-major, contiguous arrays.  B independent instances are stacked on the leading
 *     axis: X[B,N,d], C[B,K,d], assign[B,N], counts[B,K].
 *   - "device" pointers are HIP device memory owned by the caller, 16-byte aligned.
 *     The library never allocates or frees device memory; scratch space is the caller's
 *     `ws` buffer of at least fk_workspace_bytes(...) bytes (256-byte aligned), whose
 *     contents are undefined before and after a call.
 *   - X is never written.
 *   - Indices are 0-based int32 (the paper counts from 1).  Ties in the argmin: FK_F32 takes
 *     the lowest index among equal fp32 distances.  FK_F16 / FK_BF16 compare fp32 scores
 *     x.c - |c|^2/2 truncated to 19 mantissa bits; among centroids whose truncated scores are
 *     equal the lowest index wins, with one exception: inside a tile of 32 consecutive
 *     centroids (k / 32 equal) and among those of its rows that agree in bit 2 of k (one lane's
 *     16 rows), a NEGATIVE winning score (a point nearer the origin than any centroid) goes to
 *     the highest row instead.  Either way the chosen centroid's score is within 2^-19 relative
 *     of the best one, far inside the tolerance the parity tests allow.
 *     A cluster with no member keeps its previous centroid.
 *   - Inputs must be finite; for FK_F16 twice the largest centroid norm must stay finite
 *     in fp32 (always true for fp16 data).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it and return without waiting, except fk_lloyd_ooc.  The in-core calls
 *     enqueue kernels only (no memset, no allocation), so after one eager call for a shape
 *     they can be recorded into a HIP graph by stream capture and replayed.
 *   - Supported shapes: 1 <= K <= 65536, 1 <= N, B*N < 2^31, 1 <= B <= 65535, 1 <= d <= 512.
 *     The kernels work on rows whose width is a multiple of 8; for any other d the in-core
 *     entry points first copy X and C into zero-padded rows inside the workspace (zeros change
 *     no distance and no mean; costs one extra pass over X per call and room for the copy,
 *     which fk_workspace_bytes includes) and copy the centroids back without the padding;
 *     fk_lloyd_ooc lands the host rows in padded chunk buffers with a pitched copy instead.
 *     The fk_standard_* comparators need d to be a multiple of 8.  Anything else returns
 *     FK_EUNSUPPORTED or FK_EINVAL; there is no fallback path.
 *   - Calls act on the device that is current in the calling thread.  Kernel attributes,
 *     occupancy and the device's sizes (compute units, LDS, last-level cache) are asked of the
 *     runtime once per device and remembered; the options of fk_set_option are process-wide
 *     atomics.  The stage timer is the one part that is not thread safe.
 *   - Every function returns an fk_status; on failure fk_last_error() holds a message for
 *     the calling thread.  Nothing throws or aborts.
 */
#ifndef FLASHKM_H
#define FLASHKM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Storage type of X and of the low-precision centroids.  An int in the ABI: any other value is
 * answered with FK_EINVAL (in C++ the underlying type is fixed so that such a value is still a
 * valid object to pass and test). */
#ifdef __cplusplus
typedef enum : int { FK_F32 = 0, FK_F16 = 1, FK_BF16 = 2 } fk_dtype;
#else
typedef enum { FK_F32 = 0, FK_F16 = 1, FK_BF16 = 2 } fk_dtype;
#endif

typedef enum {
    FK_OK = 0,
    FK_EINVAL = 1,       /* NULL / misaligned pointer, non-positive size, bad enum */
    FK_EUNSUPPORTED = 2, /* a shape or dtype this build has no kernel for */
    FK_EWORKSPACE = 3,   /* ws_bytes smaller than fk_workspace_bytes(...) */
    FK_EHIP = 4          /* a HIP runtime call failed; see fk_last_error() */
} fk_status;

/* Message for the last failure on the calling thread (static storage, never NULL). */
const char* fk_last_error(void);

/* Device-workspace size in bytes that the in-core entry points below need for this
 * problem shape; 0 if the shape is unsupported.  Host-only, touches no GPU state. */
size_t fk_workspace_bytes(int B, int64_t N, int d, int K, fk_dtype t);

/*
 * Assignment stage (Eq. 2; Section 4.1, Algorithm 2).
 *   X       device, [B,N,d] of dtype t
 *   C       device, [B,K,d] of dtype t (the centroids as the kernel consumes them)
 *   assign  device out, [B,N] int32
 *   min_dist device out or NULL, [B,N] float: || x_i - c_{a_i} ||^2 as the kernel sees it
 *           (norm expansion of Section 3.1, fp32, clamped at 0)
 * fp16/bf16: the x.c contraction runs on MFMA with fp32 accumulation against
 * -||c_k||^2/2, the running (max, index) pair stays in registers over all centroid tiles
 * (the paper's online argmin, with the row-constant ||x||^2 dropped); fp32: plain fp32
 * direct differences.  HBM traffic is X + C read once, assign written once.
 */
fk_status fk_assign(const void* X, const void* C, int32_t* assign, float* min_dist,
                    int B, int64_t N, int d, int K, fk_dtype t,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * fk_assign for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as fk_assign, minus ws / ws_bytes: the fragment-ordered
 * centroid copy and the score bias go into a static device array inside the library
 * (16.25 MiB per GPU that uses the library, held until the process ends) instead of the
 * caller's workspace.  The call allocates and frees nothing.
 *   Limits: d a multiple of 8; for FK_F16 / FK_BF16
 *           B * ceil(K/32) * c(d) KiB <= fk_assign_static_limit() = 16 MiB, c(d) = 2, 4, 8, 16, 32
 *           for d <= 32, 64, 128, 256, 512 (K = 65536 at d = 128 with B = 1 just fits), and
 *           B * ceil(K/32) <= 2048.  Beyond that: FK_EWORKSPACE (d not a multiple of 8:
 *           FK_EUNSUPPORTED).  FK_F32 needs no scratch and has no limit of its own.
 *   Every call on a GPU shares that GPU's array and rewrites the part it needs before reading
 *   it; two calls that overlap in time on one GPU (different streams or threads) race.
 */
fk_status fk_assign_static(const void* X, const void* C, int32_t* assign, float* min_dist,
                           int B, int64_t N, int d, int K, fk_dtype t, void* stream);
size_t fk_assign_static_limit(void);

/*
 * Inverse mapping of Section 4.2 (Algorithm 3, first two lines): stable argsort of the
 * assignment vector by cluster id.
 *   assign      device, [B,N] int32 with values in [0,K)  (values outside are undefined
 *               behaviour of the result, never of memory: they are clamped)
 *   sorted_idx  device out, [B,N] int32: point indices grouped by cluster, ascending
 *               inside a cluster
 *   seg_offsets device out, [B,K+1] int32: cluster k owns sorted_idx[seg_offsets[k] ..
 *               seg_offsets[k+1]); seg_offsets[K] = N.  (This replaces the paper's
 *               sorted id sequence: K+1 offsets carry the same information.)
 */
fk_status fk_sort_inverse(const int32_t* assign, int32_t* sorted_idx, int32_t* seg_offsets,
                          int B, int64_t N, int K,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * Centroid update stage (Eq. 3; Section 4.2, Algorithm 3): sort-inverse + segment-level
 * reduction + normalisation.  No floating-point atomics: segment pieces are merged in a
 * fixed order, so results are bit-reproducible.
 *   X          device, [B,N,d] of dtype t
 *   assign     device, [B,N] int32 in [0,K)
 *   C_prev_f32 device, [B,K,d] float: rows kept for empty clusters
 *   C_out_f32  device out, [B,K,d] float (may alias C_prev_f32)
 *   C_out_lp   device out or NULL, [B,K,d] of dtype t: C_out_f32 rounded to nearest even
 *   counts     device out, [B,K] int32
 */
fk_status fk_update(const void* X, const int32_t* assign, const float* C_prev_f32,
                    float* C_out_f32, void* C_out_lp, int32_t* counts,
                    int B, int64_t N, int d, int K, fk_dtype t,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * `iters` Lloyd iterations (assignment with the current centroids, then update), all
 * enqueued on `stream` with no host synchronisation.
 *   C_f32   device in/out, [B,K,d] float master centroids
 *   C_lp    device out or NULL, [B,K,d] of dtype t: what the *next* assignment would
 *           consume (C_f32 rounded to nearest even).  Each iteration's assignment uses
 *           the rounding of the C_f32 it starts from.
 *   assign, counts  device out: those of the last iteration
 * iters == 0 is a no-op.
 */
fk_status fk_lloyd_iter(const void* X, float* C_f32, void* C_lp, int32_t* assign,
                        int32_t* counts, int B, int64_t N, int d, int K, fk_dtype t,
                        int iters, void* ws, size_t ws_bytes, void* stream);

/*
 * Out-of-core Lloyd iterations (Section 4.3, chunked stream overlap), B = 1.
 *   X_host     PINNED host memory, [N,d] of dtype t (hipHostMalloc; anything else, pageable
 *              memory included, is refused with FK_EINVAL).  Chunks of `chunk_rows` rows are
 *              copied with hipMemcpyAsync on a side stream owned by the call into two
 *              device buffers carved from dev_ws while the previous chunk is assigned and
 *              reduced on `stream`.
 *   C_f32      device in/out, [K,d] float.  The centroids are frozen during an iteration:
 *              sums and counts accumulate over the chunks, one normalisation per iteration
 *              (same result as the in-core path up to fp32 summation order).
 *   assign     device out or NULL, [N] int32 (last iteration)
 *   counts     device out, [K] int32
 *   chunk_rows rows per chunk; 0 = the largest that fits dev_ws_bytes
 *   dev_ws     device, dev_ws_bytes bytes: the whole device footprint of the call besides
 *              C_f32 / assign / counts.  fk_ooc_workspace_bytes gives the size needed for a
 *              given chunk_rows.
 * Blocks the calling thread until all iterations are done.
 */
fk_status fk_lloyd_ooc(const void* X_host, float* C_f32, int32_t* assign, int32_t* counts,
                       int64_t N, int d, int K, fk_dtype t, int iters, int64_t chunk_rows,
                       void* dev_ws, size_t dev_ws_bytes, void* stream);

/* Device bytes fk_lloyd_ooc needs for `chunk_rows` rows per chunk; 0 if unsupported. */
size_t fk_ooc_workspace_bytes(int64_t chunk_rows, int d, int K, fk_dtype t);

/*
 * Comparator only: the standard implementation the paper starts from (Section 3.1,
 * Algorithm 1).  Not used by any entry point above; built to measure, on this machine, what
 * the fused assignment and the sort-inverse update are compared against in the paper's
 * Section 5.2.
 *   fk_standard_assign  Kernel 1 writes D[B,N,K] (float, device, caller-provided: N*K*4 bytes
 *                       per instance) = ||x||^2 + ||c||^2 - 2 x.c with the x.c contraction on
 *                       MFMA; Kernel 2 reads D back and takes the row argmin.  fp16 / bf16,
 *                       d <= 128.  C is [B,K,d] of dtype t; ws as for fk_assign.
 *   fk_standard_update  Kernel 3 adds every point's features and a count into sums[B,K,d] /
 *                       counts[B,K] with atomics (order not reproducible); Kernel 4 divides.
 *                       sums is device scratch provided by the caller.  Any dtype, d <= 512.
 */
fk_status fk_standard_assign(const void* X, const void* C, float* D, int32_t* assign, int B,
                             int64_t N, int d, int K, fk_dtype t, void* ws, size_t ws_bytes,
                             void* stream);
fk_status fk_standard_update(const void* X, const int32_t* assign, const float* C_prev_f32,
                             float* C_out_f32, int32_t* counts, float* sums, int B, int64_t N,
                             int d, int K, fk_dtype t, void* stream);

/*
 * Kernel-configuration choice (the counterpart of the paper's cache-aware compile heuristic,
 * Section 4.3: a configuration is derived from the machine and the problem shape, with no
 * tuning run).  fk_plan writes a one-line description of what the in-core entry points would
 * launch for this shape into buf (host memory, NUL-terminated, truncated to buf_bytes):
 * assign kernel and tile shape, sort passes and tiling, reduction granularity, workspace.
 * Host-only.  fk_set_option changes a choice for every later call of this process, so that the
 * choices can be checked against the alternatives (value -1 = back to the rule of the shape):
 *   "assign_variant" v   tile shape v in 0..3 of the sweeping assign kernel
 *   "assign_stream"  0/1 few centroids: never / always (when they fit one LDS stage) take the
 *                        persistent streaming assign kernel
 *   "sort_stage_bins" n  the counting sort's scatter orders its tile in LDS before writing
 *                        when a pass has 32..n bins (default 1024; 0 = never)
 *   "sort_min_rounds" r  sort workgroups own at least r sub-tiles of 4096 keys (the rule gives
 *                        one up to 2^24 keys); changes fk_workspace_bytes, so set it before sizing
 *   "fused_update"   0   do not take the sort-free one-pass updates below
 *   "timer_repeat"   r   measurement only: while the stage timer runs, the assignment (or fused)
 *                        kernel and the segment reduction are each launched r times back to back
 *                        inside their interval (same outputs rewritten), so that interval /
 *                        launches approaches the kernel's own duration
 * Few clusters (FK_F16 / FK_BF16, K <= 32, d <= 128): fk_lloyd_iter computes assignment and
 * per-workgroup tables of sums in ONE pass over X (a one-hot MFMA adds each 32-point batch into
 * the K x d table; Section 4.2's on-chip partial sums with no sort needed), and fk_update
 * streams X once in storage order instead of sorting and gathering.  Same results as the
 * general path up to fp32 summation order; still no floating-point atomics, bit-reproducible.
 * Up to 256 clusters (FK_F16 / FK_BF16, 32 < K <= 256, d <= 128): fk_lloyd_iter also takes ONE
 * pass over X per iteration: a persistent workgroup per compute unit keeps the K x d table of sums
 * in the accumulators of its eight waves (32 clusters each) and adds the points it has just
 * assigned, compacted per wave, with a one-hot MFMA.  Same assignments and counts as the general
 * path, sums up to fp32 summation order, bit-reproducible.  fk_update alone keeps the
 * sort-inverse path for these shapes.
 * Small fp32 problems (FK_F32, K <= 64, d <= 128, B*N <= 2^17): fk_lloyd_iter likewise takes one
 * pass per iteration (64-point batches, distances by the same fp32 differences as fk_assign, each
 * cluster's row of the table of sums owned by one wave): at this size the iteration is bound by
 * its number of launches.  Same assignments and counts as the general path, sums up to fp32
 * summation order, bit-reproducible; fk_update alone keeps the sort-inverse path.
 * All of these passes need room for one partial table per workgroup, which fk_workspace_bytes
 * includes.
 */
int fk_plan(int B, int64_t N, int d, int K, fk_dtype t, char* buf, size_t buf_bytes);
int fk_set_option(const char* name, int value);

/*
 * Measurement aid (not a step of the method): while started, fk_lloyd_iter and fk_update
 * record a HIP event on their stream after each stage of every iteration -- assignment
 * kernel, sort-inverse, segment reduction, merge/normalise (with the centroid re-layout).
 * fk_stage_timer_stop waits for the last event and returns, per stage in that order,
 * the summed elapsed milliseconds and the number of kernel launches timed (one per interval
 * unless "timer_repeat" is set) in stage_ms[4] / stage_launches[4] (host arrays); its return value is the number of events recorded, or -1
 * on a HIP error.  One recorder per process, not thread safe; the events add a few
 * microseconds per stage, so throughput is measured with the timer stopped.
 */
void fk_stage_timer_start(void);
int fk_stage_timer_stop(double* stage_ms, int* stage_launches);

#ifdef __cplusplus
}
#endif
#endif /* FLASHKM_H */
