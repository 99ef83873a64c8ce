// Out-of-core Lloyd iterations: chunked stream overlap (paper Section 4.3).
//
// X stays in pinned host memory.  Two device chunk buffers are filled alternately by
// hipMemcpyAsync on a side stream while the compute stream runs assignment, sort-inverse
// and segment reduction on the other buffer.  Events order the two streams:
//   ready[i]  copy into buffer i finished      (compute waits)
//   freed[i]  compute on buffer i finished     (the next copy into i waits)
// The centroids are frozen for the whole iteration; per-chunk sums and counts are added
// onto running totals and normalised once after the last chunk, so the result is the
// in-core one up to fp32 summation order.
#include "fk_common.h"

namespace fk {

struct OocLayout {
    size_t chunk_bytes;   // one chunk buffer
    size_t core_bytes;    // in-core workspace for one chunk
    size_t assign_bytes;  // per-chunk assignment buffer (used when the caller keeps none)
    size_t total;
};

static bool ooc_layout(int64_t chunk_rows, int d, int K, fk_dtype t, OocLayout* L, Geometry* g) {
    if (!make_geometry(1, chunk_rows, d, K, t, g)) return false;
    // chunk buffers hold rows of the kernels' width (a multiple of 8); narrower host rows land in
    // them through a pitched copy, the padding columns are zeroed once
    L->chunk_bytes = align_up((size_t)chunk_rows * g->d * elem_size(t), 256);
    L->core_bytes = align_up(carve(*g, nullptr, false).bytes, 256);
    L->assign_bytes = align_up((size_t)chunk_rows * 4, 256);
    L->total = 2 * L->chunk_bytes + L->core_bytes + L->assign_bytes;
    return true;
}

}  // namespace fk

using namespace fk;

extern "C" {

size_t fk_ooc_workspace_bytes(int64_t chunk_rows, int d, int K, fk_dtype t) {
    OocLayout L;
    Geometry g;
    if (chunk_rows < 1 || !ooc_layout(chunk_rows, d, K, t, &L, &g)) return 0;
    return L.total;
}

fk_status fk_lloyd_ooc(const void* X_host, float* C_f32, int32_t* assign, int32_t* counts,
                       int64_t N, int d, int K, fk_dtype t, int iters, int64_t chunk_rows,
                       void* dev_ws, size_t dev_ws_bytes, void* stream) {
    if (N < 1 || d < 1 || K < 1 || iters < 0 || chunk_rows < 0) {
        set_error("fk_lloyd_ooc: N, d, K must be positive, iters and chunk_rows non-negative");
        return FK_EINVAL;
    }
    if (!X_host || !C_f32 || !counts || !dev_ws || ((uintptr_t)dev_ws & 255u) ||
        ((uintptr_t)C_f32 & 15u) || ((uintptr_t)counts & 15u) || ((uintptr_t)assign & 15u) ||
        ((uintptr_t)X_host & 15u)) {
        set_error("fk_lloyd_ooc: NULL or misaligned pointer");
        return FK_EINVAL;
    }
    {
        // X_host must be pinned (page-locked) host memory: from pageable memory hipMemcpyAsync
        // stages through a bounce buffer and the copies no longer overlap the kernels.  Both ends
        // of the array are looked up.
        const size_t bytes = (size_t)N * (size_t)d * elem_size(t);
        const char* ends[2] = {(const char*)X_host, (const char*)X_host + (bytes ? bytes - 1 : 0)};
        for (const char* p : ends) {
            hipPointerAttribute_t attr;
            const hipError_t pe = hipPointerGetAttributes(&attr, p);
            if (pe != hipSuccess) {
                (void)hipGetLastError();      // an unknown pointer is reported as an error: clear it
                set_error("fk_lloyd_ooc: X_host is not pinned host memory (the HIP runtime does not know the pointer: %s)",
                          hipGetErrorString(pe));
                return FK_EINVAL;
            }
            if (attr.type != hipMemoryTypeHost) {
                set_error("fk_lloyd_ooc: X_host must be pinned host memory (hipHostMalloc), got memory type %d",
                          (int)attr.type);
                return FK_EINVAL;
            }
        }
    }
    Geometry gfull;
    OocLayout L;
    if (chunk_rows == 0) {
        // largest multiple of 1024 rows (or all of N) whose footprint fits
        const int64_t unit = 1024;
        int64_t lo = 0, hi = cdiv(N, unit);
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) / 2;
            const int64_t rows = mid * unit < N ? mid * unit : N;
            if (ooc_layout(rows, d, K, t, &L, &gfull) && L.total <= dev_ws_bytes) lo = mid;
            else hi = mid - 1;
        }
        if (lo == 0) {
            set_error("fk_lloyd_ooc: dev_ws of %zu bytes cannot hold even a 1024-row chunk", dev_ws_bytes);
            return FK_EWORKSPACE;
        }
        chunk_rows = lo * unit < N ? lo * unit : N;
    }
    if (chunk_rows > N) chunk_rows = N;
    if (!ooc_layout(chunk_rows, d, K, t, &L, &gfull)) {
        set_error("fk_lloyd_ooc: unsupported shape chunk_rows=%lld d=%d K=%d", (long long)chunk_rows, d, K);
        return FK_EUNSUPPORTED;
    }
    if (L.total > dev_ws_bytes) {
        set_error("fk_lloyd_ooc: dev_ws too small: %zu bytes given, %zu needed for chunk_rows=%lld",
                  dev_ws_bytes, L.total, (long long)chunk_rows);
        return FK_EWORKSPACE;
    }
    if (iters == 0) return FK_OK;

    char* base = (char*)dev_ws;
    void* xbuf[2] = {base, base + L.chunk_bytes};
    void* core = base + 2 * L.chunk_bytes;
    int32_t* chunk_assign = (int32_t*)(base + 2 * L.chunk_bytes + L.core_bytes);
    const Workspace wfull = carve(gfull, core, false);
    const size_t row_bytes = (size_t)d * elem_size(t);                 // a row on the host
    const size_t dev_row_bytes = (size_t)gfull.d * elem_size(t);       // a row in a chunk buffer
    const bool pad = gfull.d != gfull.d_user;
    const int64_t nchunks = cdiv(N, chunk_rows);
    float* const C_user = C_f32;

    hipStream_t cs = (hipStream_t)stream;
    hipStream_t side = nullptr;
    hipEvent_t ready[2] = {nullptr, nullptr}, freed[2] = {nullptr, nullptr};
    fk_status st = FK_OK;
    auto cleanup = [&]() {
        for (int i = 0; i < 2; ++i) {
            if (ready[i]) (void)hipEventDestroy(ready[i]);
            if (freed[i]) (void)hipEventDestroy(freed[i]);
        }
        if (side) (void)hipStreamDestroy(side);
    };
#define OOC_HIP(call)                                      \
    do {                                                   \
        hipError_t _e = (call);                            \
        if (_e != hipSuccess) {                            \
            st = hip_fail(_e, #call);                      \
            (void)hipDeviceSynchronize();                  \
            cleanup();                                     \
            return st;                                     \
        }                                                  \
    } while (0)
#define OOC_TRY(expr)                                      \
    do {                                                   \
        st = (expr);                                       \
        if (st != FK_OK) {                                 \
            (void)hipDeviceSynchronize();                  \
            cleanup();                                     \
            return st;                                     \
        }                                                  \
    } while (0)

    OOC_HIP(hipStreamCreateWithFlags(&side, hipStreamNonBlocking));
    for (int i = 0; i < 2; ++i) {
        OOC_HIP(hipEventCreateWithFlags(&ready[i], hipEventDisableTiming));
        OOC_HIP(hipEventCreateWithFlags(&freed[i], hipEventDisableTiming));
    }
    bool used[2] = {false, false};
    if (pad) {
        OOC_HIP(hipMemsetAsync(xbuf[0], 0, 2 * L.chunk_bytes, side));
        OOC_TRY(launch_copy_rows(C_user, wfull.c_pad_f32, K, gfull.d_user, gfull.d, 4, cs));
        C_f32 = wfull.c_pad_f32;
    }

    for (int it = 0; it < iters; ++it) {
        OOC_TRY(launch_round_centroids(gfull, C_f32, t == FK_F32 ? nullptr : wfull.c_lp,
                                       wfull.c_frag, wfull.c_bias, cs));
        for (int64_t c = 0; c < nchunks; ++c) {
            const int bi = (int)(c & 1);
            const int64_t r0 = c * chunk_rows;
            const int64_t rows = (N - r0) < chunk_rows ? (N - r0) : chunk_rows;
            // side stream: refill buffer bi once its previous consumer is done
            if (used[bi]) OOC_HIP(hipStreamWaitEvent(side, freed[bi], 0));
            if (pad)
                OOC_HIP(hipMemcpy2DAsync(xbuf[bi], dev_row_bytes, (const char*)X_host + (size_t)r0 * row_bytes,
                                         row_bytes, row_bytes, (size_t)rows, hipMemcpyHostToDevice, side));
            else
                OOC_HIP(hipMemcpyAsync(xbuf[bi], (const char*)X_host + (size_t)r0 * row_bytes,
                                       (size_t)rows * row_bytes, hipMemcpyHostToDevice, side));
            OOC_HIP(hipEventRecord(ready[bi], side));
            // compute stream
            OOC_HIP(hipStreamWaitEvent(cs, ready[bi], 0));
            // A shorter tail chunk keeps the full chunk's tiling parameters and buffers
            // (every buffer is sized for chunk_rows); only the row-dependent counts shrink.
            Geometry g = gfull;
            const Workspace& w = wfull;
            g.N = rows;
            g.sort_blocks = (int)cdiv(rows, g.sort_tile);
            g.max_items = rows / g.rows_per_item + K;
            int32_t* a = assign ? assign + r0 : chunk_assign;
            if (t == FK_F32)
                OOC_TRY(launch_assign(g, xbuf[bi], C_f32, nullptr, a, nullptr, cs));
            else
                OOC_TRY(launch_assign(g, xbuf[bi], w.c_frag, w.c_bias, a, nullptr, cs));
            OOC_TRY(launch_sort_inverse(g, w, a, w.sorted_idx, w.seg_off, w.item_off, cs));
            OOC_TRY(launch_segment_reduce(g, w, xbuf[bi], w.sorted_idx, w.seg_off, w.item_off, cs));
            FinalizeArgs fa;
            fa.C_prev_f32 = C_f32;
            fa.C_out_f32 = C_f32;
            fa.C_out_lp = nullptr;
            fa.c_frag = nullptr;
            fa.c_bias = nullptr;
            fa.counts = counts;
            fa.sums = wfull.sums;
            fa.accumulate = c > 0;
            fa.normalise = (c + 1 == nchunks);
            OOC_TRY(launch_finalize(g, w, w.seg_off, w.item_off, fa, cs));
            OOC_HIP(hipEventRecord(freed[bi], cs));
            used[bi] = true;
        }
    }
    if (pad) OOC_TRY(launch_copy_rows(C_f32, C_user, K, gfull.d, gfull.d_user, 4, cs));
    OOC_HIP(hipStreamSynchronize(side));
    OOC_HIP(hipStreamSynchronize(cs));
    cleanup();
    return FK_OK;
#undef OOC_HIP
#undef OOC_TRY
}

}  // extern "C"
