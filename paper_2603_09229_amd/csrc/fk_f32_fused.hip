// Small problems in fp32 storage (K <= 64, d <= 128, at most 2^17 points in all): assignment
// (Eq. 2) and the per-cluster sums of Eq. 3 in one pass over X, without sort or gather.  At
// this size an iteration of the general path is six dependent launches of a few microseconds
// each; here it is two.  (For more points the one-point-per-thread assignment kernel followed by
// the sort-inverse update is faster: this kernel gives every wave all 64 points of a batch.)
//
// The table of sums is K x d floats; all of C fits LDS.  A workgroup of four waves walks
// 64-point batches: every wave holds the 64 points (one per lane, features in registers) and
// measures them against a quarter of the centroid rows by direct differences in fp32, exactly
// as the stand-alone fp32 assignment kernels do (so the assignments are bit-identical to
// theirs); the four candidates of a point are merged through LDS (smaller distance, then
// lower index).  Cluster k belongs to wave k % 4: that wave alone adds the batch's points of its
// clusters, in index order, to the cluster's row of a K x d table in LDS (lane = feature; LDS
// executes a wave's operations in order, so consecutive points of one cluster need no wait
// beyond the data dependency).  One owner per cluster row and a fixed order: no atomics,
// reproducible sums.  Every workgroup leaves one partial table and one count per cluster; the
// ordinary merge/normalise kernel adds them in workgroup order.
#include <algorithm>

#include "fk_common.h"
#include "fk_device.h"

namespace fk {

constexpr int kF32FusedMaxK = 64;

// Grid (G, B): workgroup g handles the 64-point batches g, g + G, ...
// partial: [B][K][G][d] floats, wg_counts: [B][K][G].
template <int DMAX>
__global__ __launch_bounds__(256) void f32_update_kernel(
    const float* __restrict__ X, const float* __restrict__ C, int32_t* __restrict__ assign,
    float* __restrict__ partial, int32_t* __restrict__ wg_counts, int64_t N, int d, int K) {
    constexpr int NR = DMAX > 64 ? 2 : 1;              // table elements per cluster and lane
    extern __shared__ float lds_f32[];
    float* sc = lds_f32;                               // [K][DMAX], zero beyond d
    float* tab = sc + kF32FusedMaxK * DMAX;            // [K][DMAX] sums
    float* xs = tab + kF32FusedMaxK * DMAX;            // [64][d]: the batch as stored
    float* cand_d = xs + 64 * DMAX;                    // [4][64]
    int* cand_k = (int*)(cand_d + 256);                // [4][64]
    int* tcnt = cand_k + 256;                          // [K] counts

    const int b = blockIdx.y, G = gridDim.x, wg = blockIdx.x;
    X += (size_t)b * N * d;
    C += (size_t)b * K * d;
    assign += (size_t)b * N;
    const int tid = threadIdx.x, lane = tid & 63;
    const int q = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int64_t nbatches = (N + 63) / 64;
    // own point's features of a batch: lane = point (every wave holds all 64 points)
    float x[DMAX];
    auto load_x = [&](int64_t t) {
        const int64_t i = t * 64 + lane;
#pragma unroll
        for (int j = 0; j < DMAX; j += 4) {
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (i < N && j < d) v = *(const floatx4*)(X + (size_t)i * d + j);
            x[j] = v[0]; x[j + 1] = v[1]; x[j + 2] = v[2]; x[j + 3] = v[3];
        }
    };
    load_x(wg);                                        // in flight while the centroids are staged

    for (int o = tid; o < K * DMAX; o += 256) {
        const int r = o / DMAX, j = o % DMAX;
        sc[o] = j < d ? C[(size_t)r * d + j] : 0.f;
        tab[o] = 0.f;
    }
    if (tid < kF32FusedMaxK) tcnt[tid] = 0;

    for (int64_t t = wg; t < nbatches; t += G) {
        const int64_t base = t * 64;
        const int rows = (int)min((int64_t)64, N - base);
        // the previous batch's readers of xs / cand are done (first pass: sc is complete)
        __syncthreads();
        {
            const floatx4* src = (const floatx4*)(X + (size_t)base * d);
            const int nvec = rows * d / 4;             // d is a multiple of 8
            for (int o = tid; o < nvec; o += 256) ((floatx4*)xs)[o] = src[o];
        }
        const int64_t i = base + lane;
        float m = INFINITY;
        int a = 0x7FFFFFFF;
        // rows q, q + 4, ... ascending with strict '<'; two rows at a time so that the two
        // dependent chains of adds overlap (each row's own sum keeps its order)
        for (int r = q; r < K; r += 8) {
            const int r1 = r + 4 < K ? r + 4 : r;      // past the end: row r again (loses the '<')
            float D0 = 0.f, D1 = 0.f;
#pragma unroll
            for (int j = 0; j < DMAX; j += 4) {
                const floatx4 c0 = *(const floatx4*)&sc[r * DMAX + j];
                const floatx4 c1 = *(const floatx4*)&sc[r1 * DMAX + j];
                const float e0 = x[j] - c0[0], e1 = x[j + 1] - c0[1];
                const float e2 = x[j + 2] - c0[2], e3 = x[j + 3] - c0[3];
                const float f0 = x[j] - c1[0], f1 = x[j + 1] - c1[1];
                const float f2 = x[j + 2] - c1[2], f3 = x[j + 3] - c1[3];
                D0 += e0 * e0; D1 += f0 * f0; D0 += e1 * e1; D1 += f1 * f1;
                D0 += e2 * e2; D1 += f2 * f2; D0 += e3 * e3; D1 += f3 * f3;
            }
            if (D0 < m) { m = D0; a = r; }
            if (D1 < m) { m = D1; a = r1; }
        }
        cand_d[q * 64 + lane] = m;
        cand_k[q * 64 + lane] = a;
        __syncthreads();                               // candidates and the batch copy are in LDS
        // every wave merges for itself: lane = point
        float bm = cand_d[lane];
        int bk = cand_k[lane];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float dm = cand_d[w * 64 + lane];
            const int dk = cand_k[w * 64 + lane];
            if (dm < bm || (dm == bm && dk < bk)) { bm = dm; bk = dk; }
        }
        bk = min(bk, K - 1);   // only reachable with non-finite input; keeps the index in range
        const bool valid = lane < rows;
        if (q == 0 && valid) assign[i] = bk;

        // the batch's points of this wave's clusters, in index order
        uint64_t mine = __ballot(valid && (bk & 3) == q);
        while (mine) {
            const int p = __builtin_ctzll(mine);
            mine &= mine - 1;
            const int k = __builtin_amdgcn_readlane(bk, p);
            float* trow = tab + k * DMAX;
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                const int j = lane + 64 * u;
                if (j < d) trow[j] += xs[p * d + j];
            }
            if (lane == 0) tcnt[k] += 1;
        }
        if (t + G < nbatches) load_x(t + G);           // lands behind the next barrier and copy
    }

    // the owner of a row wrote it: no barrier needed before reading it back
    for (int k = q; k < K; k += 4) {
        float* row = partial + (((size_t)b * K + k) * G + wg) * d;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int j = lane + 64 * u;
            if (j < d) row[j] = tab[k * DMAX + j];
        }
        if (lane == 0) wg_counts[((size_t)b * K + k) * G + wg] = tcnt[k];
    }
}

// ------------------------------------------------------------------------------------
bool f32_update_enabled(const Geometry& g) { return g.f32_grid_cap > 0 && fused_update_allowed(); }

template <int DMAX>
static fk_status launch_f32_update_t(const Geometry& g, const Workspace& w, const float* X,
                                     const float* C, int32_t* assign, int* grid_out,
                                     hipStream_t s) {
    auto kern = f32_update_kernel<DMAX>;
    const size_t lds = ((size_t)2 * kF32FusedMaxK * DMAX + 64 * DMAX + 512 + kF32FusedMaxK) * 4;
    // set / queried once per kernel and device: the launch path stays free of runtime queries afterwards
    static PerDeviceInt per_cu;
    if (per_cu.get() == 0) {
        FK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        int q = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, kern, 256, lds) != hipSuccess || q < 1) q = 1;
        per_cu.set(q);
    }
    int64_t G = cdiv((int64_t)device_cu_count() * per_cu.get(), g.B);
    G = std::min<int64_t>(G, g.f32_grid_cap);
    G = std::min<int64_t>(G, cdiv(g.N, 64));
    G = std::max<int64_t>(G, 1);
    dim3 grid((unsigned)G, g.B), block(256);
    hipLaunchKernelGGL(kern, grid, block, lds, s, X, C, assign, w.partial, w.wg_counts, g.N, g.d, g.K);
    FK_HIP(hipGetLastError());
    *grid_out = (int)G;
    return FK_OK;
}

fk_status launch_f32_update(const Geometry& g, const Workspace& w, const void* X,
                            const float* C_f32, int32_t* assign, int* grid_out, hipStream_t s) {
    if (g.f32_grid_cap <= 0) {
        set_error("fused fp32 update: shape not eligible (needs fp32 storage, K <= 64, d <= 128, B*N <= 2^17)");
        return FK_EUNSUPPORTED;
    }
    const float* Xf = (const float*)X;
    if (g.d <= 32) return launch_f32_update_t<32>(g, w, Xf, C_f32, assign, grid_out, s);
    if (g.d <= 64) return launch_f32_update_t<64>(g, w, Xf, C_f32, assign, grid_out, s);
    return launch_f32_update_t<128>(g, w, Xf, C_f32, assign, grid_out, s);
}

}  // namespace fk
