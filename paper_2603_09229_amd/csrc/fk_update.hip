// Segment-level aggregation and normalisation of the sort-inverse update (paper Section
// 4.2, Algorithm 3; Eq. 3).
//
// The paper cuts the sorted order into fixed chunks, accumulates each cluster-id segment
// of a chunk on chip and merges it with one atomic_add per segment.  Here the cut follows
// the segments instead: cluster k's run of n_k sorted positions is split into
// ceil(n_k / R) "items" of at most R positions, one wave reduces one item in registers and
// writes one partial row, and a second kernel adds a cluster's partial rows in item order.
// That keeps the paper's bound on merges (at most K + N/R rows are merged) but needs no
// atomics at all and is bit-reproducible.  X is gathered by whole rows through sorted_idx
// and never permuted in memory.
#include "fk_common.h"
#include "fk_device.h"

namespace fk {

namespace {

// Largest k in [0,K) with item_off[k] <= item, found by the whole wave 64 probes at a
// time.  Requires item < item_off[K]; the cluster found is then non-empty.
__device__ __forceinline__ int find_cluster(const int32_t* __restrict__ item_off, int K,
                                            int item, int lane) {
    int lo = 0, hi = K;
    while (hi - lo > 1) {
        const int step = (hi - lo + 63) >> 6;
        const int probe = lo + lane * step;
        const bool le = probe < hi && item_off[probe] <= item;
        const int cnt = __popcll(__ballot(le));   // monotone: a prefix of the lanes
        lo += (cnt - 1) * step;
        hi = min(hi, lo + step);
    }
    return lo;
}

}  // namespace

// WPI waves per item (1, or all 4 of the workgroup for the long items of few-cluster
// shapes).  EPL elements of 16 bytes per lane (8 for 16-bit types, 4 for fp32); 2^lpr_log2
// lanes span a row, so a wave reads 64 >> lpr_log2 rows per load instruction.  With WPI = 4
// wave w takes the 64-row batches w, w+4, ... of the item and the four wave sums are added in
// wave order through LDS.
template <int EPL, bool BF, int WPI>
__global__ __launch_bounds__(256) void segment_reduce_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ sorted_idx,
    const int32_t* __restrict__ seg_off, const int32_t* __restrict__ item_off,
    float* __restrict__ partial, int64_t N, int d, int K, int R, int64_t max_items,
    int lpr_log2) {
    __shared__ float wsum[WPI == 4 ? 4 : 1][WPI == 4 ? 512 : 1];
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t item = WPI == 4 ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
    const int part = WPI == 4 ? wave : 0;          // which share of the item this wave takes
    seg_off += (size_t)b * (K + 1);
    item_off += (size_t)b * (K + 1);
    sorted_idx += (size_t)b * N;
    if (item >= item_off[K]) return;   // uniform over the waves that share an item
    const int k = find_cluster(item_off, K, (int)item, lane);
    const int piece = (int)item - item_off[k];
    const int start = seg_off[k] + piece * R;
    const int end = min(seg_off[k + 1], start + R);

    const int LPR = 1 << lpr_log2, S = 64 >> lpr_log2;
    const int slot = lane >> lpr_log2;
    const char* X = (const char*)Xv + (size_t)b * N * d * (16 / EPL);
    // rows wider than one wave-load (64 lanes x 16 bytes) are reduced one column block at a time
    const int ncb = (d + 64 * EPL - 1) / (64 * EPL);
    for (int cb = 0; cb < ncb; ++cb) {
        const int col = cb * 64 * EPL + (lane & (LPR - 1)) * EPL;
        const bool active = col < d;
        float acc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

        constexpr int U = 8;
        for (int r0 = start + part * 64; r0 < end; r0 += 64 * WPI) {
            const int nrows = min(64, end - r0);
            const int myidx = lane < nrows ? sorted_idx[r0 + lane] : 0;
            for (int q = 0; q < nrows; q += S * U) {
                uintx4 v[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int rr = q + u * S + slot;
                    const int idx = __shfl(myidx, rr & 63);
                    ok[u] = active && rr < nrows;
                    v[u] = uintx4{0u, 0u, 0u, 0u};
                    if (ok[u]) v[u] = *(const uintx4*)(X + ((size_t)idx * d + col) * (16 / EPL));
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (EPL == 4) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[e] += __uint_as_float(v[u][e]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            acc[2 * e] += lp_to_float((uint16_t)(v[u][e] & 0xFFFFu), BF);
                            acc[2 * e + 1] += lp_to_float((uint16_t)(v[u][e] >> 16), BF);
                        }
                    }
                }
            }
        }
        // add the row slots of the wave together (fixed butterfly order)
        for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], o);
        }
        if (slot == 0 && active) {
            if (WPI == 1) {
                float* out = partial + ((size_t)b * max_items + item) * d + col;
#pragma unroll
                for (int e = 0; e < EPL; e += 4)
                    *(floatx4*)(out + e) = floatx4{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e) wsum[wave][col + e] = acc[e];
            }
        }
    }
    if (WPI == 4) {
        __syncthreads();
        for (int j = threadIdx.x; j < d; j += 256) {
            const float s = ((wsum[0][j] + wsum[1][j]) + wsum[2][j]) + wsum[3][j];
            partial[((size_t)b * max_items + item) * d + j] = s;
        }
    }
}

// One workgroup (256 threads, or 1024 when clusters have many items) per cluster: s_k = sum
// of the cluster's item rows in a fixed
// order, n_k = seg_off[k+1] - seg_off[k].  Optionally added onto sums/counts already stored
// (chunked mode), optionally normalised into centroids (Algorithm 3, last loop; an empty
// cluster keeps its previous centroid).  When c_frag is given, the rounded centroid is also
// written in MFMA fragment order together with its score bias -||c||^2/2, so the next
// assignment needs no separate re-layout pass.
__global__ __launch_bounds__(1024) void finalize_kernel(
    const float* __restrict__ partial, const int32_t* __restrict__ seg_off,
    const int32_t* __restrict__ item_off, const float* C_prev, float* C_out,
    uint16_t* __restrict__ C_lp_out, float* __restrict__ C_lp_f32_out,
    uint16_t* __restrict__ c_frag, float* __restrict__ c_bias, int32_t* __restrict__ counts,
    float* __restrict__ sums, int d, int K, int64_t max_items, int ktiles, int dch,
    int accumulate, int normalise, int bf, const int32_t* __restrict__ wg_counts, int G) {
    // dynamic LDS: 4 floats per thread for the row sums, then d floats for the squared entries
    // (a fixed worst-case array would cap the small workgroups of many-cluster shapes at a
    // few per CU)
    extern __shared__ float fin_lds[];
    float* red = fin_lds;
    float* nrm = fin_lds + 4 * blockDim.x;
    __shared__ int cred[16];
    const int b = blockIdx.y, k = blockIdx.x, tid = threadIdx.x;
    int dpow = 4;
    while (dpow < d) dpow <<= 1;
    const int LR = dpow >> 2;                     // threads per row, 4 features each
    const int slots = (int)blockDim.x / LR, slot = tid / LR, col = (tid % LR) * 4;
    int i0, i1;
    if (wg_counts) {
        // few-cluster path: cluster k owns G partial rows and G partial counts
        i0 = k * G;
        i1 = i0 + G;
        int v = 0;
        for (int g = tid; g < G; g += (int)blockDim.x) v += wg_counts[((size_t)b * K + k) * G + g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if ((tid & 63) == 0) cred[tid >> 6] = v;
    } else {
        seg_off += (size_t)b * (K + 1);
        item_off += (size_t)b * (K + 1);
        i0 = item_off[k];
        i1 = item_off[k + 1];
    }
    // read the running count before anyone overwrites it (barrier below)
    const int n_prev = accumulate ? counts[(size_t)b * K + k] : 0;
    const float* P = partial + (size_t)b * max_items * d;
    // eight rows in flight per thread; the eight running sums are added in a fixed order
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    if (col < d) {
        floatx4 a8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a8[u] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int it = i0 + slot; it < i1; it += 8 * slots) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = it + u * slots;
                if (r < i1) a8[u] += *(const floatx4*)(P + (size_t)r * d + col);
            }
        }
        acc = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
    }
    *(floatx4*)&red[slot * dpow + col] = acc;
    __syncthreads();
    const int T = (int)blockDim.x;
    int n = n_prev;
    if (wg_counts) {
        for (int q = 0; q < ((int)blockDim.x + 63) / 64; ++q) n += cred[q];
    } else {
        n += seg_off[k + 1] - seg_off[k];
    }
    for (int j = tid; j < d; j += T) {
        float s = 0.f;
        for (int q = 0; q < slots; ++q) s += red[q * dpow + j];   // fixed order
        const size_t o = ((size_t)b * K + k) * d + j;
        if (accumulate) s += sums[o];
        if (sums) sums[o] = s;
        if (normalise) {
            const float c = n > 0 ? (float)((double)s / (double)n) : C_prev[o];
            C_out[o] = c;
            const uint16_t lp = float_to_lp(c, bf);
            if (C_lp_out) C_lp_out[o] = lp;
            if (C_lp_f32_out) C_lp_f32_out[o] = c;
            if (c_frag) {
                // fragment order: tile k/32, chunk j/16, lane (j%16)/8*32 + k%32, element j%8
                const size_t pos = ((((size_t)b * ktiles + (k >> 5)) * dch + (j >> 4)) * 64 +
                                    (((j >> 3) & 1) << 5) + (k & 31)) * 8 + (j & 7);
                c_frag[pos] = lp;
                const float f = lp_to_float(lp, bf);
                nrm[j] = __fmul_rn(f, f);
            }
        }
    }
    if (tid == 0) counts[(size_t)b * K + k] = n;
    if (normalise && c_frag) {
        __syncthreads();
        // same association as the stand-alone layout kernel: groups of 8 features first (one
        // thread per group; the first wave holds them all, d <= 512), then the groups in order
        if (tid < 64) {
            float ss = 0.f;
            if (tid * 8 < d) {
                for (int e = 0; e < 8; ++e) ss = __fadd_rn(ss, nrm[tid * 8 + e]);
            }
            float n2 = 0.f;
            for (int g0 = 0; g0 * 8 < d; ++g0)
                n2 = __fadd_rn(n2, __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(ss), g0)));
            if (tid == 0) c_bias[((size_t)b * ktiles) * 32 + k] = -0.5f * n2;
        }
    }
}

// ------------------------------------------------------------------------------------
static int ceil_log2(int v) {
    int b = 0;
    while ((1 << b) < v) ++b;
    return b;
}

fk_status launch_segment_reduce(const Geometry& g, const Workspace& w, const void* X,
                                const int32_t* sorted_idx, const int32_t* seg_off,
                                const int32_t* item_off, hipStream_t s) {
    const int epl = g.t == FK_F32 ? 4 : 8;
    int lpr_log2 = ceil_log2((int)cdiv(g.d, epl));
    if (lpr_log2 > 6) lpr_log2 = 6;          // wider rows go column block by column block
    const bool wide = g.waves_per_item == 4;
    dim3 grid((unsigned)(wide ? g.max_items : cdiv(g.max_items, 4)), g.B), block(256);
#define FK_REDUCE(EPL, BF)                                                                        \
    do {                                                                                          \
        if (wide)                                                                                 \
            hipLaunchKernelGGL((segment_reduce_kernel<EPL, BF, 4>), grid, block, 0, s, X,         \
                               sorted_idx, seg_off, item_off, w.partial, g.N, g.d, g.K,           \
                               g.rows_per_item, g.max_items, lpr_log2);                           \
        else                                                                                      \
            hipLaunchKernelGGL((segment_reduce_kernel<EPL, BF, 1>), grid, block, 0, s, X,         \
                               sorted_idx, seg_off, item_off, w.partial, g.N, g.d, g.K,           \
                               g.rows_per_item, g.max_items, lpr_log2);                           \
    } while (0)
    if (g.t == FK_F32) FK_REDUCE(4, false);
    else if (g.t == FK_F16) FK_REDUCE(8, false);
    else FK_REDUCE(8, true);
#undef FK_REDUCE
    FK_HIP(hipGetLastError());
    return FK_OK;
}

fk_status launch_finalize(const Geometry& g, const Workspace& w, const int32_t* seg_off,
                          const int32_t* item_off, const FinalizeArgs& a, hipStream_t s,
                          const int32_t* wg_counts, int wg_per_cluster) {
    uint16_t* lp16 = g.t == FK_F32 ? nullptr : (uint16_t*)a.C_out_lp;
    float* lp32 = g.t == FK_F32 ? (float*)a.C_out_lp : nullptr;
    if (lp32 == a.C_out_f32) lp32 = nullptr;
    uint16_t* frag = g.t == FK_F32 ? nullptr : (uint16_t*)a.c_frag;
    // few clusters with many partial rows each: more rows in flight per workgroup
    // ... and many clusters with few rows each (up to 4, or up to 8 when there are thousands of
    // clusters to spread over the chip): the smallest workgroup that still has a thread per feature
    int threads = g.max_items / g.K > 64 ? 1024 : 256;
    if (g.d <= 128 && (g.max_items / g.K <= 4 || (g.max_items / g.K <= 8 && (int64_t)g.K * g.B >= 4096))) threads = 64;
    const size_t lds = ((size_t)4 * threads + g.d) * sizeof(float);
    hipLaunchKernelGGL(finalize_kernel, dim3(g.K, g.B), dim3(threads), lds, s, w.partial, seg_off,
                       item_off, a.C_prev_f32, a.C_out_f32, lp16, lp32, frag, a.c_bias, a.counts,
                       a.sums, g.d, g.K, g.max_items, g.ktiles, g.dchunks, a.accumulate ? 1 : 0,
                       a.normalise ? 1 : 0, g.t == FK_BF16 ? 1 : 0, wg_counts, wg_per_cluster);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

}  // namespace fk
