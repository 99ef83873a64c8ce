// The "standard" k-means iteration the paper starts from (Section 3.1, Algorithm 1), built
// only as a comparator: a distance kernel that WRITES the N x K matrix D to HBM, a row-argmin
// kernel that reads it back, a per-point atomic scatter of features and counts, and a
// normalisation kernel.  It exists to reproduce, on this machine, the two kernel-level
// comparisons of the paper's Section 5.2 (fused assign vs materialised distances; sort-inverse
// update vs atomic scatter).  Nothing in the fast path calls into this file.
//
// The distance kernel is a reasonable MFMA kernel, not a strawman: same operand layout,
// LDS staging and tile shape as the fused kernel, with the argmin epilogue replaced by
// stores of ||x||^2 - 2(x.c - ||c||^2/2).  16-bit storage types, d <= 128.
#include "fk_common.h"
#include "fk_device.h"

namespace fk {

// Kernel 1 of Algorithm 1: D[i][k] = ||x_i||^2 + ||c_k||^2 - 2 x_i.c_k, written to HBM.
// 8 waves x 64 points per workgroup; centroid tiles staged through LDS (16 KiB stages).
template <bool BF, int DCH, int ST>
__global__ __launch_bounds__(512) void std_distance_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, float* __restrict__ D, int64_t N, int d, int K,
    int ktiles) {
    constexpr int WAVES = 8, P = 2, kThreads = 512;
    constexpr int kStageVec = ST * DCH * 64;
    constexpr int kLoads = (kStageVec + kThreads - 1) / kThreads;
    __shared__ uintx4 sfrag[2][kStageVec];
    __shared__ float sbias[2][ST * 32];
    __shared__ float sxn[WAVES][P * 32];          // ||x||^2 of the wave's points
    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    c_frag += (size_t)b * ktiles * DCH * 64;
    c_bias += (size_t)b * ktiles * 32;
    D += (size_t)b * N * K;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int64_t p0 = ((int64_t)blockIdx.x * WAVES + wave) * (P * 32);
    const int total_vec = ktiles * DCH * 64;

    uintx4 xf[P][DCH];
    float xn[P];
#pragma unroll
    for (int pt = 0; pt < P; ++pt) {
        const int64_t point = p0 + pt * 32 + n;
        float acc = 0.f;
#pragma unroll
        for (int s = 0; s < DCH; ++s) {
            const int j0 = s * 16 + h * 8;
            uintx4 v = {0u, 0u, 0u, 0u};
            if (point < N && j0 < d) v = *(const uintx4*)(X + (size_t)point * d + j0);
            xf[pt][s] = v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float lo = lp_to_float((uint16_t)(v[q] & 0xFFFFu), BF);
                const float hi = lp_to_float((uint16_t)(v[q] >> 16), BF);
                acc += lo * lo + hi * hi;
            }
        }
        xn[pt] = acc + __shfl_xor(acc, 32);
        if (h == 0) sxn[wave][pt * 32 + n] = xn[pt];
    }

    auto stage_in = [&](int st, int buf) {
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int o = q * kThreads + tid;
            if (o < kStageVec) {
                uintx4 v = {0u, 0u, 0u, 0u};
                if (st * kStageVec + o < total_vec) v = c_frag[st * kStageVec + o];
                sfrag[buf][o] = v;
            }
        }
        if (tid < ST * 32) {
            const int o = st * ST * 32 + tid;
            sbias[buf][tid] = o < ktiles * 32 ? c_bias[o] : 0.f;
        }
    };
    const int nstages = (ktiles + ST - 1) / ST;
    stage_in(0, 0);
    __syncthreads();
    for (int st = 0; st < nstages; ++st) {
        const int buf = st & 1;
        if (st + 1 < nstages) stage_in(st + 1, buf ^ 1);
        const int nt = min(ST, ktiles - st * ST);
        for (int tt = 0; tt < nt; ++tt) {
            // Points on the MFMA row side, centroids on the column side: accumulator slot i
            // is point row 8*(i/4) + 4*h + i%4 of the tile and the lane's column is centroid
            // lane%32, so every store instruction below writes whole 128-byte runs of D.
            const float cb = sbias[buf][tt * 32 + n];
            floatx16 bias16;
#pragma unroll
            for (int i = 0; i < 16; ++i) bias16[i] = cb;
            floatx16 acc[P];
#pragma unroll
            for (int pt = 0; pt < P; ++pt)
                acc[pt] = mfma32<BF>(xf[pt][0], sfrag[buf][(tt * DCH) * 64 + lane], bias16);
#pragma unroll
            for (int s = 1; s < DCH; ++s) {
                const uintx4 a = sfrag[buf][(tt * DCH + s) * 64 + lane];
#pragma unroll
                for (int pt = 0; pt < P; ++pt) acc[pt] = mfma32<BF>(xf[pt][s], a, acc[pt]);
            }
            const int k = (st * ST + tt) * 32 + n;
#pragma unroll
            for (int pt = 0; pt < P; ++pt) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 x2 = *(const floatx4*)&sxn[wave][pt * 32 + 8 * q + 4 * h];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int64_t point = p0 + pt * 32 + 8 * q + 4 * h + r;
                        if (point < N && k < K)
                            D[(size_t)point * K + k] = fmaxf(0.f, x2[r] - 2.f * acc[pt][4 * q + r]);
                    }
                }
            }
        }
        __syncthreads();
    }
}

// Kernel 2 of Algorithm 1: a_i = argmin_k D[i][k] (lowest k on ties); one wave per row.
__global__ __launch_bounds__(256) void std_argmin_kernel(const float* __restrict__ D,
                                                         int32_t* __restrict__ assign,
                                                         int64_t rows, int K) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* p = D + (size_t)row * K;
    float m = INFINITY;
    int a = 0x7FFFFFFF;
    if ((K & 3) == 0) {
        // 16 bytes per lane, four loads in flight
        for (int k0 = lane * 4; k0 < K; k0 += 1024) {
            floatx4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = k0 + u * 256;
                v[u] = k < K ? *(const floatx4*)(p + k) : floatx4{INFINITY, INFINITY, INFINITY, INFINITY};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = k0 + u * 256 + e;
                    if (v[u][e] < m || (v[u][e] == m && k < a)) { m = v[u][e]; a = k; }
                }
            }
        }
    } else {
        for (int k = lane; k < K; k += 64) {
            const float v = p[k];
            if (v < m) { m = v; a = k; }
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float om = __shfl_xor(m, o);
        const int oa = __shfl_xor(a, o);
        if (om < m || (om == m && oa < a)) { m = om; a = oa; }
    }
    if (lane == 0) assign[row] = min(a, K - 1);
}

// Kernel 3 of Algorithm 1: every point adds its features and a count into its cluster's
// accumulators with atomics (16 bytes of a row per thread).
template <int EPL, bool BF>
__global__ __launch_bounds__(256) void std_scatter_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ assign, float* __restrict__ sums,
    int32_t* __restrict__ counts, int64_t rows_total, int64_t N, int d, int K, int tpr) {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = g / tpr;                      // row index over all instances
    const int col = (int)(g - row * tpr) * EPL;
    if (row >= rows_total || col >= d) return;
    const int64_t b = row / N;
    const int k = min(max(assign[row], 0), K - 1);
    float* s = sums + ((size_t)b * K + k) * d + col;
    const uintx4 v = *(const uintx4*)((const char*)Xv + ((size_t)row * d + col) * (16 / EPL));
    if (EPL == 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) unsafeAtomicAdd(s + e, __uint_as_float(v[e]));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            unsafeAtomicAdd(s + 2 * e, lp_to_float((uint16_t)(v[e] & 0xFFFFu), BF));
            unsafeAtomicAdd(s + 2 * e + 1, lp_to_float((uint16_t)(v[e] >> 16), BF));
        }
    }
    if (col == 0) atomicAdd(counts + (size_t)b * K + k, 1);
}

__global__ void std_zero_kernel(float* __restrict__ sums, int32_t* __restrict__ counts, size_t ns,
                                size_t nc) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < ns) sums[i] = 0.f;
    if (i < nc) counts[i] = 0;
}

// Kernel 4 of Algorithm 1: c_k = s_k / n_k (previous centroid where n_k = 0).
__global__ void std_normalise_kernel(const float* __restrict__ sums,
                                     const int32_t* __restrict__ counts, const float* C_prev,
                                     float* C_out, size_t n, int d) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int c = counts[i / d];
    C_out[i] = c > 0 ? (float)((double)sums[i] / (double)c) : C_prev[i];
}

template <bool BF>
static fk_status launch_distance(const Geometry& g, const void* X, const void* frag,
                                 const float* bias, float* D, hipStream_t s) {
    dim3 grid((unsigned)cdiv(g.N, 512), g.B), block(512);
    switch (g.dchunks) {
        case 2:
            hipLaunchKernelGGL((std_distance_kernel<BF, 2, 8>), grid, block, 0, s, (const uint16_t*)X,
                               (const uintx4*)frag, bias, D, g.N, g.d, g.K, g.ktiles);
            break;
        case 4:
            hipLaunchKernelGGL((std_distance_kernel<BF, 4, 4>), grid, block, 0, s, (const uint16_t*)X,
                               (const uintx4*)frag, bias, D, g.N, g.d, g.K, g.ktiles);
            break;
        case 8:
            hipLaunchKernelGGL((std_distance_kernel<BF, 8, 2>), grid, block, 0, s, (const uint16_t*)X,
                               (const uintx4*)frag, bias, D, g.N, g.d, g.K, g.ktiles);
            break;
        default:
            set_error("fk_standard_assign: d > 128 is not built for the comparator");
            return FK_EUNSUPPORTED;
    }
    FK_HIP(hipGetLastError());
    return FK_OK;
}

fk_status launch_standard_assign(const Geometry& g, const Workspace& w, const void* X,
                                 const void* C_lp, float* D, int32_t* assign, hipStream_t s) {
    if (g.t == FK_F32) {
        set_error("fk_standard_assign: fp32 storage is not built for the comparator");
        return FK_EUNSUPPORTED;
    }
    fk_status st = launch_prepare_centroids(g, C_lp, w.c_frag, w.c_bias, s);
    if (st != FK_OK) return st;
    st = g.t == FK_BF16 ? launch_distance<true>(g, X, w.c_frag, w.c_bias, D, s)
                        : launch_distance<false>(g, X, w.c_frag, w.c_bias, D, s);
    if (st != FK_OK) return st;
    const int64_t rows = (int64_t)g.B * g.N;
    hipLaunchKernelGGL(std_argmin_kernel, dim3((unsigned)cdiv(rows, 4)), dim3(256), 0, s, D, assign,
                       rows, g.K);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

fk_status launch_standard_update(const Geometry& g, const void* X, const int32_t* assign,
                                 const float* C_prev, float* C_out, int32_t* counts, float* sums,
                                 hipStream_t s) {
    const size_t ns = (size_t)g.B * g.K * g.d, nc = (size_t)g.B * g.K;
    hipLaunchKernelGGL(std_zero_kernel, dim3((unsigned)cdiv(ns, 256)), dim3(256), 0, s, sums, counts,
                       ns, nc);
    FK_HIP(hipGetLastError());
    const int epl = g.t == FK_F32 ? 4 : 8;
    const int tpr = (int)cdiv(g.d, epl);
    const int64_t rows = (int64_t)g.B * g.N;
    dim3 grid((unsigned)cdiv(rows * tpr, 256)), block(256);
    if (g.t == FK_F32)
        hipLaunchKernelGGL((std_scatter_kernel<4, false>), grid, block, 0, s, X, assign, sums, counts,
                           rows, g.N, g.d, g.K, tpr);
    else if (g.t == FK_F16)
        hipLaunchKernelGGL((std_scatter_kernel<8, false>), grid, block, 0, s, X, assign, sums, counts,
                           rows, g.N, g.d, g.K, tpr);
    else
        hipLaunchKernelGGL((std_scatter_kernel<8, true>), grid, block, 0, s, X, assign, sums, counts,
                           rows, g.N, g.d, g.K, tpr);
    FK_HIP(hipGetLastError());
    hipLaunchKernelGGL(std_normalise_kernel, dim3((unsigned)cdiv(ns, 256)), dim3(256), 0, s, sums,
                       counts, C_prev, C_out, ns, g.d);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

}  // namespace fk
