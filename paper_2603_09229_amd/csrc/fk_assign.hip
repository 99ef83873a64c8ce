// Assignment stage: fused distance + online argmin (paper Section 4.1, Algorithm 2).
//
// 16-bit inputs: the argmin of ||x - c_k||^2 equals the argmax of x.c_k - ||c_k||^2 / 2
// (norm expansion of Section 3.1 with the row-constant ||x||^2 dropped).  A wave owns
// P*32 points whose features stay in registers as MFMA B-operands for the whole sweep;
// centroid tiles (32 rows) stream through a double-buffered LDS stage as A-operands, so
// that in the 32x32 result every lane holds 16 candidate centroids of ONE point and the
// running (best score, index) pair of Algorithm 2 lives in that lane's registers.  The
// two lanes that share a point merge once, at the end, with a wavefront shuffle.
// The N x K score matrix exists only in accumulator registers.
//
// fp32 inputs: plain fp32 direct differences, one point per thread, centroid tiles in LDS.
#include "fk_common.h"

namespace fk {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float lp_to_float(uint16_t v, bool bf) {
    return bf ? __uint_as_float((uint32_t)v << 16) : (float)__builtin_bit_cast(_Float16, v);
}

// round-to-nearest-even from fp32 (finite input)
__device__ __forceinline__ uint16_t float_to_lp(float f, bool bf) {
    if (bf) {
        uint32_t u = __float_as_uint(f);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

// ------------------------------------------------------------------------------------
// Centroid layout kernel.  One workgroup per centroid tile (32 rows).  Thread g < 64*DCH
// owns the 8-feature group (row r = g%32, half h = (g/32)%2, chunk s = g/64).
//   SRC_F32: source is the fp32 master (rounded here, and written to C_lp if non-NULL);
//   else the source is already the 16-bit array.
// Writes the fragment-ordered copy and bias[k] = -||c_k||^2 / 2 computed in fp32 from the
// ROUNDED values, i.e. from exactly what the MFMA multiplies (-inf for rows >= K).
template <bool SRC_F32>
__global__ __launch_bounds__(512) void centroid_layout_kernel(
    const void* __restrict__ src, uint16_t* __restrict__ C_lp, uint16_t* __restrict__ c_frag,
    float* __restrict__ c_bias, int d, int K, int ktiles, int dch, int bf) {
    __shared__ float part[32][17];
    const int b = blockIdx.y, kt = blockIdx.x;
    const int g = threadIdx.x;
    const int l = g & 63, s = g >> 6, r = l & 31, h = l >> 5;
    const int k = kt * 32 + r, j0 = s * 16 + h * 8;
    if (s < dch) {
        uint16_t v[8];
        float ss = 0.f;
        const bool live = (k < K) && (j0 < d);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0;
        if (live) {
            const size_t o = ((size_t)b * K + k) * d + j0;
            if (SRC_F32) {
                const float* p = (const float*)src + o;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = float_to_lp(p[e], bf);
                if (C_lp) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) C_lp[o + e] = v[e];
                }
            } else {
                const uint16_t* p = (const uint16_t*)src + o;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = p[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float f = lp_to_float(v[e], bf);
                ss += f * f;
            }
        }
        uint16_t* q = c_frag + ((((size_t)b * ktiles + kt) * dch + s) * 64 + l) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = v[e];
        part[r][s * 2 + h] = ss;
    }
    __syncthreads();
    if (g < 32) {
        float n2 = 0.f;
        for (int q = 0; q < dch * 2; ++q) n2 += part[g][q];   // fixed order
        const int kk = kt * 32 + g;
        c_bias[((size_t)b * ktiles + kt) * 32 + g] = kk < K ? -0.5f * n2 : -INFINITY;
    }
}

fk_status launch_prepare_centroids(const Geometry& g, const void* C_lp, void* c_frag,
                                   float* c_bias, hipStream_t s) {
    dim3 grid(g.ktiles, g.B), block(64 * g.dchunks);
    hipLaunchKernelGGL(centroid_layout_kernel<false>, grid, block, 0, s, C_lp, (uint16_t*)nullptr,
                       (uint16_t*)c_frag, c_bias, g.d, g.K, g.ktiles, g.dchunks,
                       g.t == FK_BF16 ? 1 : 0);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

__global__ void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

fk_status launch_round_centroids(const Geometry& g, const float* C_f32, void* C_lp,
                                 void* c_frag, float* c_bias, hipStream_t s) {
    if (g.t == FK_F32) {
        if (C_lp && C_lp != (const void*)C_f32) {
            const size_t n = (size_t)g.B * g.K * g.d;
            hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s,
                               C_f32, (float*)C_lp, n);
            FK_HIP(hipGetLastError());
        }
        return FK_OK;
    }
    dim3 grid(g.ktiles, g.B), block(64 * g.dchunks);
    hipLaunchKernelGGL(centroid_layout_kernel<true>, grid, block, 0, s, (const void*)C_f32,
                       (uint16_t*)C_lp, (uint16_t*)c_frag, c_bias, g.d, g.K, g.ktiles, g.dchunks,
                       g.t == FK_BF16 ? 1 : 0);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

// ------------------------------------------------------------------------------------
template <bool BF>
__device__ __forceinline__ floatx16 mfma32(uintx4 a, uintx4 b, floatx16 c) {
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a),
                                                      __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// BF: bf16 (else fp16).  DCH: feature chunks of 16 held per point.  P: 32-point tiles per
// wave.  WAVES: waves per workgroup.  ST: centroid tiles per LDS stage.
template <bool BF, int DCH, int P, int WAVES, int ST>
__global__ __launch_bounds__(WAVES * 64) void assign_mfma_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int ktiles) {
    constexpr int kThreads = WAVES * 64;
    constexpr int kStageVec = ST * DCH * 64;            // 16-byte vectors per stage
    constexpr int kLoads = (kStageVec + kThreads - 1) / kThreads;
    __shared__ uintx4 sfrag[2][kStageVec];
    __shared__ float sbias[2][ST * 32];

    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    c_frag += (size_t)b * ktiles * DCH * 64;
    c_bias += (size_t)b * ktiles * 32;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int64_t p0 = ((int64_t)blockIdx.x * WAVES + wave) * (P * 32);

    // Point features: lane (n,h) keeps features [s*16 + h*8, +8) of point p0 + pt*32 + n.
    uintx4 xf[P][DCH];
#pragma unroll
    for (int pt = 0; pt < P; ++pt) {
        const int64_t point = p0 + pt * 32 + n;
#pragma unroll
        for (int s = 0; s < DCH; ++s) {
            const int j0 = s * 16 + h * 8;
            uintx4 v = {0u, 0u, 0u, 0u};
            if (point < N && j0 < d) v = *(const uintx4*)(X + (size_t)point * d + j0);
            xf[pt][s] = v;
        }
    }

    float best[P];
    int enc[P];   // tile * 16 + accumulator slot of the best score so far
#pragma unroll
    for (int pt = 0; pt < P; ++pt) { best[pt] = -INFINITY; enc[pt] = 0; }

    const int nstages = (ktiles + ST - 1) / ST;
    const int total_vec = ktiles * DCH * 64;
    uintx4 pre[kLoads];
    float pre_bias = 0.f;

    auto fetch = [&](int st) {
        const int base = st * kStageVec;
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int o = q * kThreads + tid;
            uintx4 v = {0u, 0u, 0u, 0u};
            if (o < kStageVec && base + o < total_vec) v = c_frag[base + o];
            pre[q] = v;
        }
        if (tid < ST * 32) {
            const int o = st * ST * 32 + tid;
            pre_bias = o < ktiles * 32 ? c_bias[o] : -INFINITY;
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int o = q * kThreads + tid;
            if (o < kStageVec) sfrag[buf][o] = pre[q];
        }
        if (tid < ST * 32) sbias[buf][tid] = pre_bias;
    };

    fetch(0);
    commit(0);
    __syncthreads();

    for (int st = 0; st < nstages; ++st) {
        const int buf = st & 1;
        if (st + 1 < nstages) fetch(st + 1);          // overlaps the MFMA sweep below
        const int nt = min(ST, ktiles - st * ST);
        for (int tt = 0; tt < nt; ++tt) {
            floatx16 acc[P];
            // accumulator slot i is centroid row 8*(i/4) + 4*h + i%4 of this tile
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 bv = *(const floatx4*)&sbias[buf][tt * 32 + 8 * q + 4 * h];
#pragma unroll
                for (int pt = 0; pt < P; ++pt) {
                    acc[pt][4 * q + 0] = bv[0];
                    acc[pt][4 * q + 1] = bv[1];
                    acc[pt][4 * q + 2] = bv[2];
                    acc[pt][4 * q + 3] = bv[3];
                }
            }
#pragma unroll
            for (int s = 0; s < DCH; ++s) {
                const uintx4 a = sfrag[buf][(tt * DCH + s) * 64 + lane];
#pragma unroll
                for (int pt = 0; pt < P; ++pt) acc[pt] = mfma32<BF>(a, xf[pt][s], acc[pt]);
            }
            // online argmax; ascending slot order + strict '>' keeps the lowest row
            const int ebase = (st * ST + tt) * 16;
#pragma unroll
            for (int pt = 0; pt < P; ++pt) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float v = acc[pt][i];
                    if (v > best[pt]) { best[pt] = v; enc[pt] = ebase + i; }
                }
            }
        }
        if (st + 1 < nstages) commit(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int pt = 0; pt < P; ++pt) {
        const int i = enc[pt] & 15;
        int k = (enc[pt] >> 4) * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
        float m = best[pt];
        const float om = __shfl_xor(m, 32);
        const int ok = __shfl_xor(k, 32);
        if (om > m || (om == m && ok < k)) { m = om; k = ok; }
        const int64_t point = p0 + pt * 32 + n;
        float xn = 0.f;
        if (min_dist) {
#pragma unroll
            for (int s = 0; s < DCH; ++s) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t w = xf[pt][s][q];
                    const float lo = lp_to_float((uint16_t)(w & 0xFFFFu), BF);
                    const float hi = lp_to_float((uint16_t)(w >> 16), BF);
                    xn += lo * lo + hi * hi;
                }
            }
            xn += __shfl_xor(xn, 32);
        }
        if (h == 0 && point < N) {
            assign[point] = k;
            if (min_dist) min_dist[point] = fmaxf(0.f, xn - 2.f * m);
        }
    }
}

// ------------------------------------------------------------------------------------
// fp32: one point per thread, features in registers, centroid tiles of TK rows in LDS,
// D_ik by direct differences in fp32; ascending k with strict '<'.
template <int DMAX, int TK>
__global__ __launch_bounds__(256) void assign_f32_kernel(
    const float* __restrict__ X, const float* __restrict__ C, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K) {
    __shared__ float sc[TK][DMAX];
    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    C += (size_t)b * K * d;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float x[DMAX];
#pragma unroll
    for (int j = 0; j < DMAX; j += 4) {
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (i < N && j < d) v = *(const floatx4*)(X + (size_t)i * d + j);
        x[j] = v[0]; x[j + 1] = v[1]; x[j + 2] = v[2]; x[j + 3] = v[3];
    }
    float m = INFINITY;
    int a = 0;
    for (int k0 = 0; k0 < K; k0 += TK) {
        __syncthreads();
        for (int o = threadIdx.x; o < TK * DMAX; o += 256) {
            const int r = o / DMAX, j = o % DMAX;
            sc[r][j] = (k0 + r < K && j < d) ? C[(size_t)(k0 + r) * d + j] : 0.f;
        }
        __syncthreads();
        const int nk = min(TK, K - k0);
        for (int r = 0; r < nk; ++r) {
            float D = 0.f;
#pragma unroll
            for (int j = 0; j < DMAX; j += 4) {
                const floatx4 c = *(const floatx4*)&sc[r][j];
                const float e0 = x[j] - c[0], e1 = x[j + 1] - c[1];
                const float e2 = x[j + 2] - c[2], e3 = x[j + 3] - c[3];
                D += e0 * e0; D += e1 * e1; D += e2 * e2; D += e3 * e3;
            }
            if (D < m) { m = D; a = k0 + r; }
        }
    }
    if (i < N) {
        assign[i] = a;
        if (min_dist) min_dist[i] = m;
    }
}

// ------------------------------------------------------------------------------------
template <bool BF, int DCH>
static fk_status launch_mfma(const Geometry& g, const void* X, const void* frag,
                             const float* bias, int32_t* assign, float* min_dist,
                             hipStream_t s) {
    constexpr int P = 2, WAVES = 4, ST = 16 / DCH;   // 16 KiB of fragments per stage
    const int64_t per_wg = (int64_t)P * 32 * WAVES;
    dim3 grid((unsigned)cdiv(g.N, per_wg), g.B), block(WAVES * 64);
    hipLaunchKernelGGL((assign_mfma_kernel<BF, DCH, P, WAVES, ST>), grid, block, 0, s,
                       (const uint16_t*)X, (const uintx4*)frag, bias, assign, min_dist, g.N,
                       g.d, g.ktiles);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

template <bool BF>
static fk_status launch_mfma_d(const Geometry& g, const void* X, const void* frag,
                               const float* bias, int32_t* assign, float* min_dist,
                               hipStream_t s) {
    switch (g.dchunks) {
        case 2: return launch_mfma<BF, 2>(g, X, frag, bias, assign, min_dist, s);
        case 4: return launch_mfma<BF, 4>(g, X, frag, bias, assign, min_dist, s);
        case 8: return launch_mfma<BF, 8>(g, X, frag, bias, assign, min_dist, s);
    }
    set_error("assign: no kernel for %d feature chunks", g.dchunks);
    return FK_EUNSUPPORTED;
}

fk_status launch_assign(const Geometry& g, const void* X, const void* C_or_frag,
                        const float* c_bias, int32_t* assign, float* min_dist, hipStream_t s) {
    if (g.t == FK_F16) return launch_mfma_d<false>(g, X, C_or_frag, c_bias, assign, min_dist, s);
    if (g.t == FK_BF16) return launch_mfma_d<true>(g, X, C_or_frag, c_bias, assign, min_dist, s);
    dim3 grid((unsigned)cdiv(g.N, 256), g.B), block(256);
    const float* Xf = (const float*)X;
    const float* Cf = (const float*)C_or_frag;
    if (g.d <= 32)
        hipLaunchKernelGGL((assign_f32_kernel<32, 32>), grid, block, 0, s, Xf, Cf, assign, min_dist, g.N, g.d, g.K);
    else if (g.d <= 64)
        hipLaunchKernelGGL((assign_f32_kernel<64, 32>), grid, block, 0, s, Xf, Cf, assign, min_dist, g.N, g.d, g.K);
    else
        hipLaunchKernelGGL((assign_f32_kernel<128, 32>), grid, block, 0, s, Xf, Cf, assign, min_dist, g.N, g.d, g.K);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

}  // namespace fk
