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
#include <stdlib.h>

#include <algorithm>

#include "fk_common.h"
#include "fk_device.h"

namespace fk {

// ------------------------------------------------------------------------------------
// Centroid layout kernel.  One workgroup per centroid tile (32 rows).  Thread g < 64*DCH
// owns the 8-feature group (row r = g%32, half h = (g/32)%2, chunk s = g/64).
//   SRC_F32: source is the fp32 master (rounded here, and written to C_lp if non-NULL);
//   else the source is already the 16-bit array.
// Writes the fragment-ordered copy and bias[k] = -||c_k||^2 / 2 computed in fp32 from the
// ROUNDED values, i.e. from exactly what the MFMA multiplies.  Rows >= K get a huge negative
// finite bias: it must survive having its low mantissa bits overwritten (-inf would turn
// into a NaN pattern) and still lose against every real score.
template <bool SRC_F32>
__global__ __launch_bounds__(512) void centroid_layout_kernel(
    const void* __restrict__ src, uint16_t* __restrict__ C_lp, uint16_t* __restrict__ c_frag,
    float* __restrict__ c_bias, int d, int K, int ktiles, int dch, int bf) {
    __shared__ float part[32][65];
    const int b = blockIdx.y, kt = blockIdx.x;
    for (int g = threadIdx.x; g < 64 * dch; g += blockDim.x) {
        const int l = g & 63, s = g >> 6, r = l & 31, h = l >> 5;
        const int k = kt * 32 + r, j0 = s * 16 + h * 8;
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
                ss = __fadd_rn(ss, __fmul_rn(f, f));   // no FMA: the update kernel repeats this sum bit for bit
            }
        }
        uint16_t* q = c_frag + ((((size_t)b * ktiles + kt) * dch + s) * 64 + l) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = v[e];
        part[r][s * 2 + h] = ss;
    }
    __syncthreads();
    if (threadIdx.x < 32) {
        const int g = threadIdx.x;
        float n2 = 0.f;
        for (int q = 0; q < dch * 2; ++q) n2 = __fadd_rn(n2, part[g][q]);   // fixed order
        const int kk = kt * 32 + g;
        c_bias[((size_t)b * ktiles + kt) * 32 + g] = kk < K ? -0.5f * n2 : kPadBias;
    }
}

fk_status launch_prepare_centroids(const Geometry& g, const void* C_lp, void* c_frag,
                                   float* c_bias, hipStream_t s) {
    dim3 grid(g.ktiles, g.B), block(std::min(512, 64 * g.dchunks));
    hipLaunchKernelGGL(centroid_layout_kernel<false>, grid, block, 0, s, C_lp, (uint16_t*)nullptr,
                       (uint16_t*)c_frag, c_bias, g.d, g.K, g.ktiles, g.dchunks,
                       g.t == FK_BF16 ? 1 : 0);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

// dst[r][j] = j < d_src ? src[r][j] : 0 for j < d_dst: pads rows with zeros (d_dst > d_src) or
// drops the padding again (d_dst < d_src)
template <typename T>
__global__ void copy_rows_kernel(const T* __restrict__ src, T* __restrict__ dst, size_t total,
                                 int d_src, int d_dst) {
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (size_t)gridDim.x * blockDim.x) {
        const size_t r = o / (size_t)d_dst;
        const int j = (int)(o - r * (size_t)d_dst);
        dst[o] = j < d_src ? src[r * (size_t)d_src + j] : T(0);
    }
}

fk_status launch_copy_rows(const void* src, void* dst, int64_t rows, int d_src, int d_dst,
                           int elem, hipStream_t s) {
    const size_t total = (size_t)rows * d_dst;
    const unsigned blocks = (unsigned)std::min<size_t>(cdiv((int64_t)total, 256), (size_t)1 << 20);
    if (elem == 2)
        hipLaunchKernelGGL(copy_rows_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s,
                           (const uint16_t*)src, (uint16_t*)dst, total, d_src, d_dst);
    else
        hipLaunchKernelGGL(copy_rows_kernel<uint32_t>, dim3(blocks), dim3(256), 0, s,
                           (const uint32_t*)src, (uint32_t*)dst, total, d_src, d_dst);
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
    dim3 grid(g.ktiles, g.B), block(std::min(512, 64 * g.dchunks));
    hipLaunchKernelGGL(centroid_layout_kernel<true>, grid, block, 0, s, (const void*)C_f32,
                       (uint16_t*)C_lp, (uint16_t*)c_frag, c_bias, g.d, g.K, g.ktiles, g.dchunks,
                       g.t == FK_BF16 ? 1 : 0);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

// ------------------------------------------------------------------------------------
// Direct global -> LDS copy of 16 bytes per lane: the wave's 64 lanes fill 1 KiB starting
// at the (wave-uniform) LDS address `lds_base`, lane i at lds_base + 16*i.
__device__ __forceinline__ void copy16_to_lds(const uintx4* gsrc, uintx4* lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// BF: bf16 (else fp16).  DCH: feature chunks of 16 held per point.  P: 32-point tiles per
// wave.  WAVES: waves per workgroup.  ST: centroid tiles per LDS stage.
//
// Score bookkeeping.  The fp32 score of a (point, centroid) pair leaves the MFMA with the
// -||c||^2/2 bias already added (the bias enters as the C operand of the first MFMA of the
// chain).  Its low 4 mantissa bits are then replaced by 15 - slot, slot being the
// accumulator index, so that ONE float max carries value and slot together: 1.5 VALU
// operations per pair instead of 3, which is what keeps the epilogue off the MFMA's
// critical path.  The truncation costs 2^-19 relative to the score, the same order as the
// fp32 rounding of a d-term dot product and ~250x below the 1e-3 tolerance band.
// Ties between scores equal after truncation: the earlier centroid tile wins; inside a tile
// the lower row wins for scores >= 0 (the usual case for a winner: x.c > ||c||^2/2), the
// higher row among the lane's 16 for negative ones.
template <bool BF, int DCH, int P, int WAVES, int ST>
__global__ __launch_bounds__(WAVES * 64) void assign_mfma_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K, int ktiles) {
    constexpr int kThreads = WAVES * 64;
    constexpr int kStageVec = ST * DCH * 64;            // 16-byte vectors per stage
    constexpr int kPieces = ST * DCH;                   // 1 KiB pieces per stage
    __shared__ uintx4 sfrag[2][kStageVec];
    __shared__ float sbias[2][ST * 32];
    static_assert(ST * 32 <= kThreads, "one bias value per thread per stage");

    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    c_frag += (size_t)b * ktiles * DCH * 64;
    c_bias += (size_t)b * ktiles * 32;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int64_t p0 = ((int64_t)blockIdx.x * WAVES + wave) * (P * 32);

    const int nstages = (ktiles + ST - 1) / ST;
    const int total_pieces = ktiles * DCH;

    // Stage copy: centroid fragments go global -> LDS without passing through registers;
    // the 32 bias values per tile take the ordinary path (one float per thread).
    auto fetch = [&](int st, int buf) -> float {
#pragma unroll
        for (int q = 0; q < (kPieces + WAVES - 1) / WAVES; ++q) {
            const int pc = q * WAVES + wave;                       // wave-uniform
            if (pc < kPieces && st * kPieces + pc < total_pieces)
                copy16_to_lds(c_frag + ((size_t)(st * kPieces + pc) * 64 + lane),
                              &sfrag[buf][pc * 64]);
        }
        float bv = kPadBias;
        if (tid < ST * 32) {
            const int o = st * ST * 32 + tid;
            if (o < ktiles * 32) bv = c_bias[o];
        }
        return bv;
    };

    float pre_bias = fetch(0, 0);

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

    float best[P];   // packed: score with low 4 bits = 15 - slot
    int btile[P];    // centroid tile of the best score so far
#pragma unroll
    for (int pt = 0; pt < P; ++pt) { best[pt] = -INFINITY; btile[pt] = 0; }

    if (tid < ST * 32) sbias[0][tid] = pre_bias;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int st = 0; st < nstages; ++st) {
        const int buf = st & 1;
        if (st + 1 < nstages) pre_bias = fetch(st + 1, buf ^ 1);   // lands during the sweep
        const int nt = min(ST, ktiles - st * ST);
        for (int tt = 0; tt < nt; ++tt) {
            // accumulator slot i is centroid row 8*(i/4) + 4*h + i%4 of this tile
            floatx16 bias16;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 bv = *(const floatx4*)&sbias[buf][tt * 32 + 8 * q + 4 * h];
                bias16[4 * q + 0] = bv[0];
                bias16[4 * q + 1] = bv[1];
                bias16[4 * q + 2] = bv[2];
                bias16[4 * q + 3] = bv[3];
            }
            uintx4 a[DCH];
#pragma unroll
            for (int s = 0; s < DCH; ++s) a[s] = sfrag[buf][(tt * DCH + s) * 64 + lane];
            floatx16 acc[P];
#pragma unroll
            for (int pt = 0; pt < P; ++pt) acc[pt] = mfma32<BF>(a[0], xf[pt][0], bias16);
#pragma unroll
            for (int s = 1; s < DCH; ++s) {
#pragma unroll
                for (int pt = 0; pt < P; ++pt) acc[pt] = mfma32<BF>(a[s], xf[pt][s], acc[pt]);
            }
            const int tile = st * ST + tt;
#pragma unroll
            for (int pt = 0; pt < P; ++pt) {
                // The running best enters the tile with its slot field set so that an equal
                // truncated score cannot displace it (all ones for a positive float, zeros
                // for a negative one): across tiles only a strictly better score wins.
                const uint32_t bb = __float_as_uint(best[pt]);
                const uint32_t fill = ~(uint32_t)((int32_t)bb >> 31) & 15u;
                const float guard = __uint_as_float((bb & 0xFFFFFFF0u) | fill);
                float m = guard;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float k0 = __uint_as_float((__float_as_uint(acc[pt][i]) & 0xFFFFFFF0u) | (uint32_t)(15 - i));
                    const float k1 = __uint_as_float((__float_as_uint(acc[pt][i + 1]) & 0xFFFFFFF0u) | (uint32_t)(14 - i));
                    m = __builtin_fmaxf(__builtin_fmaxf(m, k0), k1);
                }
                const bool improved = m != guard;
                best[pt] = improved ? m : best[pt];
                btile[pt] = improved ? tile : btile[pt];
            }
        }
        if (st + 1 < nstages) {
            if (tid < ST * 32) sbias[buf ^ 1][tid] = pre_bias;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
    }

#pragma unroll
    for (int pt = 0; pt < P; ++pt) {
        const uint32_t bits = __float_as_uint(best[pt]);
        const int i = 15 - (int)(bits & 15u);
        int k = btile[pt] * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
        float m = __uint_as_float(bits & 0xFFFFFFF0u);
        const float om = __shfl_xor(m, 32);
        const int ok = __shfl_xor(k, 32);
        if (om > m || (om == m && ok < k)) { m = om; k = ok; }
        k = min(k, K - 1);   // only reachable with non-finite input; keeps the index in range
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
// Wide features (128 < d <= 512; DCH = 16 or 32 chunks of 16).  Same sweep as above with one
// 32-point tile per wave, so that a point's features still fit the register file (4*DCH
// VGPRs), and LDS stages of 16 chunks: a whole centroid tile per stage for DCH = 16, half a
// tile for DCH = 32 (the MFMA chain of a tile then runs across two stages).
template <bool BF, int DCH, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void assign_mfma_wide_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K, int ktiles) {
    constexpr int SC = 16;                  // chunks (1 KiB pieces) per stage
    constexpr int SPT = DCH / SC;           // stages per centroid tile
    constexpr int kThreads = WAVES * 64;
    static_assert(DCH % SC == 0 && SC % WAVES == 0 && kThreads >= 32, "stage geometry");
    __shared__ uintx4 sfrag[2][SC * 64];
    __shared__ float sbias[2][32];

    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    c_frag += (size_t)b * ktiles * DCH * 64;
    c_bias += (size_t)b * ktiles * 32;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int64_t point = ((int64_t)blockIdx.x * WAVES + wave) * 32 + n;
    const int nst = ktiles * SPT;

    auto fetch = [&](int st, int buf) -> float {
#pragma unroll
        for (int q = 0; q < SC / WAVES; ++q) {
            const int pc = q * WAVES + wave;                       // wave-uniform
            copy16_to_lds(c_frag + ((size_t)(st * SC + pc) * 64 + lane), &sfrag[buf][pc * 64]);
        }
        float bv = kPadBias;
        if (tid < 32) bv = c_bias[(st / SPT) * 32 + tid];
        return bv;
    };

    float pre_bias = fetch(0, 0);
    uintx4 xf[DCH];
#pragma unroll
    for (int s = 0; s < DCH; ++s) {
        const int j0 = s * 16 + h * 8;
        uintx4 v = {0u, 0u, 0u, 0u};
        if (point < N && j0 < d) v = *(const uintx4*)(X + (size_t)point * d + j0);
        xf[s] = v;
    }
    float best = -INFINITY;
    int btile = 0;
    if (tid < 32) sbias[0][tid] = pre_bias;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    floatx16 acc;
    for (int st0 = 0; st0 < nst; st0 += SPT) {
#pragma unroll
        for (int half = 0; half < SPT; ++half) {
            const int st = st0 + half;
            const int buf = st & 1;
            if (st + 1 < nst) pre_bias = fetch(st + 1, buf ^ 1);   // lands during the sweep
            if (half == 0) {
                // accumulator slot i is centroid row 8*(i/4) + 4*h + i%4 of this tile
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 bv = *(const floatx4*)&sbias[buf][8 * q + 4 * h];
                    acc[4 * q + 0] = bv[0];
                    acc[4 * q + 1] = bv[1];
                    acc[4 * q + 2] = bv[2];
                    acc[4 * q + 3] = bv[3];
                }
            }
#pragma unroll
            for (int s = 0; s < SC; ++s)
                acc = mfma32<BF>(sfrag[buf][s * 64 + lane], xf[half * SC + s], acc);
            if (half == SPT - 1) {
                const uint32_t bb = __float_as_uint(best);
                const uint32_t fill = ~(uint32_t)((int32_t)bb >> 31) & 15u;
                const float guard = __uint_as_float((bb & 0xFFFFFFF0u) | fill);
                float m = guard;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float k0 = __uint_as_float((__float_as_uint(acc[i]) & 0xFFFFFFF0u) | (uint32_t)(15 - i));
                    const float k1 = __uint_as_float((__float_as_uint(acc[i + 1]) & 0xFFFFFFF0u) | (uint32_t)(14 - i));
                    m = __builtin_fmaxf(__builtin_fmaxf(m, k0), k1);
                }
                const bool improved = m != guard;
                best = improved ? m : best;
                btile = improved ? st / SPT : btile;
            }
            if (st + 1 < nst) {
                if (tid < 32) sbias[buf ^ 1][tid] = pre_bias;
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            __syncthreads();
        }
    }

    const uint32_t bits = __float_as_uint(best);
    const int i = 15 - (int)(bits & 15u);
    int k = btile * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
    float m = __uint_as_float(bits & 0xFFFFFFF0u);
    const float om = __shfl_xor(m, 32);
    const int ok = __shfl_xor(k, 32);
    if (om > m || (om == m && ok < k)) { m = om; k = ok; }
    k = min(k, K - 1);
    float xnorm = 0.f;
    if (min_dist) {
#pragma unroll
        for (int s = 0; s < DCH; ++s) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t w = xf[s][q];
                const float lo = lp_to_float((uint16_t)(w & 0xFFFFu), BF);
                const float hi = lp_to_float((uint16_t)(w >> 16), BF);
                xnorm += lo * lo + hi * hi;
            }
        }
        xnorm += __shfl_xor(xnorm, 32);
    }
    if (h == 0 && point < N) {
        assign[point] = k;
        if (min_dist) min_dist[point] = fmaxf(0.f, xnorm - 2.f * m);
    }
}

// ------------------------------------------------------------------------------------
// Few centroids (all of C fits one LDS stage, K <= 32 * ST): the work per point is small and
// the kernel is bound by streaming X from HBM.  Persistent waves: C is staged once per
// workgroup, then every wave walks its own sequence of 32-point batches with no further
// barrier.  A batch is copied global -> LDS (direct, no registers) with every load
// instruction covering whole contiguous rows -- the MFMA operand pattern itself would touch
// each 128-byte line four times with 32 bytes used per touch -- into a wave-private ring of
// three LDS buffers (two batches in flight while a third is computed); the
// fragments are then read back from LDS.  The 16-byte pieces of a row are stored XOR-swizzled
// by the row number so that those reads are free of bank conflicts.  Same scores, packing and
// tie rules as the sweeping kernel above.
template <bool BF, int DCH, int WAVES, int KT>
__global__ __launch_bounds__(WAVES * 64) void assign_mfma_stream_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K, int ktiles) {
    constexpr int kThreads = WAVES * 64;
    constexpr int kRows = 32;                          // points per batch
    // The centroid stage lives in its own LDS objects, the batch buffers in the dynamic one:
    // the compiler can then tell that a copy in flight into a batch buffer does not alias the
    // centroid reads, and does not make them wait for it.
    __shared__ uintx4 sfrag[KT * DCH * 64];
    __shared__ float sbias[KT * 32];
    extern __shared__ uintx4 dyn_lds[];                // per wave: a ring of 3 batch buffers
    const int ppr = d >> 3;                            // 16-byte pieces per row
    constexpr int loads = DCH;                         // copy instructions per batch, always all issued
    const int swz = (ppr & (ppr - 1)) == 0 ? min(ppr, 8) - 1 : 0;   // XOR mask for the piece index

    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    c_frag += (size_t)b * ktiles * DCH * 64;
    c_bias += (size_t)b * ktiles * 32;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    uintx4* ring = dyn_lds + (size_t)wave * 3 * loads * 64;

    for (int o = tid; o < ktiles * DCH * 64; o += kThreads) sfrag[o] = c_frag[o];
    for (int o = tid; o < ktiles * 32; o += kThreads) sbias[o] = c_bias[o];

    const int64_t nbatches = (N + kRows - 1) / kRows;
    const int64_t stride = (int64_t)gridDim.x * WAVES;
    int64_t t = (int64_t)blockIdx.x * WAVES + wave;

    // Slot j of the buffer holds piece (j % ppr) ^ (row & swz) of row j / ppr.  Every copy
    // instruction is issued with all lanes live -- slots past the end of the batch or of X
    // re-read the last valid row into buffer space nobody reads -- because the waits below
    // count instructions: one skipped for want of live lanes would let an older copy slip
    // past the wait.
    auto request = [&](int64_t batch, uintx4* buf) {
#pragma unroll
        for (int q = 0; q < loads; ++q) {
            const int j = q * 64 + lane;
            int row = j / ppr;
            const int piece = (j - row * ppr) ^ (row & swz);
            row = min(row, kRows - 1);
            const int64_t point = min(batch * kRows + row, N - 1);
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(X + (size_t)point * d + piece * 8),
                (__attribute__((address_space(3))) void*)(buf + q * 64), 16, 0, 0);
        }
    };

    // Two batches are kept in flight.  Loads of a wave complete in order, so "at most `loads`
    // outstanding" means that everything but the newest batch has landed.
    if (t < nbatches) request(t, ring);
    if (t + stride < nbatches) request(t + stride, ring + loads * 64);
    if (t + stride < nbatches) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(loads) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                       // C is in LDS; no workgroup barrier after this point

    int cur = 0;
    while (t < nbatches) {
        const int64_t t1 = t + stride, t2 = t1 + stride;
        const uintx4* bufc = ring + cur * (loads * 64);
        uintx4* buf2 = ring + (cur == 0 ? 2 : cur - 1) * (loads * 64);   // read one iteration ago

        // This lane's B operands: features [s*16 + h*8, +8) of point t*32 + n.  Read with an
        // opaque LDS instruction: the wait for the copy that filled this buffer was issued by
        // hand above / at the end of the previous iteration, and the compiler must not add a
        // wait for the younger copy still in flight.
        uintx4 xf[DCH];
#pragma unroll
        for (int s = 0; s < DCH; ++s) {
            const int piece = 2 * s + h;
            uintx4 v = {0u, 0u, 0u, 0u};
            if (piece < ppr) {
                const uint32_t addr = (uint32_t)(uintptr_t)(
                    (__attribute__((address_space(3))) const void*)(bufc + n * ppr + (piece ^ (n & swz))));
                asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
            }
            xf[s] = v;
        }
        const bool issued = t2 < nbatches;
        if (issued) request(t2, buf2);

        float best = -INFINITY;
        int btile = 0;
        for (int tt = 0; tt < ktiles; ++tt) {
            floatx16 bias16;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 bv = *(const floatx4*)&sbias[tt * 32 + 8 * q + 4 * h];
                bias16[4 * q + 0] = bv[0];
                bias16[4 * q + 1] = bv[1];
                bias16[4 * q + 2] = bv[2];
                bias16[4 * q + 3] = bv[3];
            }
            floatx16 acc = mfma32<BF>(sfrag[(tt * DCH) * 64 + lane], xf[0], bias16);
#pragma unroll
            for (int s = 1; s < DCH; ++s) acc = mfma32<BF>(sfrag[(tt * DCH + s) * 64 + lane], xf[s], acc);
            const uint32_t bb = __float_as_uint(best);
            const uint32_t fill = ~(uint32_t)((int32_t)bb >> 31) & 15u;
            const float guard = __uint_as_float((bb & 0xFFFFFFF0u) | fill);
            float m = guard;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float k0 = __uint_as_float((__float_as_uint(acc[i]) & 0xFFFFFFF0u) | (uint32_t)(15 - i));
                const float k1 = __uint_as_float((__float_as_uint(acc[i + 1]) & 0xFFFFFFF0u) | (uint32_t)(14 - i));
                m = __builtin_fmaxf(__builtin_fmaxf(m, k0), k1);
            }
            const bool improved = m != guard;
            best = improved ? m : best;
            btile = improved ? tt : btile;
        }
        {
            const uint32_t bits = __float_as_uint(best);
            const int i = 15 - (int)(bits & 15u);
            int k = btile * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            float m = __uint_as_float(bits & 0xFFFFFFF0u);
            const float om = __shfl_xor(m, 32);
            const int ok = __shfl_xor(k, 32);
            if (om > m || (om == m && ok < k)) { m = om; k = ok; }
            k = min(k, K - 1);
            const int64_t point = t * kRows + n;
            float xnorm = 0.f;
            if (min_dist) {
#pragma unroll
                for (int s = 0; s < DCH; ++s) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t w = xf[s][q];
                        const float lo = lp_to_float((uint16_t)(w & 0xFFFFu), BF);
                        const float hi = lp_to_float((uint16_t)(w >> 16), BF);
                        xnorm += lo * lo + hi * hi;
                    }
                }
                xnorm += __shfl_xor(xnorm, 32);
            }
            if (h == 0 && point < N) {
                assign[point] = k;
                if (min_dist) min_dist[point] = fmaxf(0.f, xnorm - 2.f * m);
            }
        }
        // the next batch must have landed before it is read (wave-private buffers: no barrier)
        if (issued) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(loads) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        t = t1;
        cur = cur == 2 ? 0 : cur + 1;
    }
}

// ------------------------------------------------------------------------------------
// fp32: one point per thread, features in registers, centroid tiles of TK rows in LDS,
// D_ik by direct differences in fp32; ascending k with strict '<'.
template <int DMAX, int TK, int THREADS>
__global__ __launch_bounds__(THREADS) void assign_f32_kernel(
    const float* __restrict__ X, const float* __restrict__ C, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K) {
    __shared__ float sc[TK][DMAX];
    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    C += (size_t)b * K * d;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;
    const int64_t i = (int64_t)blockIdx.x * THREADS + threadIdx.x;
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
        for (int o = threadIdx.x; o < TK * DMAX; o += THREADS) {
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

// fp32 with wide features (128 < d <= 512): the point no longer fits in registers, so each
// thread keeps 16 running distances (one per row of the LDS centroid tile) and walks its own
// row of X in blocks of 32 features, once per centroid tile (the re-reads come from cache).
__global__ __launch_bounds__(256) void assign_f32_wide_kernel(
    const float* __restrict__ X, const float* __restrict__ C, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K) {
    constexpr int TK = 16;
    extern __shared__ float sc_dyn[];                  // [TK][d]
    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    C += (size_t)b * K * d;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const float* xrow = X + (size_t)(i < N ? i : 0) * d;
    float m = INFINITY;
    int a = 0;
    for (int k0 = 0; k0 < K; k0 += TK) {
        __syncthreads();
        for (int o = threadIdx.x; o < TK * d; o += 256) {
            const int r = o / d, j = o - r * d;
            sc_dyn[o] = k0 + r < K ? C[(size_t)(k0 + r) * d + j] : 0.f;
        }
        __syncthreads();
        float D[TK];
#pragma unroll
        for (int r = 0; r < TK; ++r) D[r] = 0.f;
        for (int j0 = 0; j0 < d; j0 += 8) {             // d is a multiple of 8
            const floatx4 xa = *(const floatx4*)(xrow + j0);
            const floatx4 xb = *(const floatx4*)(xrow + j0 + 4);
#pragma unroll
            for (int r = 0; r < TK; ++r) {
                const floatx4 ca = *(const floatx4*)&sc_dyn[r * d + j0];
                const floatx4 cb = *(const floatx4*)&sc_dyn[r * d + j0 + 4];
                const float e0 = xa[0] - ca[0], e1 = xa[1] - ca[1], e2 = xa[2] - ca[2], e3 = xa[3] - ca[3];
                const float e4 = xb[0] - cb[0], e5 = xb[1] - cb[1], e6 = xb[2] - cb[2], e7 = xb[3] - cb[3];
                float t = D[r];
                t += e0 * e0; t += e1 * e1; t += e2 * e2; t += e3 * e3;
                t += e4 * e4; t += e5 * e5; t += e6 * e6; t += e7 * e7;
                D[r] = t;
            }
        }
        const int nk = min(TK, K - k0);
#pragma unroll
        for (int r = 0; r < TK; ++r)
            if (r < nk && D[r] < m) { m = D[r]; a = k0 + r; }
    }
    if (i < N) {
        assign[i] = a;
        if (min_dist) min_dist[i] = m;
    }
}

// Small fp32 problems: 64 points per workgroup, the four waves split every 32-row centroid
// tile between them (8 rows each), then the four candidates of a point are merged through
// LDS (smaller distance first, lower index on equal distances).  Four times the parallelism
// of the one-thread-per-point kernel when there are too few points to fill the chip.
template <int DMAX>
__global__ __launch_bounds__(256) void assign_f32_split_kernel(
    const float* __restrict__ X, const float* __restrict__ C, int32_t* __restrict__ assign,
    float* __restrict__ min_dist, int64_t N, int d, int K) {
    constexpr int TK = 32;
    __shared__ float sc[TK][DMAX];
    __shared__ float cand_d[4][64];
    __shared__ int cand_k[4][64];
    const int b = blockIdx.y;
    X += (size_t)b * N * d;
    C += (size_t)b * K * d;
    assign += (size_t)b * N;
    if (min_dist) min_dist += (size_t)b * N;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + lane;
    float x[DMAX];
#pragma unroll
    for (int j = 0; j < DMAX; j += 4) {
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (i < N && j < d) v = *(const floatx4*)(X + (size_t)i * d + j);
        x[j] = v[0]; x[j + 1] = v[1]; x[j + 2] = v[2]; x[j + 3] = v[3];
    }
    float m = INFINITY;
    int a = 0x7FFFFFFF;
    for (int k0 = 0; k0 < K; k0 += TK) {
        __syncthreads();
        for (int o = threadIdx.x; o < TK * DMAX; o += 256) {
            const int r = o / DMAX, j = o % DMAX;
            sc[r][j] = (k0 + r < K && j < d) ? C[(size_t)(k0 + r) * d + j] : 0.f;
        }
        __syncthreads();
        for (int rr = 0; rr < 8; ++rr) {
            const int r = q * 8 + rr;
            if (k0 + r >= K) break;
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
    cand_d[q][lane] = m;
    cand_k[q][lane] = a;
    __syncthreads();
    if (q == 0 && i < N) {
        float bm = cand_d[0][lane];
        int bk = cand_k[0][lane];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float dm = cand_d[w][lane];
            const int dk = cand_k[w][lane];
            if (dm < bm || (dm == bm && dk < bk)) { bm = dm; bk = dk; }
        }
        assign[i] = min(bk, K - 1);
        if (min_dist) min_dist[i] = bm;
    }
}

// ------------------------------------------------------------------------------------
template <bool BF, int DCH, int P, int WAVES>
static fk_status launch_mfma_v(const Geometry& g, const void* X, const void* frag,
                               const float* bias, int32_t* assign, float* min_dist,
                               hipStream_t s) {
    constexpr int ST = (16 / DCH) < 8 ? (16 / DCH) : 8;   // up to 16 KiB of fragments per stage
    const int64_t per_wg = (int64_t)P * 32 * WAVES;
    dim3 grid((unsigned)cdiv(g.N, per_wg), g.B), block(WAVES * 64);
    hipLaunchKernelGGL((assign_mfma_kernel<BF, DCH, P, WAVES, ST>), grid, block, 0, s,
                       (const uint16_t*)X, (const uintx4*)frag, bias, assign, min_dist, g.N,
                       g.d, g.K, g.ktiles);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

// Tile shape of the sweeping kernel (point tiles per wave x waves per workgroup):
//   0 = 2 x 4 (256 points, 3 workgroups per CU)     1 = 4 x 4 (512 points, 2 per CU)
//   2 = 2 x 8 (512 points, 2 per CU)                 3 = 1 x 4 (128 points, 4 per CU)
// g_variant_override >= 0 forces one (fk_set_option / FK_ASSIGN_VARIANT); otherwise it is chosen
// from the shape and the machine, the counterpart of the paper's cache-aware compile
// heuristic (Section 4.3): no tuning run, just what the runtime reports about the device
// (compute units, last-level cache) and each variant's occupancy.
static std::atomic<int> g_variant_override{[] {
    const char* e = getenv("FK_ASSIGN_VARIANT");
    return e ? atoi(e) : -1;
}()};

// MFMA flop per HBM byte at which the assignment turns from bandwidth- to compute-bound: the
// ratio of the part's dense 16-bit MFMA rate to its HBM rate (2.5 PFLOP/s over 8 TB/s).  The
// kernel does K flop per byte of X, so this is also a number of centroids.
constexpr int kRidgeCentroids = 312;

// Workgroups run in rounds of (CUs x workgroups per CU).  A variant is scored by how full its
// rounds are, (W/S) / ceil(W/S) with W workgroups over S slots, times its steady-state
// efficiency relative to the 512-point shape (bigger workgroups re-use each centroid tile
// more, measured 1.0 / 0.95 / 0.80).  Few points -> small workgroups so the chip fills at all;
// awkward point counts -> the shape with the least idle last round.  Below the ridge with X
// larger than the last-level cache the kernel waits on HBM, not on the matrix pipe, and the
// 256-point shape (three workgroups per unit, more loads in flight) is the efficient one
// instead (measured 8-12% ahead of the 512-point shape there).
int choose_assign_variant(const Geometry& g) {
    const int forced = g_variant_override.load(std::memory_order_relaxed);
    if (forced >= 0 && forced <= 3) return forced;
    const int64_t total_points = (int64_t)g.B * g.N;
    const DeviceInfo& di = device_info();
    const bool hbm_bound = g.K < kRidgeCentroids && total_points * g.d * 2 > di.llc_bytes;
    struct V { int id, points, per_cu; double eff; };
    const V cand[3] = {{2, 512, 2, hbm_bound ? 0.90 : 1.0}, {0, 256, 3, hbm_bound ? 1.0 : 0.95}, {3, 128, 4, 0.80}};
    const double cus = di.cus;
    int best = 2;
    double best_score = -1.0;
    for (const V& v : cand) {
        const double W = (double)cdiv(total_points, v.points), S = cus * v.per_cu;
        const double rounds = W <= S ? 1.0 : (double)cdiv((int64_t)W, (int64_t)S);
        const double score = v.eff * (W / S) / rounds;
        if (score > best_score + 1e-9) { best_score = score; best = v.id; }
    }
    return best;
}

void set_assign_variant_override(int v) { g_variant_override.store(v, std::memory_order_relaxed); }

// Streaming kernel or sweeping kernel for few centroids?  Measured on MI355X: with X well
// beyond the last-level cache and rows of at least 64 bytes the streaming kernel's continuous
// copies win by 10-20% for up to 64 centroids; for cache-sized X, narrow rows, or more centroids the sweeping kernel's bulk prologue
// loads and two points per lane are as fast or faster.  "Well beyond" = one and a half times
// the last-level cache the runtime reports (384 MiB on this part).  g_stream_option: -1 = that
// rule, 0 = never, 1 = whenever the centroids fit one LDS stage (FK_ASSIGN_STREAM sets the
// start value; fk_set_option("assign_stream", v) changes it).
static std::atomic<int> g_stream_option{[] {
    const char* e = getenv("FK_ASSIGN_STREAM");
    return e ? atoi(e) : -1;
}()};

void set_assign_stream_option(int v) { g_stream_option.store(v, std::memory_order_relaxed); }

bool assign_uses_stream_kernel(const Geometry& g) {
    if (g.t == FK_F32 || g.dchunks > 8) return false;
    const int st = (16 / g.dchunks) < 8 ? (16 / g.dchunks) : 8;
    const int opt = g_stream_option.load(std::memory_order_relaxed);
    if (g.ktiles > st || opt == 0) return false;
    if (opt > 0) return true;
    const int64_t x_bytes = (int64_t)g.B * g.N * g.d * 2;
    if (x_bytes < device_info().llc_bytes * 3 / 2 || g.d <= 32) return false;
    // up to two centroid tiles (beyond that the sweeping kernel's two points per lane win back
    // more than the streaming copies save: measured at d = 64, K = 128); one tile for row widths
    // above 128 bytes that are not stored swizzled
    const int limit = (g.d == 64 || g.d == 128 || g.d < 64) ? std::min(st, 2) : 1;
    return g.ktiles <= limit;
}

template <bool BF, int DCH>
static fk_status launch_mfma(const Geometry& g, const void* X, const void* frag,
                             const float* bias, int32_t* assign, float* min_dist,
                             hipStream_t s) {
    constexpr int ST = (16 / DCH) < 8 ? (16 / DCH) : 8;
    if (g.ktiles <= ST && assign_uses_stream_kernel(g)) {
        // persistent waves: as many workgroups as fit the chip, each wave striding over
        // 32-point batches
        constexpr int WAVES = 4;
        const size_t lds = (size_t)(WAVES * 3 * DCH * 64) * 16;
        const bool one_tile = g.ktiles == 1;
        auto kern = one_tile ? assign_mfma_stream_kernel<BF, DCH, WAVES, 1>
                             : assign_mfma_stream_kernel<BF, DCH, WAVES, ST>;
        // set / queried once per kernel and device (also keeps the launch path free of runtime
        // queries, so that it can be captured into a HIP graph after one eager call)
        static PerDeviceInt per_cu_cache[2];
        if (per_cu_cache[one_tile].get() == 0) {
            FK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            int q = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, kern, WAVES * 64, lds) != hipSuccess || q < 1)
                q = 1;
            per_cu_cache[one_tile].set(q);
        }
        const int per_cu = per_cu_cache[one_tile].get();
        const int64_t nbatches = cdiv(g.N, 32);
        int64_t wgs = (int64_t)device_cu_count() * per_cu;
        if (wgs > cdiv(nbatches, WAVES)) wgs = cdiv(nbatches, WAVES);
        dim3 grid((unsigned)wgs, g.B), block(WAVES * 64);
        hipLaunchKernelGGL(kern, grid, block, lds, s, (const uint16_t*)X, (const uintx4*)frag, bias,
                           assign, min_dist, g.N, g.d, g.K, g.ktiles);
        FK_HIP(hipGetLastError());
        return FK_OK;
    }
    switch (choose_assign_variant(g)) {
        case 1: return launch_mfma_v<BF, DCH, 4, 4>(g, X, frag, bias, assign, min_dist, s);
        case 0: return launch_mfma_v<BF, DCH, 2, 4>(g, X, frag, bias, assign, min_dist, s);
        case 3: return launch_mfma_v<BF, DCH, 1, 4>(g, X, frag, bias, assign, min_dist, s);
        default: return launch_mfma_v<BF, DCH, 2, 8>(g, X, frag, bias, assign, min_dist, s);
    }
}

template <bool BF, int DCH>
static fk_status launch_mfma_wide(const Geometry& g, const void* X, const void* frag,
                                  const float* bias, int32_t* assign, float* min_dist,
                                  hipStream_t s) {
    constexpr int WAVES = 8;
    dim3 grid((unsigned)cdiv(g.N, WAVES * 32), g.B), block(WAVES * 64);
    hipLaunchKernelGGL((assign_mfma_wide_kernel<BF, DCH, WAVES>), grid, block, 0, s,
                       (const uint16_t*)X, (const uintx4*)frag, bias, assign, min_dist, g.N, g.d,
                       g.K, g.ktiles);
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
        case 16: return launch_mfma_wide<BF, 16>(g, X, frag, bias, assign, min_dist, s);
        case 32: return launch_mfma_wide<BF, 32>(g, X, frag, bias, assign, min_dist, s);
    }
    set_error("assign: no kernel for %d feature chunks", g.dchunks);
    return FK_EUNSUPPORTED;
}

fk_status launch_assign(const Geometry& g, const void* X, const void* C_or_frag,
                        const float* c_bias, int32_t* assign, float* min_dist, hipStream_t s) {
    if (g.t == FK_F16) return launch_mfma_d<false>(g, X, C_or_frag, c_bias, assign, min_dist, s);
    if (g.t == FK_BF16) return launch_mfma_d<true>(g, X, C_or_frag, c_bias, assign, min_dist, s);
    const float* Xf = (const float*)X;
    const float* Cf = (const float*)C_or_frag;
    if (g.d > 128) {
        hipLaunchKernelGGL(assign_f32_wide_kernel, dim3((unsigned)cdiv(g.N, 256), g.B), dim3(256),
                           (size_t)16 * g.d * sizeof(float), s, Xf, Cf, assign, min_dist, g.N, g.d, g.K);
        FK_HIP(hipGetLastError());
        return FK_OK;
    }
    // small problems: split each centroid tile over the waves, so that even 16K points spread
    // over the chip
    const bool small = (int64_t)g.B * g.N < ((int64_t)1 << 18);
    dim3 grid((unsigned)cdiv(g.N, small ? 64 : 256), g.B), block(256);
#define FK_F32_LAUNCH(DM)                                                                         \
    do {                                                                                          \
        if (small)                                                                                \
            hipLaunchKernelGGL((assign_f32_split_kernel<DM>), grid, block, 0, s, Xf, Cf, assign,  \
                               min_dist, g.N, g.d, g.K);                                          \
        else                                                                                      \
            hipLaunchKernelGGL((assign_f32_kernel<DM, 32, 256>), grid, block, 0, s, Xf, Cf, assign, \
                               min_dist, g.N, g.d, g.K);                                          \
    } while (0)
    if (g.d <= 32) FK_F32_LAUNCH(32);
    else if (g.d <= 64) FK_F32_LAUNCH(64);
    else FK_F32_LAUNCH(128);
#undef FK_F32_LAUNCH
    FK_HIP(hipGetLastError());
    return FK_OK;
}

}  // namespace fk
