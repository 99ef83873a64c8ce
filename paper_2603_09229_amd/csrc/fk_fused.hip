// Few clusters (K <= 32, 16-bit storage, d <= 128): the centroid update without any sort or
// gather, optionally fused into the assignment pass.
//
// With so few clusters the update of Section 4.2 spends its time re-reading X through the
// sorted index; the whole table of sums is only K x d floats.  Here every wave keeps that
// table in MFMA accumulators and adds a batch of 32 points to it with one more contraction:
//     S[k][j] += sum_p onehot[k][p] * x[p][j],   onehot[k][p] = (a_p == k)
// The products are exact (x times 1 or 0) and accumulate in fp32, so this is Eq. 3's sum in a
// fixed, reproducible order -- no atomics, as in the sort-inverse path.  X is streamed once,
// row-contiguous; when the assignment is computed in the same pass (ASSIGN), one Lloyd
// iteration reads X once instead of twice.  The contraction runs over points, so its
// X-operand is the transpose of the batch as it sits in LDS: it is read with the
// transposing LDS load (each lane receives four consecutive points of one feature column).
//
// Every workgroup leaves one partial table and one count per cluster; the ordinary
// merge/normalise kernel adds a cluster's partial rows (and counts) in workgroup order.
#include <algorithm>

#include "fk_common.h"
#include "fk_device.h"

namespace fk {

// BF: bf16 (else fp16).  DCH: feature chunks of 16 per point (2, 4 or 8).  ASSIGN: compute
// the assignment here (argmax of x.c_k - ||c_k||^2/2 over the single centroid tile, same
// packed-score rules as the assignment kernels) and write it; otherwise read it.
//
// Grid (G, B).  Wave w of workgroup g handles the 32-point batches g*WAVES + w,
// + G*WAVES, ...: a fixed partition, so the partial tables are reproducible.
// partial: [B][K][G][d] floats, wg_counts: [B][K][G].
template <bool BF, int DCH, int WAVES, bool ASSIGN>
__global__ __launch_bounds__(WAVES * 64) void stream_update_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, int32_t* assign, float* __restrict__ partial,
    int32_t* __restrict__ wg_counts, int64_t N, int d, int K) {
    constexpr int kThreads = WAVES * 64;
    constexpr int kRows = 32;                          // points per batch
    constexpr int CB = DCH / 2;                        // 32-feature column blocks of the table
    constexpr int kIdVec = ASSIGN ? 0 : 16;            // 256 bytes of cluster ids behind a batch
    constexpr int kBufVec = DCH * 64 + kIdVec;         // 16-byte vectors per batch buffer
    constexpr int loads = DCH + (ASSIGN ? 0 : 1);      // copy instructions per batch, always all issued
    constexpr uint32_t kOne = BF ? 0x3F80u : 0x3C00u;  // 1.0 in the storage type
    __shared__ uintx4 sfrag[ASSIGN ? DCH * 64 : 1];
    __shared__ float sbias[32];
    extern __shared__ uintx4 dyn_lds[];                // per wave: a ring of 3 batch buffers
    const int ppr = d >> 3;                            // 16-byte pieces per row
    const int swz = (ppr & (ppr - 1)) == 0 ? min(ppr, 8) - 1 : 0;   // XOR mask for the piece index

    const int b = blockIdx.y, G = gridDim.x, wg = blockIdx.x;
    X += (size_t)b * N * d;
    assign += (size_t)b * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    uintx4* ring = dyn_lds + (size_t)wave * 3 * kBufVec;

    if (ASSIGN) {
        c_frag += (size_t)b * DCH * 64;
        c_bias += (size_t)b * 32;
        for (int o = tid; o < DCH * 64; o += kThreads) sfrag[o] = c_frag[o];
        if (tid < 32) sbias[tid] = c_bias[tid];
    }

    const int64_t nbatches = (N + kRows - 1) / kRows;
    const int64_t stride = (int64_t)G * WAVES;
    int64_t t = (int64_t)wg * WAVES + wave;

    // Slot j of a buffer holds piece (j % ppr) ^ (row & swz) of row j / ppr.  Every copy
    // instruction is issued with all lanes live (rows past the end of X or of the batch
    // re-read the last valid row): the waits below count instructions, and a stale slot
    // must hold finite values because it is multiplied by a zero of the one-hot operand.
    auto request = [&](int64_t batch, uintx4* buf) {
#pragma unroll
        for (int q = 0; q < DCH; ++q) {
            const int j = q * 64 + lane;
            int row = j / ppr;
            const int piece = j - row * ppr;
            row = min(row, kRows - 1);
            const int64_t point = min(batch * kRows + row, N - 1);
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(X + (size_t)point * d + ((piece ^ (row & swz)) << 3)),
                (__attribute__((address_space(3))) void*)(buf + q * 64), 16, 0, 0);
        }
        if (!ASSIGN) {
            const int64_t point = min(batch * kRows + lane, N - 1);
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(assign + point),
                (__attribute__((address_space(3))) void*)(buf + DCH * 64), 4, 0, 0);
        }
    };

    // Address of this lane's share of a transposing read: inside a group of 16 lanes, lane L
    // supplies the 8 bytes (row L/4, columns 4*(L%4)..+3) of a 4 x 16 block and receives
    // column L of it.  Group (lane/16): bit 0 = which 16 columns of the 32, bit 1 = h.
    const int L = lane & 15, nb = (lane >> 4) & 1;
    int tr_piece[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) tr_piece[cb] = min(4 * cb + 2 * nb + ((L & 3) >> 1), ppr - 1);

    floatx16 accS[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) accS[cb][i] = 0.f;
    int cnt = 0;

    // Two batches are kept in flight.  Copies of a wave complete in order, so "at most `loads`
    // outstanding" means that everything but the newest batch has landed.
    if (t < nbatches) request(t, ring);
    if (t + stride < nbatches) request(t + stride, ring + kBufVec);
    if (t + stride < nbatches) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(loads) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (ASSIGN) __syncthreads();           // C is in LDS; no workgroup barrier inside the loop

    int cur = 0;
    while (t < nbatches) {
        const int64_t t1 = t + stride, t2 = t1 + stride;
        const uintx4* bufc = ring + cur * kBufVec;
        uintx4* buf2 = ring + (cur == 0 ? 2 : cur - 1) * kBufVec;   // read one iteration ago

        // LDS reads through opaque instructions: the wait for the copy that filled this buffer
        // was issued by hand, and the compiler must not add one for the younger copy in flight.
        // Every group of reads sits in ONE asm statement together with its wait, with all its
        // results as outputs: no result register can be touched between issue and arrival.
        uintx4 xf[ASSIGN ? DCH : 1];
        if (ASSIGN) {
            uint32_t xa[DCH];
#pragma unroll
            for (int s = 0; s < DCH; ++s) {
                const int piece = min(2 * s + h, ppr - 1);       // chunks past d meet zero centroid features
                xa[s] = lds_addr(bufc + n * ppr + (piece ^ (n & swz)));
            }
            if constexpr (DCH == 2)
                asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(xf[0]), "=&v"(xf[1]) : "v"(xa[0]), "v"(xa[1]) : "memory");
            else if constexpr (DCH == 4)
                asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\t"
                             "ds_read_b128 %3, %7\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(xf[0]), "=&v"(xf[1]), "=&v"(xf[2]), "=&v"(xf[3])
                             : "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]) : "memory");
            else {
                static_assert(DCH == 2 || DCH == 4 || DCH == 8, "feature chunks per point");
                asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\t"
                             "ds_read_b128 %3, %7\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(xf[0]), "=&v"(xf[1]), "=&v"(xf[2]), "=&v"(xf[3])
                             : "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]) : "memory");
                asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\t"
                             "ds_read_b128 %3, %7\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(xf[4 % DCH]), "=&v"(xf[5 % DCH]), "=&v"(xf[6 % DCH]), "=&v"(xf[7 % DCH])
                             : "v"(xa[4 % DCH]), "v"(xa[5 % DCH]), "v"(xa[6 % DCH]), "v"(xa[7 % DCH]) : "memory");
            }
        }
        // transposed operand: one statement (four reads + wait) per (half batch, column block)
        uintx2 xt[2][CB][2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            uint32_t ta[CB][2];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int row = 16 * s2 + 8 * h + 4 * u + (L >> 2);
                    ta[cb][u] = lds_addr(bufc + row * ppr + (tr_piece[cb] ^ (row & swz))) + ((L & 1) << 3);
                }
#pragma unroll
            for (int cb = 0; cb + 1 < CB || cb == 0; cb += 2) {
                if (cb + 1 < CB)
                    asm volatile("ds_read_b64_tr_b16 %0, %4\n\tds_read_b64_tr_b16 %1, %5\n\t"
                                 "ds_read_b64_tr_b16 %2, %6\n\tds_read_b64_tr_b16 %3, %7\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(xt[s2][cb][0]), "=&v"(xt[s2][cb][1]), "=&v"(xt[s2][(cb + 1) % CB][0]),
                                   "=&v"(xt[s2][(cb + 1) % CB][1])
                                 : "v"(ta[cb][0]), "v"(ta[cb][1]), "v"(ta[(cb + 1) % CB][0]), "v"(ta[(cb + 1) % CB][1])
                                 : "memory");
                else
                    asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(xt[s2][cb][0]), "=&v"(xt[s2][cb][1]) : "v"(ta[cb][0]), "v"(ta[cb][1]) : "memory");
            }
        }
        int k = 0;
        if (!ASSIGN)
            asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(k) : "v"(lds_addr(bufc + DCH * 64) + (uint32_t)(n << 2)) : "memory");

        const bool issued = t2 < nbatches;
        if (issued) request(t2, buf2);

        const int64_t point = t * kRows + n;
        const bool valid = point < N;
        if (ASSIGN) {
            floatx16 bias16;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 bv = *(const floatx4*)&sbias[8 * q + 4 * h];
                bias16[4 * q + 0] = bv[0];
                bias16[4 * q + 1] = bv[1];
                bias16[4 * q + 2] = bv[2];
                bias16[4 * q + 3] = bv[3];
            }
            floatx16 acc = mfma32<BF>(sfrag[lane], xf[0], bias16);
#pragma unroll
            for (int s = 1; s < DCH; ++s) acc = mfma32<BF>(sfrag[s * 64 + lane], xf[s], acc);
            // score with its low 4 mantissa bits replaced by 15 - slot: one max carries both
            float m = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float k0 = __uint_as_float((__float_as_uint(acc[i]) & 0xFFFFFFF0u) | (uint32_t)(15 - i));
                const float k1 = __uint_as_float((__float_as_uint(acc[i + 1]) & 0xFFFFFFF0u) | (uint32_t)(14 - i));
                m = __builtin_fmaxf(__builtin_fmaxf(m, k0), k1);
            }
            const uint32_t bits = __float_as_uint(m);
            const int i = 15 - (int)(bits & 15u);
            k = 8 * (i >> 2) + 4 * h + (i & 3);
            m = __uint_as_float(bits & 0xFFFFFFF0u);
            const float om = __shfl_xor(m, 32);
            const int ok = __shfl_xor(k, 32);
            if (om > m || (om == m && ok < k)) { m = om; k = ok; }
            k = min(k, K - 1);
            if (h == 0 && valid) assign[point] = k;
        } else {
            k = min(max(k, 0), K - 1);
        }

        // one-hot rows: bit p of E says that point p of the batch belongs to cluster n (this
        // lane's row of the table), built from the bit planes of the 32 cluster ids
        uint32_t E = (uint32_t)__ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 5; ++bit) {
            const uint32_t pl = (uint32_t)__ballot((k >> bit) & 1);
            E &= ((n >> bit) & 1) ? pl : ~pl;
        }
        cnt += __popc(E);
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const uint32_t byte = (E >> (16 * s2 + 8 * h)) & 0xFFu;
            uintx4 A;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t two = (byte >> (2 * q)) & 3u;
                A[q] = ((two & 1u) | ((two & 2u) << 15)) * kOne;
            }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const uintx4 Bt = {xt[s2][cb][0][0], xt[s2][cb][0][1], xt[s2][cb][1][0], xt[s2][cb][1][1]};
                accS[cb] = mfma32<BF>(A, Bt, accS[cb]);
            }
        }

        // the next batch must have landed before it is read (wave-private buffers: no barrier)
        if (issued) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(loads) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        t = t1;
        cur = cur == 2 ? 0 : cur + 1;
    }

    // The waves' tables meet in LDS (the ring is free now) and are added in wave order.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    constexpr int dpad = DCH * 16;
    float* comb = (float*)dyn_lds;                     // [WAVES][32][dpad]
    int* ccnt = (int*)(comb + WAVES * 32 * dpad);      // [WAVES][32]
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            comb[(wave * 32 + 8 * (i >> 2) + 4 * h + (i & 3)) * dpad + 32 * cb + n] = accS[cb][i];
    if (h == 0) ccnt[wave * 32 + n] = cnt;
    __syncthreads();
    for (int o = tid; o < K * d; o += kThreads) {
        const int kk = o / d, j = o - kk * d;
        float s = comb[kk * dpad + j];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) s += comb[(w * 32 + kk) * dpad + j];
        partial[(((size_t)b * K + kk) * G + wg) * d + j] = s;
    }
    if (tid < K) {
        int c = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) c += ccnt[w * 32 + tid];
        wg_counts[((size_t)b * K + tid) * G + wg] = c;
    }
}

// ------------------------------------------------------------------------------------
static std::atomic<int> g_fused_option{-1};   // -1 / 1: use when the shape allows, 0: never

void set_fused_update_option(int v) { g_fused_option.store(v, std::memory_order_relaxed); }

bool fused_update_allowed() { return g_fused_option.load(std::memory_order_relaxed) != 0; }

bool fused_update_enabled(const Geometry& g) { return g.fused_grid_cap > 0 && fused_update_allowed(); }

template <bool BF, int DCH, bool ASSIGN>
static fk_status launch_stream_update_t(const Geometry& g, const Workspace& w, const void* X,
                                        int32_t* assign, int* grid_out, hipStream_t s) {
    constexpr int WAVES = 4;
    auto kern = stream_update_kernel<BF, DCH, WAVES, ASSIGN>;
    const size_t lds = (size_t)WAVES * 3 * (DCH * 64 + (ASSIGN ? 0 : 16)) * 16;
    // set / queried once per kernel and device: the launch path stays free of runtime queries afterwards
    static PerDeviceInt per_cu;
    if (per_cu.get() == 0) {
        FK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        int q = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, kern, WAVES * 64, lds) != hipSuccess || q < 1)
            q = 1;
        per_cu.set(q);
    }
    const int64_t nbatches = cdiv(g.N, 32);
    int64_t G = cdiv((int64_t)device_cu_count() * per_cu.get(), g.B);
    G = std::min<int64_t>(G, g.fused_grid_cap);
    G = std::min<int64_t>(G, cdiv(nbatches, WAVES));
    G = std::max<int64_t>(G, 1);
    dim3 grid((unsigned)G, g.B), block(WAVES * 64);
    hipLaunchKernelGGL(kern, grid, block, lds, s, (const uint16_t*)X, (const uintx4*)w.c_frag,
                       (const float*)w.c_bias, assign, w.partial, w.wg_counts, g.N, g.d, g.K);
    FK_HIP(hipGetLastError());
    *grid_out = (int)G;
    return FK_OK;
}

template <bool ASSIGN>
static fk_status launch_stream_update_d(const Geometry& g, const Workspace& w, const void* X,
                                        int32_t* assign, int* grid_out, hipStream_t s) {
    const bool bf = g.t == FK_BF16;
    switch (g.dchunks) {
        case 2: return bf ? launch_stream_update_t<true, 2, ASSIGN>(g, w, X, assign, grid_out, s)
                          : launch_stream_update_t<false, 2, ASSIGN>(g, w, X, assign, grid_out, s);
        case 4: return bf ? launch_stream_update_t<true, 4, ASSIGN>(g, w, X, assign, grid_out, s)
                          : launch_stream_update_t<false, 4, ASSIGN>(g, w, X, assign, grid_out, s);
        case 8: return bf ? launch_stream_update_t<true, 8, ASSIGN>(g, w, X, assign, grid_out, s)
                          : launch_stream_update_t<false, 8, ASSIGN>(g, w, X, assign, grid_out, s);
    }
    set_error("fused update: no kernel for %d feature chunks", g.dchunks);
    return FK_EUNSUPPORTED;
}

fk_status launch_stream_update(const Geometry& g, const Workspace& w, const void* X,
                               int32_t* assign, bool compute_assign, int* grid_out,
                               hipStream_t s) {
    if (g.fused_grid_cap <= 0) {
        set_error("fused update: shape not eligible (needs 16-bit storage, K <= 32, d <= 128)");
        return FK_EUNSUPPORTED;
    }
    return compute_assign ? launch_stream_update_d<true>(g, w, X, assign, grid_out, s)
                          : launch_stream_update_d<false>(g, w, X, assign, grid_out, s);
}

}  // namespace fk
