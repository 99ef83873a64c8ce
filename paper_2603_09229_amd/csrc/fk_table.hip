// Up to 256 clusters (16-bit storage, 32 < K <= 256, d <= 128): assignment and centroid sums
// in ONE pass over X, with the whole K x d table of sums held on chip.
//
// Section 4.2 of the paper keeps a segment's partial sum on chip and merges it once; with a
// table this small the whole of it fits the register file of one workgroup (K x d fp32 =
// 128 KiB at K = 256, d = 128), so a persistent workgroup can add every point it assigns
// straight into the table and X is read once per Lloyd iteration instead of twice, with no
// sort at all.  The split: wave w of the 8 owns clusters [32w, 32w + 32) and keeps their 32 x d
// block of sums in MFMA accumulators (d/32 x 16 registers per lane).
//
// Per batch of 256 points a workgroup
//   1. lands the batch in LDS (rows were prefetched into registers with row-contiguous loads
//      during the previous batch and are written out XOR-swizzled by row),
//   2. computes the assignment of 32 points per wave exactly as the assignment kernels do
//      (centroid fragments resident in LDS as MFMA A operands, packed-score argmax),
//   3. publishes the 256 cluster ids in LDS, and
//   4. every wave compacts, in index order, the points that belong to its 32 clusters into a
//      list and adds them 32 at a time with one more contraction,
//          S[k][j] += sum_p onehot[k][p] * x[p][j],   onehot[k][p] = (a_p == k),
//      whose products are exact (x times 1 or 0) and accumulate in fp32: Eq. 3's sum.  The
//      compaction is what makes the one-hot product cheap here: each wave multiplies only its
//      own ~1/8 of the points instead of all of them.  The contraction runs over points, so
//      its X operand is read from the row-major batch with the transposing LDS load, the row
//      of each list entry supplying the address.
// Every cluster row has exactly one owner and points are visited in index order, so the sums
// are accumulated in a fixed order: no atomics, bit-reproducible.  Each workgroup leaves one
// partial table and one count per cluster, partial[B][K][G][d] / wg_counts[B][K][G], which the
// merge/normalise kernel adds in workgroup order.
#include <algorithm>

#include "fk_common.h"
#include "fk_device.h"

namespace fk {

typedef short shortx4 __attribute__((ext_vector_type(4)));

// BF: bf16 (else fp16).  DCH: feature chunks of 16 per point (2, 4 or 8).
// Dynamic LDS: centroid fragments [ktiles][DCH][64] x 16 B | batch rows [256][d/8] x 16 B |
// bias [ktiles][32] floats | cluster ids [256] ints | per-wave point lists [8][256 + 32] ints.
template <bool BF, int DCH>
__global__ __launch_bounds__(512) void table_update_kernel(
    const uint16_t* __restrict__ X, const uintx4* __restrict__ c_frag,
    const float* __restrict__ c_bias, int32_t* __restrict__ assign, float* __restrict__ partial,
    int32_t* __restrict__ wg_counts, int64_t N, int d, int K, int ktiles) {
    constexpr int kThreads = 512, kRows = 256;
    constexpr int CB = DCH / 2;                                // 32-feature column blocks of the table
    constexpr int kList = kRows + 32;                          // list entries per wave (padded to whole chunks)
    constexpr uint32_t kOne = BF ? 0x3F80u : 0x3C00u;          // 1.0 in the storage type
    extern __shared__ uintx4 dyn_lds[];
    const int ppr = d >> 3;                                    // 16-byte pieces per row
    const int swz = (ppr & (ppr - 1)) == 0 ? ppr - 1 : 0;      // XOR mask for the piece index
    uintx4* sfrag = dyn_lds;
    uintx4* xl = sfrag + ktiles * DCH * 64;
    float* sbias = (float*)(xl + kRows * ppr);
    int* sa = (int*)(sbias + ktiles * 32);
    int* slist = sa + kRows;

    const int b = blockIdx.y, G = gridDim.x, wg = blockIdx.x;
    X += (size_t)b * N * d;
    assign += (size_t)b * N;
    c_frag += (size_t)b * ktiles * DCH * 64;
    c_bias += (size_t)b * ktiles * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;

    const int64_t nbatches = (N + kRows - 1) / kRows;

    // Row-contiguous prefetch of a batch: in round i thread t takes piece t % (2*DCH) of row
    // i * 256/DCH + t / (2*DCH), so a wave-wide load covers whole rows (threads whose piece lies
    // beyond a narrower row idle).  Rows past the end of X re-read the last row (their cluster
    // id is published as -1 and nobody adds them).
    constexpr int kPieces = 2 * DCH, kRowsPerRound = kThreads / kPieces;
    const int my_piece = tid % kPieces, my_row0 = tid / kPieces;
    const bool piece_live = my_piece < ppr;
    uintx4 xn[DCH];
    auto prefetch = [&](int64_t batch) {
#pragma unroll
        for (int i = 0; i < DCH; ++i) {
            const int64_t point = min(batch * kRows + i * kRowsPerRound + my_row0, N - 1);
            if (piece_live) xn[i] = *(const uintx4*)(X + (size_t)point * d + my_piece * 8);
        }
    };

    int64_t t = wg;
    if (t < nbatches) prefetch(t);
    for (int o = tid; o < ktiles * DCH * 64; o += kThreads) sfrag[o] = c_frag[o];
    for (int o = tid; o < ktiles * 32; o += kThreads) sbias[o] = c_bias[o];

    // this wave's 32 x d block of the table: accS[cb][i] is cluster row 8*(i/4) + 4*h + i%4,
    // feature 32*cb + n
    floatx16 accS[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) accS[cb][i] = 0.f;
    int cnt = 0;                                               // points of cluster 32*wave + n so far
    int* mylist = slist + wave * kList;
    // Address pattern of the transposing read: inside a group of 16 lanes, lane L supplies the
    // 8 bytes (row L/4, columns 4*(L%4)..+3) of a 4 x 16 block and receives column L of it.
    // Group (lane/16): bit 0 = which 16 columns of the 32, bit 1 = h.
    const int L = lane & 15, nb = (lane >> 4) & 1;
    int tr_piece[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) tr_piece[cb] = min(4 * cb + 2 * nb + ((L & 3) >> 1), ppr - 1);

    for (; t < nbatches; t += G) {
        // 1. the prefetched rows go to LDS, swizzled so that the 16 lanes that share a piece
        //    index hit 16 different bank groups
        if (piece_live) {
#pragma unroll
            for (int i = 0; i < DCH; ++i) {
                const int row = i * kRowsPerRound + my_row0;
                xl[row * ppr + (my_piece ^ (row & swz))] = xn[i];
            }
        }
        __syncthreads();
        if (t + G < nbatches) prefetch(t + G);                 // lands while this batch is processed

        // 2. this wave's 32 points as MFMA B operands: features [s*16 + h*8, +8) of point n
        const int row = wave * 32 + n;
        uintx4 xf[DCH];
#pragma unroll
        for (int s = 0; s < DCH; ++s) {
            const int piece = min(2 * s + h, ppr - 1);      // chunks past d meet zero centroid features
            xf[s] = xl[row * ppr + (piece ^ (row & swz))];
        }
        float best = -INFINITY;
        int btile = 0;
        // packed argmax of one tile's 16 scores per lane: low 4 mantissa bits = 15 - slot (same
        // rules as the assignment kernels)
        auto fold = [&](const floatx16& acc, int tile) {
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
            btile = improved ? tile : btile;
        };
        auto bias_of = [&](int tile) {
            floatx16 bias16;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 bv = *(const floatx4*)&sbias[tile * 32 + 8 * q + 4 * h];
                bias16[4 * q + 0] = bv[0];
                bias16[4 * q + 1] = bv[1];
                bias16[4 * q + 2] = bv[2];
                bias16[4 * q + 3] = bv[3];
            }
            return bias16;
        };
        // centroid tiles two at a time: two independent MFMA chains keep the matrix pipe busy
        // while one waits for its own previous result
        int tt = 0;
        for (; tt + 1 < ktiles; tt += 2) {
            floatx16 acc_a = bias_of(tt), acc_b = bias_of(tt + 1);
#pragma unroll
            for (int s = 0; s < DCH; ++s) {
                acc_a = mfma32<BF>(sfrag[(tt * DCH + s) * 64 + lane], xf[s], acc_a);
                acc_b = mfma32<BF>(sfrag[((tt + 1) * DCH + s) * 64 + lane], xf[s], acc_b);
            }
            fold(acc_a, tt);
            fold(acc_b, tt + 1);
        }
        if (tt < ktiles) {
            floatx16 acc = bias_of(tt);
#pragma unroll
            for (int s = 0; s < DCH; ++s) acc = mfma32<BF>(sfrag[(tt * DCH + s) * 64 + lane], xf[s], acc);
            fold(acc, tt);
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
            const int64_t point = t * kRows + row;
            if (h == 0) {
                const bool valid = point < N;
                sa[row] = valid ? k : -1;
                if (valid) assign[point] = k;
            }
        }
        __syncthreads();

        // 3. this wave's points (cluster id in [32*wave, 32*wave + 32)), compacted in index order
        //    into its list: entry = batch row | cluster-in-wave << 8
        int nmine = 0;
#pragma unroll
        for (int g = 0; g < kRows / 64; ++g) {
            const int a = sa[g * 64 + lane];
            const bool match = (a >> 5) == wave;               // -1 (no point) matches no wave
            const uint64_t mm = __ballot(match);
            const int pos = nmine + __popcll(mm & ((1ull << lane) - 1ull));
            if (match) mylist[pos] = (g * 64 + lane) | ((a & 31) << 8);
            nmine += __popcll(mm);
        }
        // pad the last chunk of 32 with entries no cluster claims (row 0 holds finite data and
        // meets a zero of the one-hot operand)
        if (lane < 32) mylist[nmine + lane] = 32 << 8;
        __builtin_amdgcn_wave_barrier();
        // 4. one-hot contraction, 32 list entries at a time
        for (int c0 = 0; c0 < nmine; c0 += 32) {
            // all list reads of the chunk first: this lane's entry, and the rows it addresses for
            // the transposing reads (entries 16*s2 + 8*h + 4*u + L/4)
            const int e = mylist[c0 + n];
            int r[2][2];
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int u = 0; u < 2; ++u) r[s2][u] = mylist[c0 + 16 * s2 + 8 * h + 4 * u + (L >> 2)] & 255;
            shortx4 xt[2][CB][2];
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int rr = r[s2][u];
                        const char* src = (const char*)(xl + rr * ppr + (tr_piece[cb] ^ (rr & swz))) + ((L & 1) << 3);
                        xt[s2][cb][u] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)src);
                    }
            const int kc = e >> 8;                             // 0..31, or 32 for padding
            // bit p of E: entry p of the chunk belongs to cluster row n of this wave
            uint32_t E = 0xFFFFFFFFu;
#pragma unroll
            for (int bit = 0; bit < 6; ++bit) {
                const uint32_t pl = (uint32_t)__ballot((kc >> bit) & 1);
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
                    const uintx2 lo = __builtin_bit_cast(uintx2, xt[s2][cb][0]), hi = __builtin_bit_cast(uintx2, xt[s2][cb][1]);
                    const uintx4 Bt = {lo[0], lo[1], hi[0], hi[1]};
                    accS[cb] = mfma32<BF>(A, Bt, accS[cb]);
                }
            }
        }
        __syncthreads();                                       // rows and ids are free again
    }

    // one partial table row and one count per cluster of this workgroup
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int k = wave * 32 + 8 * (i >> 2) + 4 * h + (i & 3), j = 32 * cb + n;
            if (k < K && j < d) partial[(((size_t)b * K + k) * G + wg) * d + j] = accS[cb][i];
        }
    if (h == 0 && wave * 32 + n < K)
        wg_counts[((size_t)b * K + wave * 32 + n) * G + wg] = cnt;
}

// ------------------------------------------------------------------------------------
bool table_update_enabled(const Geometry& g) { return g.table_grid_cap > 0 && fused_update_allowed(); }

template <bool BF, int DCH>
static fk_status launch_table_update_t(const Geometry& g, const Workspace& w, const void* X,
                                       int32_t* assign, int* grid_out, hipStream_t s) {
    auto kern = table_update_kernel<BF, DCH>;
    const size_t lds = (size_t)g.ktiles * DCH * 1024 + (size_t)256 * g.d * 2 + (size_t)g.ktiles * 128 +
                       256 * 4 + 8 * (256 + 32) * 4;
    static PerDeviceInt attr_set;
    if (!attr_set.get()) {
        FK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)device_info().lds_bytes));
        attr_set.set(1);
    }
    if ((int64_t)lds > device_info().lds_bytes) {
        set_error("table update: %zu bytes of LDS needed, %lld available", lds, (long long)device_info().lds_bytes);
        return FK_EUNSUPPORTED;
    }
    // one persistent workgroup per compute unit, shared out over the instances
    int64_t G = std::max<int64_t>(1, device_cu_count() / g.B);
    G = std::min<int64_t>(G, g.table_grid_cap);
    G = std::min<int64_t>(G, cdiv(g.N, 256));
    dim3 grid((unsigned)G, g.B), block(512);
    hipLaunchKernelGGL(kern, grid, block, lds, s, (const uint16_t*)X, (const uintx4*)w.c_frag,
                       (const float*)w.c_bias, assign, w.partial, w.wg_counts, g.N, g.d, g.K, g.ktiles);
    FK_HIP(hipGetLastError());
    *grid_out = (int)G;
    return FK_OK;
}

fk_status launch_table_update(const Geometry& g, const Workspace& w, const void* X, int32_t* assign,
                              int* grid_out, hipStream_t s) {
    if (g.table_grid_cap <= 0) {
        set_error("table update: shape not eligible (needs 16-bit storage, 32 < K <= 256, d <= 128)");
        return FK_EUNSUPPORTED;
    }
    const bool bf = g.t == FK_BF16;
    switch (g.dchunks) {
        case 2: return bf ? launch_table_update_t<true, 2>(g, w, X, assign, grid_out, s)
                          : launch_table_update_t<false, 2>(g, w, X, assign, grid_out, s);
        case 4: return bf ? launch_table_update_t<true, 4>(g, w, X, assign, grid_out, s)
                          : launch_table_update_t<false, 4>(g, w, X, assign, grid_out, s);
        case 8: return bf ? launch_table_update_t<true, 8>(g, w, X, assign, grid_out, s)
                          : launch_table_update_t<false, 8>(g, w, X, assign, grid_out, s);
    }
    set_error("table update: no kernel for %d feature chunks", g.dchunks);
    return FK_EUNSUPPORTED;
}

}  // namespace fk
