// Inverse mapping of the sort-inverse update (paper Section 4.2, Algorithm 3, first two
// lines): a stable argsort of the assignment vector by cluster id, done as a counting
// sort (one pass when K <= 2048 bins, two least-significant-digit passes above that).
//
// The paper treats argsort as a given primitive.  Here the exclusive scan of the cluster
// histogram doubles as the segment table: seg_off[k] .. seg_off[k+1] is cluster k's run in
// sorted order, so the sorted id sequence is only materialised by the two-pass variant.
// Stability makes point indices ascend inside a segment, which keeps the later row gather
// monotone in address.
//
// Only integer LDS counters are used; no floating-point data is touched here.
#include <stdlib.h>

#include "fk_common.h"

namespace fk {

namespace {

__device__ __forceinline__ int clamp_key(int k, int kmax) { return min(max(k, 0), kmax); }

// Lanes of the wave whose `digit` equals this lane's, among lanes in `valid`.
__device__ __forceinline__ uint64_t match_digit(int digit, int nbits, uint64_t valid) {
    uint64_t peers = valid;
    // digits have at most 11 bits; unrolled, each step guarded by a wave-uniform test
#pragma unroll
    for (int b = 0; b < 11; ++b) {
        if (b < nbits) {
            const bool bit = (digit >> b) & 1;
            const uint64_t bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
    }
    return peers;
}

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << (threadIdx.x & 63)) - 1ull;
}

// In-place exclusive scan of v[0..n) in LDS by the whole workgroup; returns the total.
// `scratch` holds at least 33 ints.  Ends with a barrier.
__device__ int block_exclusive_scan(int* v, int n, int* scratch) {
    const int T = blockDim.x, tid = threadIdx.x;
    const int per = (n + T - 1) / T;
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += v[i];
    // inclusive scan of the per-thread sums inside each wave
    int inc = sum;
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) scratch[wave] = inc;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        const int nw = (T + 63) >> 6;
        for (int w = 0; w < nw; ++w) { const int t = scratch[w]; scratch[w] = run; run += t; }
        scratch[32] = run;
    }
    __syncthreads();
    int run = scratch[wave] + inc - sum;
    for (int i = lo; i < hi; ++i) { const int t = v[i]; v[i] = run; run += t; }
    const int total = scratch[32];
    __syncthreads();
    return total;
}

}  // namespace

// ------------------------------------------------------------------------------------
// Tiling shared by the histogram and scatter kernels: a workgroup of WAVES waves (8, or 4
// when the per-wave counters of a wide digit would not fit in LDS) owns `rounds` consecutive
// sub-tiles of 4096 keys.  With one round, wave w owns 4096/WAVES consecutive keys as batches
// of 64, batch j at offset j*64 + lane; with several, the scatter gives each wave `rounds` such
// runs back to back (the histogram only counts, any partition of the tile serves it).  All
// loads of a round are issued before any is used.
constexpr int kSubTile = 4096;

// Keys come back clamped to [0, kmax]; -1 marks a lane past the end of the array.
template <int kBatches>
__device__ __forceinline__ void load_round(const int32_t* __restrict__ keys, int64_t base,
                                           int64_t N, int lane, int kmax, int (&k)[kBatches]) {
#pragma unroll
    for (int j = 0; j < kBatches; ++j) {
        const int64_t i = base + j * 64 + lane;
        k[j] = i < N ? keys[i] : -1;
    }
#pragma unroll
    for (int j = 0; j < kBatches; ++j) {
        const int64_t i = base + j * 64 + lane;
        k[j] = i < N ? clamp_key(k[j], kmax) : -1;
    }
}

// Per-workgroup digit histogram, written transposed: H[b][bin][blk].
template <int kSortWaves>
__global__ __launch_bounds__(kSortWaves * 64) void sort_hist_kernel(
    const int32_t* __restrict__ keys, int32_t* __restrict__ H, int64_t N, int rounds, int NB,
    int shift, int mask, int kmax, int nbits) {
    constexpr int kSortThreads = kSortWaves * 64, kBatches = kSubTile / kSortThreads;
    extern __shared__ int lds[];
    int* hist = lds;
    const int b = blockIdx.y, blk = blockIdx.x, nb = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    keys += (size_t)b * N;
    // Few bins: hot bins would serialise the LDS adds of a wave (lanes hitting one address are
    // processed one after the other), so each group of lanes (lane % 16) counts into its own
    // copy of the histogram and the copies are added at the end.
    const int copies = NB <= 64 ? 16 : 1;
    int* my_hist = hist + (copies > 1 ? (lane & 15) * NB : 0);
    for (int i = tid; i < NB * copies; i += kSortThreads) hist[i] = 0;
    __syncthreads();
    // rounds are software-pipelined: the next round's keys are requested before this round's
    // are counted
    const int64_t base0 = (int64_t)blk * rounds * kSubTile + wave * (kBatches * 64);
    int k[kBatches], kn[kBatches];
    load_round(keys, base0, N, lane, kmax, k);
    for (int r = 0; r < rounds; ++r) {
        const int64_t nbase = base0 + (int64_t)(r + 1) * kSubTile;
        const bool more = r + 1 < rounds && nbase < N;
        if (more) load_round(keys, nbase, N, lane, kmax, kn);
        // one LDS add per key (cheaper than resolving duplicates with ballots first)
#pragma unroll
        for (int j = 0; j < kBatches; ++j)
            if (k[j] >= 0) atomicAdd(&my_hist[(k[j] >> shift) & mask], 1);
        if (!more) break;
#pragma unroll
        for (int j = 0; j < kBatches; ++j) k[j] = kn[j];
    }
    __syncthreads();
    int32_t* out = H + (size_t)b * NB * nb + blk;
    for (int i = tid; i < NB; i += kSortThreads) {
        int c = 0;
        for (int q = 0; q < copies; ++q) c += hist[q * NB + i];
        out[(size_t)i * nb] = c;
    }
}

// Exclusive scan of H[b][bin][0..nb) in place; tot[b][bin] = row sum.  TPB threads (one wave,
// or the whole workgroup for long rows) share a bin, each owning a contiguous run of entries.
template <int TPB>
__global__ __launch_bounds__(256) void sort_binscan_kernel(int32_t* __restrict__ H,
                                                           int32_t* __restrict__ tot, int nb,
                                                           int NB) {
    __shared__ int wsum[4];
    const int b = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bin = TPB == 64 ? blockIdx.x * 4 + wave : blockIdx.x;
    const int t = TPB == 64 ? lane : threadIdx.x;          // index inside the bin's team
    const bool live = bin < NB;
    int32_t* row = H + ((size_t)b * NB + (live ? bin : 0)) * nb;
    const int per = (nb + TPB - 1) / TPB;
    const int lo = live ? min(nb, t * per) : 0, hi = live ? min(nb, lo + per) : 0;
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += row[i];
    int inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(inc, o);
        if (lane >= o) inc += v;
    }
    int base = 0, total = inc;                             // total valid in lane 63
    if (TPB == 256) {
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        for (int w = 0; w < wave; ++w) base += wsum[w];
        total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
        if (live && threadIdx.x == 0) tot[(size_t)b * NB + bin] = total;
    } else if (live && lane == 63) {
        tot[(size_t)b * NB + bin] = total;
    }
    int run = base + inc - sum;
    for (int i = lo; i < hi; ++i) {
        const int v = row[i];
        row[i] = run;
        run += v;
    }
}

// Stable scatter.  Waves walk their keys in input order, so equal keys keep their order.
//   vals_in == NULL: values are the key positions (first pass).
//   keys_out may be NULL.  seg_off / item_off are written by workgroup 0 when non-NULL
//   (single-pass sort: bins are cluster ids, so the bin offsets are the segment table).
template <int kSortWaves>
__global__ __launch_bounds__(kSortWaves * 64) void sort_scatter_kernel(
    const int32_t* __restrict__ keys, const int32_t* __restrict__ vals_in,
    const int32_t* __restrict__ H, const int32_t* __restrict__ tot,
    int32_t* __restrict__ vals_out, int32_t* __restrict__ keys_out,
    int32_t* __restrict__ seg_off, int32_t* __restrict__ item_off, int64_t N, int rounds,
    int NB, int shift, int mask, int kmax, int nbits, int R, int staged, int solo) {
    constexpr int kSortThreads = kSortWaves * 64, kBatches = kSubTile / kSortThreads;
    extern __shared__ int lds[];
    int* off = lds;                    // [NB]
    int* scratch = off + NB;           // [40]
    int* wcnt = scratch + 40;          // [kSortWaves][NB]
    // staged only: [NB] bin starts, then the tile's keys and values in sorted order
    int* gdel = wcnt + kSortWaves * NB;
    int* skey = gdel + NB;
    int* sval = skey + kSubTile;
    const int b = blockIdx.y, blk = blockIdx.x, nb = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    keys += (size_t)b * N;
    if (vals_in) vals_in += (size_t)b * N;
    vals_out += (size_t)b * N;
    if (keys_out) keys_out += (size_t)b * N;
    tot += (size_t)b * NB;
    H += (size_t)b * NB * nb + blk;

    // first round's keys are requested before the offset scans below need them
    int k[kBatches];
    // a wave owns `rounds` consecutive batches-of-8 (contiguous in the input, so that wave order
    // is input order and the sort stays stable with several rounds)
    const int64_t base0 = (int64_t)blk * rounds * kSubTile + (int64_t)wave * rounds * (kBatches * 64);
    constexpr int kRoundStep = kBatches * 64;
    load_round(keys, base0, N, lane, kmax, k);
    // this workgroup's column of the scanned histogram table (one entry per bin, a cache line
    // apart): requested now, needed only after the counting pass
    constexpr int kHPer = 2048 / kSortThreads;
    int hcol[kHPer];
#pragma unroll
    for (int q = 0; q < kHPer; ++q) {
        const int i = tid + q * kSortThreads;
        hcol[q] = (!solo && i < NB) ? H[(size_t)i * nb] : 0;
    }

    // Bin totals -> off[] (exclusive scan: where each bin starts in the output), plus the
    // segment and item tables when asked for.  The totals come from the scan kernel, or, when
    // one workgroup sorts the whole instance (solo), from its own per-wave counts after the
    // counting pass -- no histogram or scan kernel runs then.
    auto offsets_from_totals = [&]() {
        auto total_of = [&](int i) -> int {
            if (!solo) return tot[i];
            int t = 0;
            for (int w = 0; w < kSortWaves; ++w) t += wcnt[w * NB + i];
            return t;
        };
        if (item_off && blk == 0) {
            // exclusive scan of ceil(n_k / R): where each cluster's items start
            for (int i = tid; i < NB; i += kSortThreads) off[i] = (total_of(i) + R - 1) / R;
            __syncthreads();
            const int items = block_exclusive_scan(off, NB, scratch);
            int32_t* io = item_off + (size_t)b * (NB + 1);
            for (int i = tid; i < NB; i += kSortThreads) io[i] = off[i];
            if (tid == 0) io[NB] = items;
            __syncthreads();
        }
        for (int i = tid; i < NB; i += kSortThreads) off[i] = total_of(i);
        __syncthreads();
        const int total = block_exclusive_scan(off, NB, scratch);
        if (seg_off && blk == 0) {
            int32_t* so = seg_off + (size_t)b * (NB + 1);
            for (int i = tid; i < NB; i += kSortThreads) so[i] = off[i];
            if (tid == 0) so[NB] = total;
        }
    };
    for (int i = tid; i < kSortWaves * NB; i += kSortThreads) wcnt[i] = 0;
    __syncthreads();
    if (!solo) offsets_from_totals();

    int* mine = wcnt + wave * NB;
    const uint64_t lt = lanemask_lt();
    // info[j] = rank among equal digits of the batch | (size of that group << 8)
    int info[kBatches];

    if (rounds == 1) {
        // Keys, ranks and each key's position inside its wave's run of the digit stay in
        // registers between the two passes.  Pass 1: every lane reads the wave's running count
        // of its digit, then the first lane of each group of equal digits adds the group's
        // size; LDS executes a wave's operations in order, so the eight batches need no wait
        // between them.
        int pre[kBatches];
#pragma unroll
        for (int j = 0; j < kBatches; ++j) {
            const bool valid = k[j] >= 0;
            const int digit = valid ? (k[j] >> shift) & mask : 0;
            const uint64_t peers = match_digit(digit, nbits, __ballot(valid));
            const int rank = __popcll(peers & lt), cnt = __popcll(peers);
            info[j] = rank;
            pre[j] = valid ? mine[digit] : 0;
            __builtin_amdgcn_wave_barrier();
            if (valid && rank == 0) atomicAdd(&mine[digit], cnt);
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        if (solo) offsets_from_totals();
        int v[kBatches];
        if (vals_in) {
#pragma unroll
            for (int j = 0; j < kBatches; ++j) {
                const int64_t i = base0 + j * 64 + lane;
                v[j] = i < N ? vals_in[i] : 0;
            }
        }
        if (staged) {
            // Few bins, long runs: the tile is first put in sorted order in LDS and then
            // written by consecutive threads, so that a store instruction covers a few
            // contiguous runs instead of 64 scattered words.
            for (int i = tid; i < NB; i += kSortThreads) {
                int run = 0;
                for (int w = 0; w < kSortWaves; ++w) {
                    const int t = wcnt[w * NB + i];
                    wcnt[w * NB + i] = run;           // where wave w's run starts inside the bin's
                    run += t;
                }
                gdel[i] = run;                        // the tile's count of bin i
            }
            __syncthreads();
            block_exclusive_scan(gdel, NB, scratch);  // -> where bin i starts inside the tile
#pragma unroll
            for (int j = 0; j < kBatches; ++j) {
                if (k[j] >= 0) {
                    const int digit = (k[j] >> shift) & mask;
                    const int lp = gdel[digit] + mine[digit] + pre[j] + info[j];
                    skey[lp] = k[j];
                    sval[lp] = vals_in ? v[j] : (int32_t)(base0 + j * 64 + lane);
                }
            }
            __syncthreads();
            // global position = position in the tile + (global start of the tile's run of the bin
            // - its start inside the tile)
#pragma unroll
            for (int q = 0; q < kHPer; ++q) {
                const int i = tid + q * kSortThreads;
                if (i < NB) gdel[i] = off[i] + hcol[q] - gdel[i];
            }
            __syncthreads();
            const int64_t tile0 = (int64_t)blk * kSubTile;
            const int live = (int)min((int64_t)kSubTile, N - tile0);
            for (int i = tid; i < live; i += kSortThreads) {
                const int key = skey[i];
                const int pos = i + gdel[(key >> shift) & mask];
                vals_out[pos] = sval[i];
                if (keys_out) keys_out[pos] = key;
            }
            return;
        }
        // counts -> start positions: global bin offset + earlier workgroups + earlier waves
#pragma unroll
        for (int q = 0; q < kHPer; ++q) {
            const int i = tid + q * kSortThreads;
            if (i < NB) {
                int run = off[i] + hcol[q];
                for (int w = 0; w < kSortWaves; ++w) {
                    const int t = wcnt[w * NB + i];
                    wcnt[w * NB + i] = run;
                    run += t;
                }
            }
        }
        __syncthreads();
        // pass 2: position = start of the wave's run + position inside the run
        int start[kBatches];
#pragma unroll
        for (int j = 0; j < kBatches; ++j) start[j] = k[j] >= 0 ? mine[(k[j] >> shift) & mask] : 0;
#pragma unroll
        for (int j = 0; j < kBatches; ++j) {
            if (k[j] >= 0) {
                const int pos = start[j] + pre[j] + info[j];
                vals_out[pos] = vals_in ? v[j] : (int32_t)(base0 + j * 64 + lane);
                if (keys_out) keys_out[pos] = k[j];
            }
        }
        return;
    }

    // More than one round per workgroup (beyond 16M keys per instance): ranks are recomputed
    // in the second pass and the wave's cursors advance batch by batch.
    auto rank_round = [&](bool count) {
#pragma unroll
        for (int j = 0; j < kBatches; ++j) {
            const bool valid = k[j] >= 0;
            const int digit = valid ? (k[j] >> shift) & mask : 0;
            const uint64_t peers = match_digit(digit, nbits, __ballot(valid));
            const int rank = __popcll(peers & lt), cnt = __popcll(peers);
            info[j] = rank | (cnt << 8);
            if (count && valid && rank == 0) mine[digit] += cnt;
            __builtin_amdgcn_wave_barrier();
        }
    };
    // pass 1: per-wave digit counts
    rank_round(true);
    for (int r = 1; r < rounds; ++r) {
        const int64_t base = base0 + (int64_t)r * kRoundStep;
        if (base >= N) break;
        load_round(keys, base, N, lane, kmax, k);
        rank_round(true);
    }
    __syncthreads();
    if (solo) offsets_from_totals();
    // counts -> start positions: global bin offset + earlier workgroups + earlier waves
#pragma unroll
    for (int q = 0; q < kHPer; ++q) {
        const int i = tid + q * kSortThreads;
        if (i < NB) {
            int run = off[i] + hcol[q];
            for (int w = 0; w < kSortWaves; ++w) {
                const int t = wcnt[w * NB + i];
                wcnt[w * NB + i] = run;
                run += t;
            }
        }
    }
    __syncthreads();
    // pass 2: write, advancing the wave's cursors batch by batch
    for (int r = 0; r < rounds; ++r) {
        const int64_t base = base0 + (int64_t)r * kRoundStep;
        if (base >= N) break;
        load_round(keys, base, N, lane, kmax, k);
        rank_round(false);
        int v[kBatches];
        if (vals_in) {
#pragma unroll
            for (int j = 0; j < kBatches; ++j) {
                const int64_t i = base + j * 64 + lane;
                v[j] = i < N ? vals_in[i] : 0;
            }
        }
#pragma unroll
        for (int j = 0; j < kBatches; ++j) {
            const bool valid = k[j] >= 0;
            const int key = valid ? k[j] : 0;
            const int digit = (key >> shift) & mask;
            const int rank = info[j] & 255, cnt = info[j] >> 8;
            int pos = 0;
            if (valid) pos = mine[digit] + rank;
            __builtin_amdgcn_wave_barrier();
            if (valid) {
                vals_out[pos] = vals_in ? v[j] : (int32_t)(base + j * 64 + lane);
                if (keys_out) keys_out[pos] = key;
                if (rank == 0) mine[digit] += cnt;
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// Two-pass sort only: segment table from the sorted id sequence.  Position j opens the
// segments of every id in (ks[j-1], ks[j]]; ids above the last key get N.
__global__ void sort_boundaries_kernel(const int32_t* __restrict__ ks,
                                       int32_t* __restrict__ seg_off, int64_t N, int K) {
    const int b = blockIdx.y;
    ks += (size_t)b * N;
    seg_off += (size_t)b * (K + 1);
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    const int cur = ks[j];
    const int prev = j == 0 ? -1 : ks[j - 1];
    for (int k = prev + 1; k <= cur; ++k) seg_off[k] = (int32_t)j;
    if (j == N - 1)
        for (int k = cur + 1; k <= K; ++k) seg_off[k] = (int32_t)N;
}

// Two-pass sort only: item_off = exclusive scan of ceil(n_k / R) for K up to 65536.
__global__ __launch_bounds__(1024) void item_offsets_kernel(const int32_t* __restrict__ seg_off,
                                                            int32_t* __restrict__ item_off,
                                                            int K, int R) {
    __shared__ int sc[1024 + 40];
    const int b = blockIdx.x;
    seg_off += (size_t)b * (K + 1);
    item_off += (size_t)b * (K + 1);
    const int per = (K + 1023) / 1024;
    const int lo = min(K, (int)threadIdx.x * per), hi = min(K, lo + per);
    int sum = 0;
    for (int k = lo; k < hi; ++k) sum += (seg_off[k + 1] - seg_off[k] + R - 1) / R;
    sc[threadIdx.x] = sum;
    __syncthreads();
    const int total = block_exclusive_scan(sc, 1024, sc + 1024);
    int run = sc[threadIdx.x];
    for (int k = lo; k < hi; ++k) {
        item_off[k] = run;
        run += (seg_off[k + 1] - seg_off[k] + R - 1) / R;
    }
    if (threadIdx.x == 0) item_off[K] = total;
}

// ------------------------------------------------------------------------------------
static int ceil_log2(int v) {
    int b = 0;
    while ((1 << b) < v) ++b;
    return b;
}

// upper limit of the LDS-staged scatter, in bins (fk_set_option("sort_stage_bins"); 0 = never)
static std::atomic<int> g_stage_max_bins{1024};

void set_sort_stage_bins(int v) { g_stage_max_bins.store(v < 0 ? 1024 : v, std::memory_order_relaxed); }

static fk_status sort_pass(const Geometry& g, const Workspace& w, const int32_t* keys,
                           const int32_t* vals_in, int32_t* vals_out, int32_t* keys_out,
                           int32_t* seg_off, int32_t* item_off, int NB, int shift, int mask,
                           hipStream_t s) {
    const int nbits = ceil_log2(NB) < 1 ? 1 : ceil_log2(NB);
    const int rounds = g.sort_tile / kSubTile;
    int32_t* H = w.block_hist;
    int32_t* tot = w.digit_off;
    dim3 grid(g.sort_blocks, g.B);
    const bool wide = NB > 1024;       // 8 waves of counters would not fit in LDS
    // one workgroup per instance: the scatter kernel counts for itself
    const int solo = g.sort_blocks == 1 ? 1 : 0;
    if (!solo) {
        const size_t hist_lds = (size_t)NB * (NB <= 64 ? 16 : 1) * sizeof(int);
        if (wide)
            hipLaunchKernelGGL(sort_hist_kernel<4>, grid, dim3(256), hist_lds, s, keys, H, g.N,
                               rounds, NB, shift, mask, g.K - 1, nbits);
        else
            hipLaunchKernelGGL(sort_hist_kernel<8>, grid, dim3(512), hist_lds, s, keys, H, g.N,
                               rounds, NB, shift, mask, g.K - 1, nbits);
        FK_HIP(hipGetLastError());
        if (g.sort_blocks > 512)
            hipLaunchKernelGGL(sort_binscan_kernel<256>, dim3((unsigned)NB, g.B), dim3(256), 0, s, H,
                               tot, g.sort_blocks, NB);
        else
            hipLaunchKernelGGL(sort_binscan_kernel<64>, dim3((unsigned)cdiv(NB, 4), g.B), dim3(256), 0,
                               s, H, tot, g.sort_blocks, NB);
        FK_HIP(hipGetLastError());
    }
    const int waves = wide ? 4 : 8;
    // One tile per workgroup: sorted in LDS first, then written in contiguous runs.  Measured
    // (2^20 .. 2^25 keys): pays from 32 bins (below that a wave's stores already fall into few
    // runs) up to 1024 (beyond, the LDS footprint costs more than the runs, 1-2 keys, give);
    // 2x on the 64..256-bin passes of the two-pass sort.
    const int staged = rounds == 1 && NB >= 32 && NB <= g_stage_max_bins.load(std::memory_order_relaxed) ? 1 : 0;
    const size_t lds = (size_t)(NB + 40 + waves * NB + (staged ? NB + 2 * kSubTile : 0)) * sizeof(int);
    if (lds > 64 * 1024) {
        static PerDeviceInt attr_set[2];
        if (!attr_set[wide].get()) {
            FK_HIP(hipFuncSetAttribute(wide ? (const void*)sort_scatter_kernel<4> : (const void*)sort_scatter_kernel<8>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
            attr_set[wide].set(1);
        }
    }
    if (wide)
        hipLaunchKernelGGL(sort_scatter_kernel<4>, grid, dim3(256), lds, s, keys, vals_in, H, tot,
                           vals_out, keys_out, seg_off, item_off, g.N, rounds, NB, shift, mask,
                           g.K - 1, nbits, g.rows_per_item, staged, solo);
    else
        hipLaunchKernelGGL(sort_scatter_kernel<8>, grid, dim3(512), lds, s, keys, vals_in, H, tot,
                           vals_out, keys_out, seg_off, item_off, g.N, rounds, NB, shift, mask,
                           g.K - 1, nbits, g.rows_per_item, staged, solo);
    FK_HIP(hipGetLastError());
    return FK_OK;
}

fk_status launch_sort_inverse(const Geometry& g, const Workspace& w, const int32_t* assign,
                              int32_t* sorted_idx, int32_t* seg_off, int32_t* item_off,
                              hipStream_t s) {
    if (g.sort_passes == 1)
        return sort_pass(g, w, assign, nullptr, sorted_idx, nullptr, seg_off, item_off, g.K, 0,
                         0x7FFFFFFF, s);
    const int lb = g.pass_bits[0], hb = g.pass_bits[1];
    fk_status st = sort_pass(g, w, assign, nullptr, w.vals_tmp, w.keys_tmp, nullptr, nullptr,
                             1 << lb, 0, (1 << lb) - 1, s);
    if (st != FK_OK) return st;
    st = sort_pass(g, w, w.keys_tmp, w.vals_tmp, sorted_idx, w.keys_sorted, nullptr, nullptr,
                   1 << hb, lb, (1 << hb) - 1, s);
    if (st != FK_OK) return st;
    hipLaunchKernelGGL(sort_boundaries_kernel, dim3((unsigned)cdiv(g.N, 256), g.B), dim3(256), 0,
                       s, w.keys_sorted, seg_off, g.N, g.K);
    FK_HIP(hipGetLastError());
    if (item_off) {
        hipLaunchKernelGGL(item_offsets_kernel, dim3(g.B), dim3(1024), 0, s, seg_off, item_off,
                           g.K, g.rows_per_item);
        FK_HIP(hipGetLastError());
    }
    return FK_OK;
}

}  // namespace fk
