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
#include "fk_common.h"

namespace fk {

namespace {

__device__ __forceinline__ int clamp_key(int k, int kmax) { return min(max(k, 0), kmax); }

// Lanes of the wave whose `digit` equals this lane's, among lanes in `valid`.
__device__ __forceinline__ uint64_t match_digit(int digit, int nbits, uint64_t valid) {
    uint64_t peers = valid;
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (digit >> b) & 1;
        const uint64_t bal = __ballot(bit);
        peers &= bit ? bal : ~bal;
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
// Per-workgroup digit histogram.  Workgroup `blk` of instance b owns keys
// [blk*T, min(N,(blk+1)*T)); writes H[b][blk][0..NB).
__global__ __launch_bounds__(1024) void sort_hist_kernel(
    const int32_t* __restrict__ keys, int32_t* __restrict__ H, int64_t N, int T, int NB,
    int shift, int mask, int kmax, int nbits) {
    extern __shared__ int lds[];
    int* hist = lds;
    const int b = blockIdx.y, blk = blockIdx.x, nb = gridDim.x;
    keys += (size_t)b * N;
    for (int i = threadIdx.x; i < NB; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    const int64_t lo = (int64_t)blk * T, hi = min(N, lo + T);
    for (int64_t i0 = lo; i0 < hi; i0 += blockDim.x) {
        const int64_t i = i0 + threadIdx.x;
        const bool valid = i < hi;
        const int digit = valid ? (clamp_key(keys[i], kmax) >> shift) & mask : 0;
        const uint64_t peers = match_digit(digit, nbits, __ballot(valid));
        // one LDS add per distinct digit per wave keeps hot bins from serialising
        if (valid && (peers & lanemask_lt()) == 0) atomicAdd(&hist[digit], __popcll(peers));
    }
    __syncthreads();
    int32_t* out = H + ((size_t)b * nb + blk) * NB;
    for (int i = threadIdx.x; i < NB; i += blockDim.x) out[i] = hist[i];
}

// Exclusive scan of H along the workgroup axis, per bin, in place; tot[b][bin] = column sum.
// A workgroup of 256 threads covers BG bins x (256/BG) contiguous ranges of workgroups.
__global__ __launch_bounds__(256) void sort_binscan_kernel(int32_t* __restrict__ H,
                                                           int32_t* __restrict__ tot, int nb,
                                                           int NB, int bg_log2) {
    __shared__ int ssum[256];
    const int b = blockIdx.y;
    const int BG = 1 << bg_log2, SEG = 256 >> bg_log2;
    const int binl = threadIdx.x & (BG - 1), seg = threadIdx.x >> bg_log2;
    const int bin = blockIdx.x * BG + binl;
    const int per = (nb + SEG - 1) / SEG;
    const int lo = min(nb, seg * per), hi = min(nb, lo + per);
    int32_t* col = H + (size_t)b * nb * NB + bin;
    int sum = 0;
    if (bin < NB)
        for (int r = lo; r < hi; ++r) sum += col[(size_t)r * NB];
    ssum[threadIdx.x] = sum;
    __syncthreads();
    int run = 0;
    for (int s2 = 0; s2 < seg; ++s2) run += ssum[(s2 << bg_log2) + binl];
    if (bin < NB) {
        if (seg == SEG - 1) tot[(size_t)b * NB + bin] = run + sum;
        for (int r = lo; r < hi; ++r) {
            const int t = col[(size_t)r * NB];
            col[(size_t)r * NB] = run;
            run += t;
        }
    }
}

// Stable scatter.  Each wave owns a contiguous sub-range of the workgroup's keys and walks
// it in order, so equal keys keep their input order.
//   vals_in == NULL: values are the key positions (first pass).
//   keys_out may be NULL.  seg_off / item_off are written by workgroup 0 when non-NULL
//   (single-pass sort: bins are cluster ids, so the bin offsets are the segment table).
__global__ __launch_bounds__(1024) void sort_scatter_kernel(
    const int32_t* __restrict__ keys, const int32_t* __restrict__ vals_in,
    const int32_t* __restrict__ H, const int32_t* __restrict__ tot,
    int32_t* __restrict__ vals_out, int32_t* __restrict__ keys_out,
    int32_t* __restrict__ seg_off, int32_t* __restrict__ item_off, int64_t N, int T, int NB,
    int shift, int mask, int kmax, int nbits, int R) {
    extern __shared__ int lds[];
    const int waves = blockDim.x >> 6;
    int* off = lds;                    // [NB]
    int* scratch = off + NB;           // [40]
    int* wcnt = scratch + 40;          // [waves][NB]
    const int b = blockIdx.y, blk = blockIdx.x, nb = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    keys += (size_t)b * N;
    if (vals_in) vals_in += (size_t)b * N;
    vals_out += (size_t)b * N;
    if (keys_out) keys_out += (size_t)b * N;
    tot += (size_t)b * NB;
    H += ((size_t)b * nb + blk) * NB;

    if (item_off && blk == 0) {
        // exclusive scan of ceil(n_k / R): where each cluster's items start
        for (int i = tid; i < NB; i += blockDim.x) off[i] = (tot[i] + R - 1) / R;
        __syncthreads();
        const int total = block_exclusive_scan(off, NB, scratch);
        int32_t* io = item_off + (size_t)b * (NB + 1);
        for (int i = tid; i < NB; i += blockDim.x) io[i] = off[i];
        if (tid == 0) io[NB] = total;
        __syncthreads();
    }
    for (int i = tid; i < NB; i += blockDim.x) off[i] = tot[i];
    for (int i = tid; i < waves * NB; i += blockDim.x) wcnt[i] = 0;
    __syncthreads();
    const int total = block_exclusive_scan(off, NB, scratch);
    if (seg_off && blk == 0) {
        int32_t* so = seg_off + (size_t)b * (NB + 1);
        for (int i = tid; i < NB; i += blockDim.x) so[i] = off[i];
        if (tid == 0) so[NB] = total;
    }

    const int tw = T / waves;          // keys per wave, a multiple of 64
    const int64_t lo = (int64_t)blk * T + (int64_t)wave * tw;
    const int64_t hi = min(N, lo + tw);
    int* mine = wcnt + wave * NB;
    // pass 1: count this wave's digits
    for (int64_t i0 = lo; i0 < hi; i0 += 64) {
        const int64_t i = i0 + lane;
        const bool valid = i < hi;
        const int digit = valid ? (clamp_key(keys[i], kmax) >> shift) & mask : 0;
        const uint64_t peers = match_digit(digit, nbits, __ballot(valid));
        if (valid && (peers & lanemask_lt()) == 0) mine[digit] += __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // turn counts into start positions: global bin offset + earlier workgroups + earlier waves
    for (int i = tid; i < NB; i += blockDim.x) {
        int run = off[i] + H[i];
        for (int w = 0; w < waves; ++w) {
            const int t = wcnt[w * NB + i];
            wcnt[w * NB + i] = run;
            run += t;
        }
    }
    __syncthreads();
    // pass 2: rank inside each 64-key batch, write, advance the wave's cursors
    for (int64_t i0 = lo; i0 < hi; i0 += 64) {
        const int64_t i = i0 + lane;
        const bool valid = i < hi;
        const int key = valid ? clamp_key(keys[i], kmax) : 0;
        const int digit = (key >> shift) & mask;
        const uint64_t peers = match_digit(digit, nbits, __ballot(valid));
        const int rank = __popcll(peers & lanemask_lt());
        int pos = 0;
        if (valid) pos = mine[digit] + rank;
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            vals_out[pos] = vals_in ? vals_in[i] : (int32_t)i;
            if (keys_out) keys_out[pos] = key;
            if (rank == 0) mine[digit] += __popcll(peers);
        }
        __builtin_amdgcn_wave_barrier();
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

static fk_status sort_pass(const Geometry& g, const Workspace& w, const int32_t* keys,
                           const int32_t* vals_in, int32_t* vals_out, int32_t* keys_out,
                           int32_t* seg_off, int32_t* item_off, int NB, int shift, int mask,
                           hipStream_t s) {
    const int nbits = ceil_log2(NB) < 1 ? 1 : ceil_log2(NB);
    const int waves = NB <= 512 ? 16 : (NB <= 1024 ? 8 : 4);
    const int threads = waves * 64;
    int32_t* H = w.block_hist;
    int32_t* tot = w.digit_off;
    dim3 grid(g.sort_blocks, g.B);
    hipLaunchKernelGGL(sort_hist_kernel, grid, dim3(1024), NB * sizeof(int), s, keys, H, g.N,
                       g.sort_tile, NB, shift, mask, g.K - 1, nbits);
    FK_HIP(hipGetLastError());
    int bg_log2 = ceil_log2(NB);
    if (bg_log2 > 6) bg_log2 = 6;
    hipLaunchKernelGGL(sort_binscan_kernel, dim3((unsigned)cdiv(NB, 1 << bg_log2), g.B),
                       dim3(256), 0, s, H, tot, g.sort_blocks, NB, bg_log2);
    FK_HIP(hipGetLastError());
    const size_t lds = (size_t)(NB + 40 + waves * NB) * sizeof(int);
    hipLaunchKernelGGL(sort_scatter_kernel, grid, dim3(threads), lds, s, keys, vals_in, H, tot,
                       vals_out, keys_out, seg_off, item_off, g.N, g.sort_tile, NB, shift, mask,
                       g.K - 1, nbits, g.rows_per_item);
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
