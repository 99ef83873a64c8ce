// Internal declarations shared by the flashkm translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "flashkm.h"

namespace fk {

// ---------------------------------------------------------------- errors
void set_error(const char* fmt, ...);
fk_status hip_fail(hipError_t e, const char* what);

#define FK_HIP(call)                                           \
    do {                                                       \
        hipError_t _e = (call);                                \
        if (_e != hipSuccess) return fk::hip_fail(_e, #call);  \
    } while (0)

#define FK_TRY(expr)                       \
    do {                                   \
        fk_status _s = (expr);             \
        if (_s != FK_OK) return _s;        \
    } while (0)

// ---------------------------------------------------------------- small helpers
constexpr int kWave = 64;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t elem_size(fk_dtype t) { return t == FK_F32 ? 4 : 2; }
// What the host-side choices need to know about the current device, asked of the runtime once
// per device: compute units, LDS per compute unit, and the size of the last-level cache (the
// largest cache the HSA runtime lists for the agent; the L2 size HIP reports if that fails).
// With no GPU in the process: 256 units, 160 KiB, 256 MiB (MI355X).
struct DeviceInfo {
    int cus;
    int64_t lds_bytes;
    int64_t llc_bytes;
};
constexpr int kMaxDevices = 64;
int current_device();                 // ordinal of the current HIP device, 0 if there is none
const DeviceInfo& device_info();
inline int device_cu_count() { return device_info().cus; }

// A value remembered per device (kernel attributes set, occupancy queried): 0 = not yet known.
// Racing first calls compute the same value twice, which is harmless.
struct PerDeviceInt {
    std::atomic<int> v[kMaxDevices];
    int get() const { return v[current_device()].load(std::memory_order_relaxed); }
    void set(int x) { v[current_device()].store(x, std::memory_order_relaxed); }
};

// ---------------------------------------------------------------- problem geometry
//
// Centroids for the MFMA path are kept in "fragment order": centroid tile (32 rows) x
// feature chunk (16 features) x lane (64) x 8 elements, so that a 32x32x16 MFMA A-operand
// is one 16-byte LDS read per lane at lane*16.  Rows beyond K and features beyond d are
// zero; their score bias is -inf so they never win.
struct Geometry {
    int B;
    int64_t N;        // points per instance
    int d, K;         // d: row width the kernels see (a multiple of 8)
    int d_user;       // row width of the caller's arrays; when it differs from d, X and C are
                      // first copied into zero-padded rows of width d (zeros change no distance
                      // and no mean) and the centroids copied back without the padding
    fk_dtype t;
    int dchunks;      // ceil(d / 16)
    int ktiles;       // ceil(K / 32)
    // counting sort
    int sort_bits;    // bits of a cluster id, ceil(log2 K), >= 1
    int sort_passes;  // 1 when K <= 2048, else 2
    int pass_bits[2];
    int sort_tile;    // keys per sort workgroup
    int sort_blocks;  // workgroups per instance = ceil(N / sort_tile)
    // segment reduction
    int rows_per_item;   // R: sorted positions reduced into one partial row
    int waves_per_item;  // 1, or 4 (a whole workgroup) for the long items of few-cluster shapes
    int64_t max_items;   // upper bound on sum_k ceil(n_k / R) per instance
    // sort-free update for few clusters (16-bit storage, K <= 32, d <= 128): most workgroups
    // per instance it may use, 0 when the shape is not eligible
    int fused_grid_cap;
    // one-pass update with the K x d table split over the registers of a workgroup (16-bit
    // storage, 32 < K <= 256, d <= 128): most workgroups per instance, 0 when not eligible
    int table_grid_cap;
    // one-pass assignment + sums for small fp32 problems (K <= 64, d <= 128, at most 2^17 points
    // in all; see fk_f32_fused.hip): most workgroups per instance, 0 when not eligible
    int f32_grid_cap;
};

// Carved device workspace (all pointers 256-byte aligned inside the caller's buffer).
struct Workspace {
    void* c_lp;          // [B,K,d] low-precision centroids consumed by assign (lloyd only)
    void* c_frag;        // [B,ktiles,dchunks,64,8] fragment-ordered centroids (16-bit types)
    float* c_bias;       // [B,ktiles*32] -||c||^2/2, -inf for padding rows
    int32_t* sorted_idx; // [B,N]
    int32_t* seg_off;    // [B,K+1]
    int32_t* item_off;   // [B,K+1] exclusive scan of ceil(n_k / R)
    int32_t* block_hist; // [B,bins,sort_blocks] per-workgroup digit histograms
    int32_t* digit_off;  // [B,2048+1] digit offsets of the current radix pass
    int32_t* keys_tmp;   // [B,N] keys after pass 1 (two-pass sort only)
    int32_t* vals_tmp;   // [B,N] values after pass 1 (two-pass sort only)
    int32_t* keys_sorted;// [B,N] sorted keys (two-pass sort only)
    float* partial;      // [B,max(max_items, K*(largest one-pass grid cap)),d] per-item segment sums
    int32_t* wg_counts;  // [B,K,grid cap] per-workgroup counts (one-pass updates only)
    float* sums;         // [B,K,d] accumulated sums (chunked mode)
    void* x_pad;         // [B,N,d] zero-padded copy of X            (only when d != d_user)
    float* c_pad_f32;    // [B,K,d] zero-padded fp32 centroids       (only when d != d_user)
    void* c_pad_lp;      // [B,K,d] zero-padded centroids, dtype t   (only when d != d_user)
    size_t bytes;        // total bytes carved
};

bool make_geometry(int B, int64_t N, int d, int K, fk_dtype t, Geometry* g);
// Lays the workspace out from `base` (may be NULL to only compute the size).  padded_x = false
// leaves out the zero-padded copy of X (the out-of-core call pads through its pitched copies).
Workspace carve(const Geometry& g, void* base, bool padded_x = true);

// ---------------------------------------------------------------- kernel launchers
// Each enqueues on `s` and returns FK_OK / FK_EHIP.  Pointers are device pointers.

// C (dtype t, [B,K,d]) -> fragment-ordered copy + score bias.  16-bit types only.
fk_status launch_prepare_centroids(const Geometry& g, const void* C_lp, void* c_frag,
                                   float* c_bias, hipStream_t s);
// C_f32 -> C_lp (round to nearest even), and for 16-bit types also c_frag / c_bias.
fk_status launch_round_centroids(const Geometry& g, const float* C_f32, void* C_lp,
                                 void* c_frag, float* c_bias, hipStream_t s);
// Fused distance + online argmin.  16-bit: reads c_frag/c_bias; fp32: reads C directly.
fk_status launch_assign(const Geometry& g, const void* X, const void* C_or_frag,
                        const float* c_bias, int32_t* assign, float* min_dist, hipStream_t s);
// Tile shape the sweeping assign kernel would use for this problem (see fk_assign.hip).
int choose_assign_variant(const Geometry& g);
void set_assign_variant_override(int v);   // -1 = choose from the shape
// Few centroids: persistent streaming kernel instead of the sweeping one (see fk_assign.hip).
bool assign_uses_stream_kernel(const Geometry& g);
void set_assign_stream_option(int v);      // -1 = by shape, 0 = never, 1 = whenever eligible
// Stable argsort by cluster id -> sorted_idx, seg_off (+ item_off when w.item_off != NULL).
fk_status launch_sort_inverse(const Geometry& g, const Workspace& w, const int32_t* assign,
                              int32_t* sorted_idx, int32_t* seg_off, int32_t* item_off,
                              hipStream_t s);
// Largest bin count for which the scatter stages its tile through LDS (-1 = the built-in 1024).
void set_sort_stage_bins(int v);
// Per-item segment sums of gathered rows -> w.partial.
fk_status launch_segment_reduce(const Geometry& g, const Workspace& w, const void* X,
                                const int32_t* sorted_idx, const int32_t* seg_off,
                                const int32_t* item_off, hipStream_t s);
// Merge item sums per cluster; optionally accumulate into sums/counts; optionally
// normalise and emit centroids (fp32 master, rounded copy, fragment copy, bias).
struct FinalizeArgs {
    const float* C_prev_f32;
    float* C_out_f32;
    void* C_out_lp;      // may be NULL
    void* c_frag;        // may be NULL
    float* c_bias;       // may be NULL
    int32_t* counts;     // [B,K]
    float* sums;         // [B,K,d] (needed when accumulate || !normalise)
    bool accumulate;     // add onto sums / counts already there
    bool normalise;      // divide and write centroids
};
// With wg_counts (few-cluster path) cluster k owns partial rows [k*G, (k+1)*G) and the counts
// wg_counts[b][k][0..G) instead of what seg_off / item_off say (those may then be NULL).
fk_status launch_finalize(const Geometry& g, const Workspace& w, const int32_t* seg_off,
                          const int32_t* item_off, const FinalizeArgs& a, hipStream_t s,
                          const int32_t* wg_counts = nullptr, int wg_per_cluster = 0);

// Few clusters: stream X once, add every 32-point batch into per-workgroup K x d tables with a
// one-hot MFMA (no sort, no gather); with compute_assign the assignment is computed (and
// written) in the same pass, otherwise read.  Leaves w.partial / w.wg_counts ready for
// launch_finalize with max_items = K * (*grid_out) and wg_per_cluster = *grid_out.
fk_status launch_stream_update(const Geometry& g, const Workspace& w, const void* X,
                               int32_t* assign, bool compute_assign, int* grid_out,
                               hipStream_t s);
bool fused_update_enabled(const Geometry& g);
void set_fused_update_option(int v);       // 0 = never, otherwise whenever the shape allows
bool fused_update_allowed();               // the option above is not 0

// Up to 256 clusters: assignment and sums in one pass over X with the table of sums in the
// registers of a persistent workgroup (see fk_table.hip).  Computes and writes the assignment;
// leaves w.partial / w.wg_counts as launch_stream_update does.
fk_status launch_table_update(const Geometry& g, const Workspace& w, const void* X,
                              int32_t* assign, int* grid_out, hipStream_t s);
bool table_update_enabled(const Geometry& g);

// Small fp32 problems, up to 64 clusters: assignment and sums in one pass over X (see
// fk_f32_fused.hip).  C_f32 [B,K,d] are the centroids to assign against.  Computes and writes the
// assignment; leaves w.partial / w.wg_counts as launch_stream_update does.
fk_status launch_f32_update(const Geometry& g, const Workspace& w, const void* X,
                            const float* C_f32, int32_t* assign, int* grid_out, hipStream_t s);
bool f32_update_enabled(const Geometry& g);

// Row re-layout for widths that are not a multiple of 8: dst[r][j] = j < d_src ? src[r][j] : 0
// for j < d_dst (padding, d_dst > d_src) or dst[r][j] = src[r][j] for j < d_dst (un-padding,
// d_dst < d_src).  elem = bytes per element (2 or 4).
fk_status launch_copy_rows(const void* src, void* dst, int64_t rows, int d_src, int d_dst,
                           int elem, hipStream_t s);

// Comparator: the standard implementation (paper Algorithm 1); see fk_standard.hip.
fk_status launch_standard_assign(const Geometry& g, const Workspace& w, const void* X,
                                 const void* C_lp, float* D, int32_t* assign, hipStream_t s);
fk_status launch_standard_update(const Geometry& g, const void* X, const int32_t* assign,
                                 const float* C_prev, float* C_out, int32_t* counts, float* sums,
                                 hipStream_t s);

}  // namespace fk
