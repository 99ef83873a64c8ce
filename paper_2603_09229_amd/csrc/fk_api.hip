// C-ABI entry points of flashkm.h: argument checks, workspace carving, kernel sequencing.
// The arithmetic lives in fk_assign.hip / fk_sort.hip / fk_update.hip.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include <hsa/hsa.h>

#include "fk_common.h"

namespace fk {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

fk_status hip_fail(hipError_t e, const char* what) {
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return FK_EHIP;
}

// ---------------------------------------------------------------- stage timer
// Optional HIP-event marks between the stages of an iteration (off by default; one process-
// wide recorder, not thread safe: a measurement aid, not part of the compute path).
enum { kStageAssign = 0, kStageSort = 1, kStageReduce = 2, kStageFinalize = 3, kStages = 4 };
struct StageTimer {
    bool on = false;
    std::vector<hipEvent_t> pool;     // events owned by the recorder, reused across runs
    size_t used = 0;
    std::vector<int> stage;           // stage closed by mark i (-1 = opens an iteration)
    std::vector<int> launches;        // kernel launches of that stage inside the interval
    int repeat = 1;                   // fk_set_option("timer_repeat")
};
static StageTimer g_timer;

// While the recorder runs, the two bandwidth- or MFMA-sized kernels of an iteration (assignment
// or fused pass; segment reduction) are launched this many times back to back inside their
// interval: they only read their inputs and rewrite the same outputs, so the result does not
// change, and interval / launches then approaches the kernel's own duration (the events' cost
// is paid once per interval).
static int timer_repeat() { return g_timer.on ? g_timer.repeat : 1; }

static void timer_mark(hipStream_t s, int stage, int launches = 1) {
    if (!g_timer.on) return;
    if (g_timer.used == g_timer.pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { g_timer.on = false; return; }
        g_timer.pool.push_back(e);
    }
    if (hipEventRecord(g_timer.pool[g_timer.used], s) != hipSuccess) { g_timer.on = false; return; }
    g_timer.stage.push_back(stage);
    g_timer.launches.push_back(launches);
    ++g_timer.used;
}

static int ceil_log2(int v) {
    int b = 0;
    while ((1 << b) < v) ++b;
    return b;
}

static std::atomic<int> g_sort_min_rounds{0};   // fk_set_option("sort_min_rounds")

bool make_geometry(int B, int64_t N, int d_user, int K, fk_dtype t, Geometry* g) {
    if (B < 1 || N < 1 || K < 1 || K > 65536 || d_user < 1 || d_user > 512) return false;
    const int d = (d_user + 7) / 8 * 8;
    g->d_user = d_user;
    if (t != FK_F32 && t != FK_F16 && t != FK_BF16) return false;
    if ((int64_t)B * N >= ((int64_t)1 << 31)) return false;
    if (B > 65535) return false;                 // instances are the y dimension of every launch
    g->B = B; g->N = N; g->d = d; g->K = K; g->t = t;
    g->dchunks = d <= 32 ? 2 : (d <= 64 ? 4 : (d <= 128 ? 8 : (d <= 256 ? 16 : 32)));
    g->ktiles = (int)cdiv(K, 32);
    int nbmax;
    if (K <= 2048) {
        g->sort_passes = 1;
        g->sort_bits = ceil_log2(K) < 1 ? 1 : ceil_log2(K);
        g->pass_bits[0] = g->sort_bits;
        g->pass_bits[1] = 0;
        nbmax = K;
    } else {
        g->sort_passes = 2;
        g->sort_bits = ceil_log2(K);
        g->pass_bits[0] = g->sort_bits / 2;
        g->pass_bits[1] = g->sort_bits - g->pass_bits[0];
        nbmax = 1 << g->pass_bits[1];
    }
    // sort workgroups own whole sub-tiles of 4096 keys, one each (keys then stay in registers
    // between the scatter's two passes) until the table of per-workgroup histograms gets too
    // large: at most 4096 workgroups per instance with more than 256 bins, 65536 with fewer
    // (every pass of the two-pass sort, and the single pass for K <= 256)
    (void)nbmax;
    const int64_t max_blocks = (g->sort_passes == 1 && K > 256) ? 4096 : 65536;
    int64_t T = 4096 * cdiv(N, (int64_t)4096 * max_blocks);
    // (an instance of at most 4096 keys is one tile: the scatter kernel then counts for itself
    // and no histogram / scan kernel runs)
    // testing aid: larger tiles than the rule would pick (the several-rounds-per-workgroup form
    // of the sort kernels is otherwise only reached beyond 2^24 keys)
    const int min_rounds = g_sort_min_rounds.load(std::memory_order_relaxed);
    if (min_rounds > 1 && T < (int64_t)4096 * min_rounds) T = (int64_t)4096 * min_rounds;
    g->sort_tile = (int)T;
    g->sort_blocks = (int)cdiv(N, T);
    // rows reduced into one partial row: 256 by one wave, or, for N above 4M points, N/4096 by
    // the four waves of a workgroup (at most ~4096 + K partial rows to merge afterwards)
    int64_t R = 256;
    g->waves_per_item = 1;
    if (N > ((int64_t)1 << 22)) { R = cdiv(N, 4096); g->waves_per_item = 4; }
    g->rows_per_item = (int)R;
    g->max_items = N / R + K;
    // never more workgroups than there are groups of four 32-point batches
    g->fused_grid_cap = 0;
    if (t != FK_F32 && K <= 32 && d <= 128)
        g->fused_grid_cap = (int)std::min<int64_t>(B >= 1024 ? 1 : 1024 / B, cdiv(cdiv(N, 32), 4));
    // one persistent workgroup per compute unit at most (256 on this part), 256-point batches
    g->table_grid_cap = 0;
    if (t != FK_F32 && K > 32 && K <= 256 && d <= 128)
        g->table_grid_cap = (int)std::min<int64_t>(B >= 256 ? 1 : 256 / B, cdiv(N, 256));
    // small fp32 problems (at most 2^17 points in all, where the iteration is bound by its
    // number of launches: measured 1.5x at 2^14 points, break-even near 2^18): 64-point batches,
    // up to 2048 workgroups in all
    g->f32_grid_cap = 0;
    if (t == FK_F32 && K <= 64 && d <= 128 && (int64_t)B * N <= ((int64_t)1 << 17))
        g->f32_grid_cap = (int)std::min<int64_t>(B >= 2048 ? 1 : 2048 / B, cdiv(N, 64));
    return true;
}

Workspace carve(const Geometry& g, void* base, bool padded_x) {
    Workspace w;
    memset(&w, 0, sizeof(w));
    size_t off = 0;
    char* p = (char*)base;
    auto take = [&](size_t bytes) -> void* {
        void* r = p ? (void*)(p + off) : nullptr;
        off += align_up(bytes, 256);
        return r;
    };
    const size_t BN = (size_t)g.B * (size_t)g.N;
    const int nbmax = g.sort_passes == 1 ? g.K : (1 << g.pass_bits[1]);
    // sort buffers first: their placement depends on (B, N, K) only
    w.sorted_idx = (int32_t*)take(BN * 4);
    w.seg_off = (int32_t*)take((size_t)g.B * (g.K + 1) * 4);
    w.item_off = (int32_t*)take((size_t)g.B * (g.K + 1) * 4);
    w.block_hist = (int32_t*)take((size_t)g.B * g.sort_blocks * nbmax * 4);
    w.digit_off = (int32_t*)take((size_t)g.B * 2049 * 4);
    if (g.sort_passes == 2) {
        w.keys_tmp = (int32_t*)take(BN * 4);
        w.vals_tmp = (int32_t*)take(BN * 4);
        w.keys_sorted = (int32_t*)take(BN * 4);
    }
    const size_t sort_end = off;
    (void)sort_end;
    // shape/dtype dependent part
    const size_t BKd = (size_t)g.B * g.K * g.d;
    w.c_lp = take(BKd * elem_size(g.t));
    if (g.t != FK_F32) {
        w.c_frag = take((size_t)g.B * g.ktiles * g.dchunks * 64 * 16);
        w.c_bias = (float*)take((size_t)g.B * g.ktiles * 32 * 4);
    }
    const size_t fused_rows = (size_t)g.K * std::max({g.fused_grid_cap, g.table_grid_cap, g.f32_grid_cap});
    w.partial = (float*)take((size_t)g.B * std::max((size_t)g.max_items, fused_rows) * g.d * 4);
    if (fused_rows > 0) w.wg_counts = (int32_t*)take((size_t)g.B * fused_rows * 4);
    w.sums = (float*)take(BKd * 4);
    if (g.d != g.d_user) {
        if (padded_x) w.x_pad = take(BN * g.d * elem_size(g.t));
        w.c_pad_f32 = (float*)take(BKd * 4);
        w.c_pad_lp = take(BKd * elem_size(g.t));
    }
    w.bytes = off;
    return w;
}

static size_t sort_workspace_bytes(const Geometry& g) {
    const size_t BN = (size_t)g.B * (size_t)g.N;
    const int nbmax = g.sort_passes == 1 ? g.K : (1 << g.pass_bits[1]);
    size_t off = 0;
    off += align_up(BN * 4, 256);
    off += 2 * align_up((size_t)g.B * (g.K + 1) * 4, 256);
    off += align_up((size_t)g.B * g.sort_blocks * nbmax * 4, 256);
    off += align_up((size_t)g.B * 2049 * 4, 256);
    if (g.sort_passes == 2) off += 3 * align_up(BN * 4, 256);
    return off;
}

int current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return dev >= 0 && dev < kMaxDevices ? dev : 0;
}

namespace {

// Largest cache of the GPU agent with ordinal `want` (HSA lists L1, L2 and, where there is one,
// the memory-side last-level cache); 0 if the runtime cannot be asked.
struct CacheQuery { int want, seen; int64_t best; };

hsa_status_t on_cache(hsa_cache_t cache, void* data) {
    uint32_t size = 0;                    // this runtime counts in KiB (L2 4096, L3 262144 on MI355X)
    if (hsa_cache_get_info(cache, HSA_CACHE_INFO_SIZE, &size) == HSA_STATUS_SUCCESS) {
        auto* q = (CacheQuery*)data;
        if (((int64_t)size << 10) > q->best) q->best = (int64_t)size << 10;
    }
    return HSA_STATUS_SUCCESS;
}

hsa_status_t on_agent(hsa_agent_t agent, void* data) {
    hsa_device_type_t type;
    if (hsa_agent_get_info(agent, HSA_AGENT_INFO_DEVICE, &type) != HSA_STATUS_SUCCESS ||
        type != HSA_DEVICE_TYPE_GPU)
        return HSA_STATUS_SUCCESS;
    auto* q = (CacheQuery*)data;
    if (q->seen++ == q->want) (void)hsa_agent_iterate_caches(agent, on_cache, data);
    return HSA_STATUS_SUCCESS;
}

int64_t largest_cache_bytes(int dev) {
    if (hsa_init() != HSA_STATUS_SUCCESS) return 0;
    CacheQuery q{dev, 0, 0};
    (void)hsa_iterate_agents(on_agent, &q);
    (void)hsa_shut_down();          // the runtime is reference counted: HIP keeps its own hold
    return q.best;
}

}  // namespace

const DeviceInfo& device_info() {
    static DeviceInfo info[kMaxDevices];
    static std::atomic<int> known[kMaxDevices];
    const int dev = current_device();
    if (!known[dev].load(std::memory_order_acquire)) {
        static std::mutex mu;
        std::lock_guard<std::mutex> lock(mu);
        if (!known[dev].load(std::memory_order_relaxed)) {
            DeviceInfo d{256, (int64_t)160 << 10, (int64_t)256 << 20};
            int count = 0, v = 0;
            if (hipGetDeviceCount(&count) == hipSuccess && count > 0) {
                if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) d.cus = v;
                if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) == hipSuccess && v > 0)
                    d.lds_bytes = v;
                int64_t llc = largest_cache_bytes(dev);
                if (llc == 0 && hipDeviceGetAttribute(&v, hipDeviceAttributeL2CacheSize, dev) == hipSuccess && v > 0) llc = v;
                if (llc > 0) d.llc_bytes = llc;
            } else {
                (void)hipGetLastError();
            }
            info[dev] = d;
            known[dev].store(1, std::memory_order_release);
        }
    }
    return info[dev];
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

static fk_status check_common(const char* fn, int B, int64_t N, int d, int K, fk_dtype t,
                              const void* ws, size_t ws_bytes, Geometry* g) {
    if (B < 1 || N < 1 || K < 1 || d < 1) {
        set_error("%s: B, N, d, K must be positive (B=%d N=%lld d=%d K=%d)", fn, B, (long long)N, d, K);
        return FK_EINVAL;
    }
    if (t != FK_F32 && t != FK_F16 && t != FK_BF16) {
        set_error("%s: unknown dtype %d", fn, (int)t);
        return FK_EINVAL;
    }
    if (!make_geometry(B, N, d, K, t, g)) {
        set_error("%s: unsupported shape B=%d N=%lld d=%d K=%d (need 1<=d<=512, K<=65536, B<=65535, B*N<2^31)",
                  fn, B, (long long)N, d, K);
        return FK_EUNSUPPORTED;
    }
    if (!ws || ((uintptr_t)ws & 255u)) {
        set_error("%s: workspace pointer is NULL or not 256-byte aligned", fn);
        return FK_EINVAL;
    }
    const size_t need = carve(*g, nullptr).bytes;
    if (ws_bytes < need) {
        set_error("%s: workspace too small: %zu bytes given, %zu needed", fn, ws_bytes, need);
        return FK_EWORKSPACE;
    }
    return FK_OK;
}

#define FK_REQUIRE_PTR(fn, p)                                                      \
    do {                                                                           \
        if (!(p) || !fk::aligned16(p)) {                                           \
            fk::set_error("%s: %s is NULL or not 16-byte aligned", fn, #p);        \
            return FK_EINVAL;                                                      \
        }                                                                          \
    } while (0)
#define FK_OPTIONAL_PTR(fn, p)                                                     \
    do {                                                                           \
        if ((p) && !fk::aligned16(p)) {                                            \
            fk::set_error("%s: %s is not 16-byte aligned", fn, #p);                \
            return FK_EINVAL;                                                      \
        }                                                                          \
    } while (0)

// few clusters: one streaming pass over X builds per-workgroup tables of sums (computing the
// assignment on the way when asked to), then the usual merge/normalise
static fk_status run_stream_update(const Geometry& g, const Workspace& w, const void* X,
                                   int32_t* assign, bool compute_assign, const FinalizeArgs& fa,
                                   hipStream_t s) {
    int G = 0;
    const int rep = timer_repeat();
    for (int r = 0; r < rep; ++r) {
        if (g.fused_grid_cap > 0)
            FK_TRY(launch_stream_update(g, w, X, assign, compute_assign, &G, s));
        else if (g.table_grid_cap > 0)
            FK_TRY(launch_table_update(g, w, X, assign, &G, s));    // always computes the assignment
        else
            FK_TRY(launch_f32_update(g, w, X, fa.C_prev_f32, assign, &G, s));   // likewise
    }
    timer_mark(s, compute_assign ? kStageAssign : kStageReduce, rep);
    Geometry gm = g;
    gm.max_items = (int64_t)g.K * G;       // partial rows per instance as that pass wrote them
    FK_TRY(launch_finalize(gm, w, nullptr, nullptr, fa, s, w.wg_counts, G));
    timer_mark(s, kStageFinalize);
    return FK_OK;
}

// update = sort-inverse + segment reduce + merge/normalise, all into the carved workspace
static fk_status run_update(const Geometry& g, const Workspace& w, const void* X,
                            const int32_t* assign, const FinalizeArgs& fa, hipStream_t s) {
    if (fused_update_enabled(g)) return run_stream_update(g, w, X, (int32_t*)assign, false, fa, s);
    FK_TRY(launch_sort_inverse(g, w, assign, w.sorted_idx, w.seg_off, w.item_off, s));
    timer_mark(s, kStageSort);
    const int rep = timer_repeat();
    for (int r = 0; r < rep; ++r)
        FK_TRY(launch_segment_reduce(g, w, X, w.sorted_idx, w.seg_off, w.item_off, s));
    timer_mark(s, kStageReduce, rep);
    FK_TRY(launch_finalize(g, w, w.seg_off, w.item_off, fa, s));
    timer_mark(s, kStageFinalize);
    return FK_OK;
}

// ---------------------------------------------------------------- static scratch
// Scratch of the allocation-free entry point fk_assign_static: the fragment-ordered centroid
// copy followed by the score bias.  The array lives in the code object (every GPU that loads
// the library holds its own copy until the process ends); in host code its name is only a
// handle for hipGetSymbolAddress, never an address to hand to a kernel.
constexpr size_t kStaticFragBytes = (size_t)16 << 20;    // B * ceil(K/32) * dchunks KiB
constexpr size_t kStaticBiasBytes = (size_t)256 << 10;   // B * ceil(K/32) * 32 floats
static __device__ __align__(256) __attribute__((used)) unsigned char
    scratch[kStaticFragBytes + kStaticBiasBytes];

static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};            // device address of `scratch`, per device

// Device address of the static scratch on the current device (looked up once per device).
static fk_status static_scratch(unsigned char** out) {
    int dev = 0;
    FK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("fk_assign_static: device ordinal %d out of range (0..%d)", dev, kMaxDevices - 1);
        return FK_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        FK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255u)) {
            set_error("fk_assign_static: static scratch has no usable device address");
            return FK_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = (unsigned char*)g_scratch_ptr[dev];
    return FK_OK;
}

}  // namespace fk

using namespace fk;

extern "C" {

const char* fk_last_error(void) { return fk::g_err; }

void fk_stage_timer_start(void) {
    g_timer.used = 0;
    g_timer.stage.clear();
    g_timer.launches.clear();
    g_timer.on = true;
}

int fk_stage_timer_stop(double* stage_ms, int* stage_launches) {
    g_timer.on = false;
    for (int i = 0; i < kStages; ++i) { stage_ms[i] = 0.0; stage_launches[i] = 0; }
    if (g_timer.used == 0) return 0;
    if (hipEventSynchronize(g_timer.pool[g_timer.used - 1]) != hipSuccess) return -1;
    for (size_t i = 1; i < g_timer.used; ++i) {
        int st = g_timer.stage[i];
        // the gap between one iteration's last mark and the next iteration's opening mark
        // is the centroid re-layout: booked under the merge/normalise stage
        const bool relayout = st < 0 && g_timer.stage[i - 1] == kStageFinalize;
        if (st < 0 && !relayout) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_timer.pool[i - 1], g_timer.pool[i]) != hipSuccess) return -1;
        if (relayout) { stage_ms[kStageFinalize] += ms; continue; }
        stage_ms[st] += ms;
        stage_launches[st] += g_timer.launches[i];
    }
    const int n = (int)g_timer.used;
    g_timer.used = 0;             // a later stop without a start reports nothing
    g_timer.stage.clear();
    g_timer.launches.clear();
    return n;
}

int fk_set_option(const char* name, int value) {
    if (name && strcmp(name, "assign_variant") == 0 && value >= -1 && value <= 3) {
        set_assign_variant_override(value);
        return FK_OK;
    }
    if (name && strcmp(name, "assign_stream") == 0 && value >= -1 && value <= 1) {
        set_assign_stream_option(value);
        return FK_OK;
    }
    if (name && strcmp(name, "sort_min_rounds") == 0 && value >= -1 && value <= 64) {
        g_sort_min_rounds.store(value, std::memory_order_relaxed);
        return FK_OK;
    }
    if (name && strcmp(name, "sort_stage_bins") == 0 && value >= -1 && value <= 2048) {
        set_sort_stage_bins(value);
        return FK_OK;
    }
    if (name && strcmp(name, "timer_repeat") == 0 && value >= -1 && value <= 64) {
        g_timer.repeat = value < 1 ? 1 : value;
        return FK_OK;
    }
    if (name && strcmp(name, "fused_update") == 0 && value >= -1 && value <= 1) {
        set_fused_update_option(value);
        return FK_OK;
    }
    set_error("fk_set_option: unknown option or value out of range");
    return FK_EINVAL;
}

int fk_plan(int B, int64_t N, int d, int K, fk_dtype t, char* buf, size_t buf_bytes) {
    Geometry g;
    if (!buf || buf_bytes == 0) {
        set_error("fk_plan: no buffer");
        return FK_EINVAL;
    }
    if (!make_geometry(B, N, d, K, t, &g)) {
        snprintf(buf, buf_bytes, "unsupported");
        return FK_EUNSUPPORTED;
    }
    char assign[96];
    if (t == FK_F32)
        snprintf(assign, sizeof(assign), "%s", g.d > 128 ? "f32_wide" : ((int64_t)B * N < (1 << 18) ? "f32_split" : "f32"));
    else if (g.dchunks > 8)
        snprintf(assign, sizeof(assign), "mfma_wide(chunks=%d,points_per_wg=256)", g.dchunks);
    else if (assign_uses_stream_kernel(g))
        snprintf(assign, sizeof(assign), "mfma_stream(tiles=%d)", g.ktiles);
    else {
        static const int pts[4] = {256, 512, 512, 128};
        const int v = choose_assign_variant(g);
        snprintf(assign, sizeof(assign), "mfma_sweep(variant=%d,points_per_wg=%d)", v, pts[v]);
    }
    if (table_update_enabled(g)) {
        snprintf(buf, buf_bytes,
                 "assign+update=table_update(K x d table in the registers of a workgroup, X read once "
                 "per iteration, no sort; at most %d workgroups per instance) fk_assign alone=%s "
                 "fk_update alone=sort-inverse workspace=%zu",
                 g.table_grid_cap, assign, carve(g, nullptr).bytes);
    } else if (fused_update_enabled(g)) {
        snprintf(buf, buf_bytes,
                 "assign+update=stream_update(one-hot MFMA, X read once per iteration, no sort; "
                 "at most %d workgroups per instance) fk_assign alone=%s workspace=%zu",
                 g.fused_grid_cap, assign, carve(g, nullptr).bytes);
    } else if (f32_update_enabled(g)) {
        snprintf(buf, buf_bytes,
                 "assign+update=f32_update(K x d table in the registers of a workgroup, X read once "
                 "per iteration, no sort; at most %d workgroups per instance) fk_assign alone=%s "
                 "fk_update alone=sort-inverse workspace=%zu",
                 g.f32_grid_cap, assign, carve(g, nullptr).bytes);
    } else {
        snprintf(buf, buf_bytes,
                 "assign=%s ktiles=%d sort=%dpass(tile=%d,blocks=%d) reduce=%s(rows_per_item=%d) "
                 "max_items=%lld workspace=%zu",
                 assign, g.ktiles, g.sort_passes, g.sort_tile, g.sort_blocks,
                 g.waves_per_item == 4 ? "workgroup_per_item" : "wave_per_item", g.rows_per_item,
                 (long long)g.max_items, carve(g, nullptr).bytes);
    }
    if (g.d != g.d_user) {
        const size_t n = strlen(buf);
        if (n + 1 < buf_bytes) snprintf(buf + n, buf_bytes - n, " rows_padded=%d->%d", g.d_user, g.d);
    }
    {
        const DeviceInfo& di = device_info();
        const size_t n = strlen(buf);
        if (n + 1 < buf_bytes)
            snprintf(buf + n, buf_bytes - n, " device(cus=%d,lds=%lldKiB,llc=%lldMiB)", di.cus,
                     (long long)(di.lds_bytes >> 10), (long long)(di.llc_bytes >> 20));
    }
    return FK_OK;
}

size_t fk_workspace_bytes(int B, int64_t N, int d, int K, fk_dtype t) {
    Geometry g;
    if (!make_geometry(B, N, d, K, t, &g)) return 0;
    return carve(g, nullptr).bytes;
}

fk_status fk_assign(const void* X, const void* C, int32_t* assign, float* min_dist, int B,
                    int64_t N, int d, int K, fk_dtype t, void* ws, size_t ws_bytes,
                    void* stream) {
    Geometry g;
    FK_TRY(check_common("fk_assign", B, N, d, K, t, ws, ws_bytes, &g));
    FK_REQUIRE_PTR("fk_assign", X);
    FK_REQUIRE_PTR("fk_assign", C);
    FK_REQUIRE_PTR("fk_assign", assign);
    FK_OPTIONAL_PTR("fk_assign", min_dist);
    hipStream_t s = (hipStream_t)stream;
    const Workspace w = carve(g, ws);
    if (g.d != g.d_user) {
        // rows that are not a multiple of 8 wide: work on zero-padded copies
        FK_TRY(launch_copy_rows(X, w.x_pad, (int64_t)B * N, g.d_user, g.d, (int)elem_size(t), s));
        FK_TRY(launch_copy_rows(C, w.c_pad_lp, (int64_t)B * K, g.d_user, g.d, (int)elem_size(t), s));
        X = w.x_pad;
        C = w.c_pad_lp;
    }
    if (t == FK_F32) return launch_assign(g, X, C, nullptr, assign, min_dist, s);
    FK_TRY(launch_prepare_centroids(g, C, w.c_frag, w.c_bias, s));
    return launch_assign(g, X, w.c_frag, w.c_bias, assign, min_dist, s);
}

size_t fk_assign_static_limit(void) { return kStaticFragBytes; }

fk_status fk_assign_static(const void* X, const void* C, int32_t* assign, float* min_dist, int B,
                           int64_t N, int d, int K, fk_dtype t, void* stream) {
    const char* fn = "fk_assign_static";
    if (B < 1 || N < 1 || K < 1 || d < 1) {
        set_error("%s: B, N, d, K must be positive (B=%d N=%lld d=%d K=%d)", fn, B, (long long)N, d, K);
        return FK_EINVAL;
    }
    if (t != FK_F32 && t != FK_F16 && t != FK_BF16) {
        set_error("%s: unknown dtype %d", fn, (int)t);
        return FK_EINVAL;
    }
    Geometry g;
    if (!make_geometry(B, N, d, K, t, &g)) {
        set_error("%s: unsupported shape B=%d N=%lld d=%d K=%d", fn, B, (long long)N, d, K);
        return FK_EUNSUPPORTED;
    }
    if (g.d != g.d_user) {
        set_error("%s: d must be a multiple of 8 (a padded copy of X would not fit the static scratch)", fn);
        return FK_EUNSUPPORTED;
    }
    FK_REQUIRE_PTR(fn, X);
    FK_REQUIRE_PTR(fn, C);
    FK_REQUIRE_PTR(fn, assign);
    FK_OPTIONAL_PTR(fn, min_dist);
    hipStream_t s = (hipStream_t)stream;
    if (t == FK_F32) return launch_assign(g, X, C, nullptr, assign, min_dist, s);   // no scratch at all
    const size_t frag_bytes = (size_t)B * g.ktiles * g.dchunks * 64 * 16;
    const size_t bias_bytes = (size_t)B * g.ktiles * 32 * 4;
    if (frag_bytes > kStaticFragBytes || bias_bytes > kStaticBiasBytes) {
        set_error("%s: centroids too large for the static scratch: B*ceil(K/32)*%d KiB = %zu bytes, limit %zu",
                  fn, g.dchunks, frag_bytes, kStaticFragBytes);
        return FK_EWORKSPACE;
    }
    unsigned char* base = nullptr;
    FK_TRY(static_scratch(&base));
    void* c_frag = base;
    float* c_bias = (float*)(base + kStaticFragBytes);
    // both regions are rewritten in full for this shape before the assign kernel reads them, so
    // nothing left by an earlier call is ever read
    FK_TRY(launch_prepare_centroids(g, C, c_frag, c_bias, s));
    return launch_assign(g, X, c_frag, c_bias, assign, min_dist, s);
}

fk_status fk_sort_inverse(const int32_t* assign, int32_t* sorted_idx, int32_t* seg_offsets,
                          int B, int64_t N, int K, void* ws, size_t ws_bytes, void* stream) {
    Geometry g;
    if (B < 1 || N < 1 || K < 1) {
        set_error("fk_sort_inverse: B, N, K must be positive");
        return FK_EINVAL;
    }
    if (!make_geometry(B, N, 8, K, FK_F32, &g)) {
        set_error("fk_sort_inverse: unsupported shape B=%d N=%lld K=%d", B, (long long)N, K);
        return FK_EUNSUPPORTED;
    }
    if (!ws || ((uintptr_t)ws & 255u)) {
        set_error("fk_sort_inverse: workspace pointer is NULL or not 256-byte aligned");
        return FK_EINVAL;
    }
    if (ws_bytes < sort_workspace_bytes(g)) {
        set_error("fk_sort_inverse: workspace too small: %zu bytes given, %zu needed", ws_bytes,
                  sort_workspace_bytes(g));
        return FK_EWORKSPACE;
    }
    FK_REQUIRE_PTR("fk_sort_inverse", assign);
    FK_REQUIRE_PTR("fk_sort_inverse", sorted_idx);
    FK_REQUIRE_PTR("fk_sort_inverse", seg_offsets);
    const Workspace w = carve(g, ws);
    return launch_sort_inverse(g, w, assign, sorted_idx, seg_offsets, nullptr, (hipStream_t)stream);
}

fk_status fk_update(const void* X, const int32_t* assign, const float* C_prev_f32,
                    float* C_out_f32, void* C_out_lp, int32_t* counts, int B, int64_t N, int d,
                    int K, fk_dtype t, void* ws, size_t ws_bytes, void* stream) {
    Geometry g;
    FK_TRY(check_common("fk_update", B, N, d, K, t, ws, ws_bytes, &g));
    FK_REQUIRE_PTR("fk_update", X);
    FK_REQUIRE_PTR("fk_update", assign);
    FK_REQUIRE_PTR("fk_update", C_prev_f32);
    FK_REQUIRE_PTR("fk_update", C_out_f32);
    FK_OPTIONAL_PTR("fk_update", C_out_lp);
    FK_REQUIRE_PTR("fk_update", counts);
    const Workspace w = carve(g, ws);
    hipStream_t s = (hipStream_t)stream;
    const bool pad = g.d != g.d_user;
    if (pad) {
        FK_TRY(launch_copy_rows(X, w.x_pad, (int64_t)B * N, g.d_user, g.d, (int)elem_size(t), s));
        FK_TRY(launch_copy_rows(C_prev_f32, w.c_pad_f32, (int64_t)B * K, g.d_user, g.d, 4, s));
        X = w.x_pad;
    }
    FinalizeArgs fa;
    fa.C_prev_f32 = pad ? w.c_pad_f32 : C_prev_f32;
    fa.C_out_f32 = pad ? w.c_pad_f32 : C_out_f32;
    fa.C_out_lp = pad ? (C_out_lp ? w.c_pad_lp : nullptr) : C_out_lp;
    fa.c_frag = nullptr;
    fa.c_bias = nullptr;
    fa.counts = counts;
    fa.sums = nullptr;
    fa.accumulate = false;
    fa.normalise = true;
    timer_mark(s, -1);
    FK_TRY(run_update(g, w, X, assign, fa, s));
    if (pad) {
        FK_TRY(launch_copy_rows(w.c_pad_f32, C_out_f32, (int64_t)B * K, g.d, g.d_user, 4, s));
        if (C_out_lp)
            FK_TRY(launch_copy_rows(w.c_pad_lp, C_out_lp, (int64_t)B * K, g.d, g.d_user, (int)elem_size(t), s));
    }
    return FK_OK;
}

fk_status fk_standard_assign(const void* X, const void* C, float* D, int32_t* assign, int B,
                             int64_t N, int d, int K, fk_dtype t, void* ws, size_t ws_bytes,
                             void* stream) {
    Geometry g;
    FK_TRY(check_common("fk_standard_assign", B, N, d, K, t, ws, ws_bytes, &g));
    if (g.d != g.d_user) {
        set_error("fk_standard_assign: the comparator needs d to be a multiple of 8");
        return FK_EUNSUPPORTED;
    }
    FK_REQUIRE_PTR("fk_standard_assign", X);
    FK_REQUIRE_PTR("fk_standard_assign", C);
    FK_REQUIRE_PTR("fk_standard_assign", D);
    FK_REQUIRE_PTR("fk_standard_assign", assign);
    const Workspace w = carve(g, ws);
    return launch_standard_assign(g, w, X, C, D, assign, (hipStream_t)stream);
}

fk_status fk_standard_update(const void* X, const int32_t* assign, const float* C_prev_f32,
                             float* C_out_f32, int32_t* counts, float* sums, int B, int64_t N,
                             int d, int K, fk_dtype t, void* stream) {
    Geometry g;
    if (!make_geometry(B, N, d, K, t, &g)) {
        set_error("fk_standard_update: unsupported shape B=%d N=%lld d=%d K=%d", B, (long long)N, d, K);
        return FK_EUNSUPPORTED;
    }
    if (g.d != g.d_user) {
        set_error("fk_standard_update: the comparator needs d to be a multiple of 8");
        return FK_EUNSUPPORTED;
    }
    FK_REQUIRE_PTR("fk_standard_update", X);
    FK_REQUIRE_PTR("fk_standard_update", assign);
    FK_REQUIRE_PTR("fk_standard_update", C_prev_f32);
    FK_REQUIRE_PTR("fk_standard_update", C_out_f32);
    FK_REQUIRE_PTR("fk_standard_update", counts);
    FK_REQUIRE_PTR("fk_standard_update", sums);
    return launch_standard_update(g, X, assign, C_prev_f32, C_out_f32, counts, sums,
                                  (hipStream_t)stream);
}

fk_status fk_lloyd_iter(const void* X, float* C_f32, void* C_lp, int32_t* assign,
                        int32_t* counts, int B, int64_t N, int d, int K, fk_dtype t, int iters,
                        void* ws, size_t ws_bytes, void* stream) {
    Geometry g;
    FK_TRY(check_common("fk_lloyd_iter", B, N, d, K, t, ws, ws_bytes, &g));
    if (iters < 0) {
        set_error("fk_lloyd_iter: iters must be >= 0");
        return FK_EINVAL;
    }
    FK_REQUIRE_PTR("fk_lloyd_iter", X);
    FK_REQUIRE_PTR("fk_lloyd_iter", C_f32);
    FK_OPTIONAL_PTR("fk_lloyd_iter", C_lp);
    FK_REQUIRE_PTR("fk_lloyd_iter", assign);
    FK_REQUIRE_PTR("fk_lloyd_iter", counts);
    if (iters == 0) return FK_OK;
    hipStream_t s = (hipStream_t)stream;
    const Workspace w = carve(g, ws);
    const bool pad = g.d != g.d_user;
    float* const C_user = C_f32;
    void* const C_lp_user = C_lp;
    if (pad) {
        // rows that are not a multiple of 8 wide: iterate on zero-padded copies of X and C,
        // copy the centroids back without the padding at the end
        FK_TRY(launch_copy_rows(X, w.x_pad, (int64_t)B * N, g.d_user, g.d, (int)elem_size(t), s));
        FK_TRY(launch_copy_rows(C_f32, w.c_pad_f32, (int64_t)B * K, g.d_user, g.d, 4, s));
        X = w.x_pad;
        C_f32 = w.c_pad_f32;
        C_lp = C_lp ? w.c_pad_lp : nullptr;
    }
    void* lp = C_lp ? C_lp : w.c_lp;
    // what the first assignment consumes: the master rounded to the storage type
    FK_TRY(launch_round_centroids(g, C_f32, t == FK_F32 ? nullptr : lp, w.c_frag, w.c_bias, s));
    for (int it = 0; it < iters; ++it) {
        timer_mark(s, -1);
        // few clusters: assignment and sums in one pass over X (see run_stream_update)
        const bool fused = fused_update_enabled(g) || table_update_enabled(g) || f32_update_enabled(g);
        if (!fused) {
            const int rep = timer_repeat();
            for (int r = 0; r < rep; ++r) {
                if (t == FK_F32)
                    FK_TRY(launch_assign(g, X, C_f32, nullptr, assign, nullptr, s));
                else
                    FK_TRY(launch_assign(g, X, w.c_frag, w.c_bias, assign, nullptr, s));
            }
            timer_mark(s, kStageAssign, rep);
        }
        FinalizeArgs fa;
        fa.C_prev_f32 = C_f32;
        fa.C_out_f32 = C_f32;
        fa.C_out_lp = (t == FK_F32) ? (it + 1 == iters ? C_lp : nullptr) : lp;
        fa.c_frag = w.c_frag;      // re-laid out for the next assignment by the same kernel
        fa.c_bias = w.c_bias;
        fa.counts = counts;
        fa.sums = nullptr;
        fa.accumulate = false;
        fa.normalise = true;
        if (fused) {
            FK_TRY(run_stream_update(g, w, X, assign, true, fa, s));
        } else {
            FK_TRY(run_update(g, w, X, assign, fa, s));
        }
    }
    if (pad) {
        FK_TRY(launch_copy_rows(C_f32, C_user, (int64_t)B * K, g.d, g.d_user, 4, s));
        if (C_lp_user)
            FK_TRY(launch_copy_rows(C_lp, C_lp_user, (int64_t)B * K, g.d, g.d_user, (int)elem_size(t), s));
    }
    return FK_OK;
}

}  // extern "C"
