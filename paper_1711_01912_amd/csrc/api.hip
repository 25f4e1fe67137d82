// The C ABI declared in include/cpeval.h: argument checks, plan selection,
// cost-table upload and the order in which the stages are enqueued.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>

#include "launch.hpp"

using namespace cpeval;

struct cp_profile {
    int32_t slots = 0, count = 0;
    std::vector<hipEvent_t> ev;          // slots * (CP_NUM_STAGES + 1)
    std::vector<int32_t> launches;       // slots * 2
};

namespace {

// Pinned staging slots for the cost tables of calls with more than 64 devices (up to 1 MB),
// reused round-robin; a slot is only rewritten after the copy that last read it has finished,
// so the ninth such call in flight waits for the first.
struct StageSlot {
    void *host = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool pending = false;
};
constexpr int kStageSlots = 8;
StageSlot g_stage[kStageSlots];
int g_stage_next = 0;
std::mutex g_stage_mu;

int stage_and_copy(const void *src, size_t bytes, void *dst, hipStream_t st) {
    std::lock_guard<std::mutex> lock(g_stage_mu);
    StageSlot &s = g_stage[g_stage_next];
    g_stage_next = (g_stage_next + 1) % kStageSlots;
    if (s.pending) {
        if (hipEventSynchronize(s.done) != hipSuccess) return CP_ERR_HIP;
        s.pending = false;
    }
    if (!s.done && hipEventCreateWithFlags(&s.done, hipEventDisableTiming) != hipSuccess)
        return CP_ERR_HIP;
    if (s.cap < bytes) {
        if (s.host) (void)hipHostFree(s.host);
        s.host = nullptr;
        s.cap = 0;
        size_t cap = std::max<size_t>(bytes, 4096);
        if (hipHostMalloc(&s.host, cap, hipHostMallocDefault) != hipSuccess) return CP_ERR_HIP;
        s.cap = cap;
    }
    std::memcpy(s.host, src, bytes);
    if (hipMemcpyAsync(dst, s.host, bytes, hipMemcpyHostToDevice, st) != hipSuccess) return CP_ERR_HIP;
    if (hipEventRecord(s.done, st) != hipSuccess) return CP_ERR_HIP;
    s.pending = true;
    return CP_OK;
}

// Cost tables written by kernels whose arguments carry the values: no staging memory, no
// copy engine.  One launch moves kTableChunkWords table entries.
constexpr int kTableChunkWords = 448;                       // 3.5 KB of kernel arguments
struct TableChunk { uint64_t v[kTableChunkWords]; };

__global__ void table_write_kernel(TableChunk chunk, uint64_t *dst, int32_t count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = chunk.v[i];
}

int write_tables_by_kernel(const void *src, size_t entries, void *dst, hipStream_t st) {
    const uint64_t *from = (const uint64_t *)src;
    uint64_t *to = (uint64_t *)dst;
    for (size_t at = 0; at < entries; at += kTableChunkWords) {
        TableChunk chunk;
        const int32_t count = (int32_t)std::min<size_t>(kTableChunkWords, entries - at);
        std::memcpy(chunk.v, from + at, (size_t)count * 8);
        hipLaunchKernelGGL(table_write_kernel, dim3((count + 255) / 256), dim3(256), 0, st, chunk, to + at, count);
    }
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
}

// Cost tables of one call into device memory.  Up to 64 devices (66 KB) they travel as kernel
// arguments: nothing is allocated, nothing waits, and calls on different streams or threads
// do not meet.  Larger tables go through the pinned staging ring above.
int upload_tables(const void *src, size_t entries, void *dst, hipStream_t st, bool by_kernel_only = false) {
    if (by_kernel_only || entries <= table_words(kMagicMaxK)) return write_tables_by_kernel(src, entries, dst, st);
    return stage_and_copy(src, entries * 8, dst, st);
}

// Scratch memory of cp_eval_static: one array per GPU, part of the loaded code object, never
// allocated or freed.  In host code the array's name is only a handle: the device address is
// looked up once per device and kept.
static __device__ __align__(256) uint8_t scratch[CP_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

int static_scratch(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CP_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CP_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CP_OK;
}

constexpr size_t kWindowLdsLimit = kLdsBudget - 256;   // room for the kernel's static LDS
constexpr size_t kSharedStaticLds = 512;               // static LDS of the shared-window and streamed kernels beyond that

bool window_fits(const Packed &p, int32_t k, size_t tick_bytes, size_t limit = kWindowLdsLimit,
                 WindowCfg *cfg_b = nullptr, WindowCfg *cfg_t = nullptr, bool tab4 = false) {
    if (!p.have_window || k > kMagicMaxK) return false;
    WindowCfg b, t;
    (void)tab4;
    if (!window_config(p.win_b, k, tick_bytes, limit, b)) return false;
    if (!window_config(p.win_t, k, tick_bytes, limit, t)) return false;
    if (cfg_b) *cfg_b = b;
    if (cfg_t) *cfg_t = t;
    return true;
}

// The shared-window kernel with `groups` partitions per workgroup, both directions.
bool shared_fits(const Packed &p, int32_t k, size_t tick_bytes, int groups, size_t limit, SharedCfg *cfg_b,
                 SharedCfg *cfg_t, bool tab4 = false) {
    if (!p.have_window || k > kMagicMaxK || tick_bytes != 4 || limit <= kSharedStaticLds) return false;
    SharedCfg b, t;
    if (!shared_config(p.win_b, k, groups, limit - kSharedStaticLds, b, tab4)) return false;
    if (!shared_config(p.win_t, k, groups, limit - kSharedStaticLds, t, tab4)) return false;
    if (cfg_b) *cfg_b = b;
    if (cfg_t) *cfg_t = t;
    return true;
}

// The streamed resident-window kernel, both directions.
bool stream_fits(const Packed &p, int32_t k, size_t tick_bytes, size_t limit, StreamCfg *cfg_b, StreamCfg *cfg_t) {
    if (!p.have_window || k > kMagicMaxK || tick_bytes != 4 || limit <= kSharedStaticLds) return false;
    StreamCfg b, t;
    if (!stream_config(p.win_b, k, limit - kSharedStaticLds, false, b)) return false;
    if (!stream_config(p.win_t, k, limit - kSharedStaticLds, false, t)) return false;
    if (cfg_b) *cfg_b = b;
    if (cfg_t) *cfg_t = t;
    return true;
}

size_t pperm_bytes(const Packed &p, const WindowDir &d, int32_t batch) {
    (void)p;
    return align_up((size_t)batch * (size_t)d.ticks * (size_t)d.wpad);
}

// LDS one workgroup may use on the current device, minus the kernel's static part.
size_t device_window_lds_limit() {
    int dev = 0, bytes = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
        return 0;
    size_t lim = std::min<size_t>((size_t)std::max(bytes, 0), kLdsBudget);
    return lim > 256 ? lim - 256 : 0;
}

// Which plan is cheaper for this batch, from measured unit costs on MI355X: the
// resident-window plan walks every tick once per partition, 256 compute units times
// as many workgroups as fit one unit's LDS at a time (about 0.6 us per tick plus
// 0.045 us per slice); the wave-column plan pays about 6.3 us per level launch plus
// its gathers at about 4 TB/s.
// Workgroups of the resident-window kernel one compute unit holds at a time: LDS, and the
// wavefronts the register file takes (the loaders keep nl x dr 16-byte loads in registers:
// about 64 registers per lane with one load per tick, 80 with two or three, more beyond).
double window_wg_per_cu(const WindowCfg &c) {
    const int groups = std::max(1, c.groups);
    const double waves = c.nl <= 1 ? 32.0 : (c.nl <= 3 ? 24.0 : (c.nl == 4 ? 20.0 : 16.0));
    return std::max<double>(1.0, std::floor(std::min<double>(
        (double)(kLdsBudget / std::max<size_t>(c.lds_bytes, 1)), waves / (groups * (c.nc + c.nlw + c.nfw)))));
}

double window_sweep_us(const WindowDir &d, const WindowCfg &c, int32_t batch) {
    const double cus = 256.0;
    const int groups = std::max(1, c.groups);         // partitions per workgroup
    const double rounds = std::ceil((double)batch / (cus * window_wg_per_cu(c) * groups));
    return rounds * (double)d.ticks * (0.58 + 0.03 * d.smax);
}

// The shared-window kernel: one workgroup per compute unit, 2 or 4 partitions each.  A tick
// costs 1.33 (2.03) times the resident-window kernel's (large sparse workload: 0.745 us ->
// 0.99 us -> 1.51 us per tick for 1, 2, 4 partitions).
double shared_sweep_us(const WindowDir &d, int groups, int32_t batch) {
    const double rounds = std::ceil((double)batch / (256.0 * groups));
    return rounds * (double)d.ticks * (groups == 4 ? 2.03 : 1.33) * (0.58 + 0.03 * d.smax);
}

// A mask pass of its own streams b and tl once: 6.2 - 6.5 TB/s for 32-bit ticks in aligned rows
// (measured), 4.4 for the plain kernel.
constexpr double kMaskPassBytesPerUs = 6.0e6;

// Both sweeps under the wave-column plan.
double column_plan_us(const Packed &p, int32_t batch, size_t tick_bytes) {
    auto column_us = [&](const ColumnDir &d) {
        double launches = 0;
        for (size_t l = 0; l < d.lvl_count.size(); ++l)
            launches += (d.lvl_hubs[l] > 0) + (d.lvl_count[l] > d.lvl_hubs[l]);
        const double bytes = ((double)p.n + (double)p.m) * batch * (1.0 + (double)tick_bytes);
        // (measured: 6.3 us per launch; the gathers of a sweep at 6.0 - 7.0 TB/s with four
        // neighbours' loads in flight per lane)
        return launches * 6.3 + bytes / 6.5e6;
    };
    return column_us(p.col_b) + column_us(p.col_t);
}

// CP_PLAN_AUTO among the window plans (the caller has found the resident-window plan runnable
// and preferable to the wave-column plan).  Sharing a workgroup pays where one workgroup of the
// resident-window kernel fills a compute unit (wide ticks, a long ring): there the batch can
// only overlap inside a workgroup.  Narrow graphs, whose workgroups sit several to a unit
// already, gain nothing from it (measured: 2,016 vertices x 8,192 partitions 0.62 ms per sweep
// against 0.56 and 0.80 ms; 5,271 vertices x 16,384 partitions 1.08 against 1.31 and 1.05 ms).
// mask_penalty_us: what the shared plans pay for the mask pass the other plan would not need.
// mask_penalty_us: what a mask pass of its own would cost the shared plans; mask_t_factor: what
// writing the mask inside their t sweep costs instead, as a factor on that sweep (measured 1.22).
int choose_window_plan(const Packed &p, int32_t k, size_t tick_bytes, size_t lds_limit, const WindowCfg &cb,
                       const WindowCfg &ct, int32_t batch, double mask_penalty_us, SharedCfg *sh_b, SharedCfg *sh_t,
                       bool tab4 = false, double mask_t_factor = 1.0, double *us_out = nullptr) {
    int best = CP_PLAN_RESIDENT_WINDOW;
    double best_us = window_sweep_us(p.win_b, cb, batch) + window_sweep_us(p.win_t, ct, batch);
    if (us_out) *us_out = best_us;
    if (window_wg_per_cu(cb) > 1.0 || window_wg_per_cu(ct) > 1.0) return best;
    for (int groups = 2; groups <= 4; groups += 2) {
        SharedCfg b, t;
        if (!shared_fits(p, k, tick_bytes, groups, lds_limit, &b, &t, tab4)) continue;
        const double us = shared_sweep_us(p.win_b, groups, batch) +
                          shared_sweep_us(p.win_t, groups, batch) * mask_t_factor + mask_penalty_us;
        if (us < best_us) {
            best_us = us;
            best = groups == 4 ? CP_PLAN_SHARED_WINDOW_4 : CP_PLAN_SHARED_WINDOW_2;
            if (sh_b) *sh_b = b;
            if (sh_t) *sh_t = t;
        }
    }
    if (us_out) *us_out = best_us;
    return best;
}

size_t tables_bytes(int32_t k) { return align_up(table_words(k) * 8); }

// One call's tables as they lie in device memory: the 8-byte entries (multiply-shift constants,
// or plain divisors), then, where they exist, the 4-byte entries.
std::vector<uint64_t> table_image(const CostTables &tabs, int32_t k) {
    std::vector<uint64_t> img(table_words(k), 0);
    const size_t entries = table_entries(k);
    std::memcpy(img.data(), tabs.magic_ok ? (const void *)tabs.magic.data() : (const void *)tabs.divisor.data(),
                entries * 8);
    if (tabs.tab4_ok) std::memcpy(img.data() + entries, tabs.tab4.data(), entries * 4);
    return img;
}
size_t column_scratch_bytes(const Packed &p, int32_t batch, int tick_bytes) {
    return align_up((size_t)p.n * (size_t)batch * (size_t)tick_bytes);
}

int check_eval_sizes(const cp_graph *g, int32_t batch, int32_t k, int assign_layout, int plan) {
    if (!g) return CP_ERR_NULL;
    if (batch < 1 || k < 1 || k > 255) return CP_ERR_SIZE;
    if (assign_layout != CP_ASSIGN_PARTITION_MAJOR && assign_layout != CP_ASSIGN_VERTEX_MAJOR)
        return CP_ERR_ARG;
    if (plan < CP_PLAN_AUTO || plan > CP_PLAN_STREAMED_WINDOW) return CP_ERR_ARG;
    return CP_OK;
}

struct PctPlan {
    int b_bits = 1, key_bits = 1, key_bytes = 4;
    int64_t max_b = 0;
    size_t keys_bytes = 0, vals_bytes = 0, counts_bytes = 0, total = 0;
};

int bit_length(uint64_t x) {
    int b = 0;
    while (x) { ++b; x >>= 1; }
    return b;
}

int pct_plan(const cp_graph *g, int32_t batch, int32_t k, int64_t max_b, PctPlan &out) {
    int rc = check_eval_sizes(g, batch, k, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO);
    if (rc) return rc;
    if (max_b < 0) return CP_ERR_ARG;
    const Packed &p = g->packed;
    out.max_b = max_b > 0 ? max_b : std::max<int64_t>(p.info.raw_path_bound, 1);
    out.b_bits = std::max(1, bit_length((uint64_t)out.max_b));
    out.key_bits = out.b_bits + bit_length((uint64_t)(k - 1));
    if (out.key_bits > 64) return CP_ERR_OVERFLOW;
    out.key_bytes = out.key_bits <= 32 ? 4 : 8;
    const int64_t tiles = pct_sort_tiles(p.n);
    if (tiles * (int64_t)batch >= (int64_t)1 << 31) return CP_ERR_SIZE;
    const size_t items = (size_t)p.n * (size_t)batch;
    out.keys_bytes = align_up(items * (size_t)out.key_bytes);
    out.vals_bytes = align_up(items * sizeof(int32_t));
    out.counts_bytes = pct_counts_bytes(p.n, batch);
    out.total = 2 * out.keys_bytes + out.vals_bytes + out.counts_bytes;
    return CP_OK;
}

}  // namespace

namespace {

struct SimPlan {
    size_t tab = 0, tie_inv = 0, per_i32 = 0, per_u64 = 0, total = 0;
    bool pct = false, with_tie = false;
};

int sim_plan(const cp_graph *g, int32_t batch, int32_t k, int policy, bool with_tie, SimPlan &out) {
    if (!g) return CP_ERR_NULL;
    if (batch < 1 || k < 1 || k > kWave) return CP_ERR_SIZE;
    if (policy != CP_POLICY_FIFO && policy != CP_POLICY_PCT) return CP_ERR_ARG;
    const size_t n = (size_t)g->packed.n;
    out.pct = policy == CP_POLICY_PCT;
    out.with_tie = with_tie && !out.pct;
    out.tab = tables_bytes(k);
    out.tie_inv = out.with_tie ? align_up(n * 4) : 0;
    out.per_i32 = align_up(n * (size_t)batch * 4);
    out.per_u64 = align_up(n * (size_t)batch * 8);
    out.total = out.tab + out.tie_inv + 3 * out.per_i32 + (out.pct ? 2 : 1) * out.per_u64;
    return CP_OK;
}

template <typename WT>
void min_weights(const Packed &p, uint64_t s_min, uint64_t &min_c, uint64_t &min_t, long double &sum_w) {
    const WT *c = (const WT *)(p.blob.data() + p.c_off);
    const WT *t = (const WT *)(p.blob.data() + p.col_b.wt_off);
    min_c = UINT64_MAX;
    min_t = UINT64_MAX;
    sum_w = 0;
    for (int32_t v = 0; v < p.n; ++v) {
        const uint64_t cv = (uint64_t)c[v];
        min_c = std::min<uint64_t>(min_c, cv);
        sum_w += (long double)(cv / s_min + (cv % s_min != 0));
    }
    for (int64_t e = 0; e < p.m; ++e) min_t = std::min<uint64_t>(min_t, (uint64_t)t[e]);
}

}  // namespace

extern "C" {

int cp_graph_create(int32_t n, int64_t m, int32_t L,
                    const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *succ_t,
                    const int32_t *pred_ptr, const int32_t *pred_idx, const int32_t *pred_eid,
                    const int64_t *c, const int32_t *level_ptr, const int32_t *level_vtx,
                    cp_graph **out) {
    if (!out) return CP_ERR_NULL;
    *out = nullptr;
    cp_graph *g = new (std::nothrow) cp_graph;
    if (!g) return CP_ERR_ALLOC;
    int rc;
    try {
        rc = pack_graph(n, m, L, succ_ptr, succ_idx, succ_t, pred_ptr, pred_idx, pred_eid, c,
                        level_ptr, level_vtx, g->packed);
    } catch (const std::bad_alloc &) {
        rc = CP_ERR_ALLOC;
    }
    if (rc != CP_OK) {
        delete g;
        return rc;
    }
    cp_graph_info &info = g->packed.info;
    WindowCfg cb, ct;
    info.window_ok = window_fits(g->packed, 1, (size_t)info.min_tick_bytes, kWindowLdsLimit, &cb, &ct) ? 1 : 0;
    // the choice is made per call (it depends on the batch); this is the one for 256 partitions
    info.auto_plan = CP_PLAN_WAVE_COLUMN;
    if (info.window_ok) {
        double window_us = 0.0;
        const int wplan = choose_window_plan(g->packed, 1, (size_t)info.min_tick_bytes, kWindowLdsLimit, cb, ct, 256,
                                             0.0, nullptr, nullptr, false, 1.0, &window_us);
        if (window_us <= column_plan_us(g->packed, 256, (size_t)info.min_tick_bytes)) info.auto_plan = wplan;
    }
    *out = g;
    return CP_OK;
}

int cp_graph_get_info(const cp_graph *g, cp_graph_info *out) {
    if (!g || !out) return CP_ERR_NULL;
    *out = g->packed.info;
    out->uploaded = g->device_blob ? 1 : 0;
    return CP_OK;
}

int cp_graph_upload(cp_graph *g, void *device_blob, size_t blob_bytes, void *stream) {
    if (!g || !device_blob) return CP_ERR_NULL;
    if (blob_bytes < g->packed.blob.size() || ((uintptr_t)device_blob % kAlign) != 0)
        return CP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(device_blob, g->packed.blob.data(), g->packed.blob.size(),
                       hipMemcpyHostToDevice, st) != hipSuccess)
        return CP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CP_ERR_HIP;
    g->device_blob = device_blob;
    return CP_OK;
}

void cp_graph_destroy(cp_graph *g) { delete g; }

int cp_eval_workspace_bytes(const cp_graph *g, int32_t batch, int32_t k, int assign_layout,
                            int plan, int out_layout, int tick_dtype, size_t *out_bytes) {
    if (!out_bytes) return CP_ERR_NULL;
    int rc = check_eval_sizes(g, batch, k, assign_layout, plan);
    if (rc) return rc;
    if (out_layout != CP_OUT_VERTEX_MAJOR && out_layout != CP_OUT_PARTITION_MAJOR) return CP_ERR_ARG;
    if (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64) return CP_ERR_ARG;
    size_t bytes = tables_bytes(k);
    // the wave-column plan reads device ids vertex-major; under CP_PLAN_AUTO it may be
    // the one that runs, whatever the graph prefers, if the cost model rules the other out
    size_t column = 0, window = 0;
    const bool may_column = plan == CP_PLAN_AUTO || plan == CP_PLAN_WAVE_COLUMN || plan == CP_PLAN_COLUMN_SLICE;
    if (assign_layout == CP_ASSIGN_PARTITION_MAJOR && may_column)
        column = align_up((size_t)g->packed.n * (size_t)batch);
    // the wave-column plan sweeps vertex-major: partition-major outputs are transposed
    // out of two scratch arrays
    if (out_layout == CP_OUT_PARTITION_MAJOR && may_column)
        column += 2 * column_scratch_bytes(g->packed, batch, tick_dtype);
    // the resident-window plan gathers the device ids into sweep order, once per direction
    if (plan != CP_PLAN_WAVE_COLUMN && plan != CP_PLAN_COLUMN_SLICE && g->packed.have_window)
        window = pperm_bytes(g->packed, g->packed.win_b, batch) + pperm_bytes(g->packed, g->packed.win_t, batch);
    *out_bytes = bytes + std::max(column, window);
    return CP_OK;
}

int cp_eval_choose_plan(const cp_graph *g, int32_t batch, int32_t k, const int64_t *speeds,
                        const int64_t *bandwidth, int tick_dtype, int *plan_out) {
    int rc = check_eval_sizes(g, batch, k, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO);
    if (rc) return rc;
    if (!speeds || !bandwidth || !plan_out) return CP_ERR_NULL;
    if (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64) return CP_ERR_ARG;
    const Packed &p = g->packed;
    CostTables tabs;
    try {
        rc = build_cost_tables(k, speeds, bandwidth, p.narrow, p.info.max_c, p.info.max_t, tabs);
    } catch (const std::bad_alloc &) {
        rc = CP_ERR_ALLOC;
    }
    if (rc) return rc;
    WindowCfg cfg_b, cfg_t;
    const bool can_window = tabs.magic_ok && window_fits(p, k, (size_t)tick_dtype, device_window_lds_limit(),
                                                         &cfg_b, &cfg_t);
    *plan_out = CP_PLAN_WAVE_COLUMN;
    if (can_window) {
        double window_us = 0.0;
        const int wplan = choose_window_plan(p, k, (size_t)tick_dtype, device_window_lds_limit(), cfg_b, cfg_t, batch,
                                             0.0, nullptr, nullptr, tabs.tab4_ok, 1.0, &window_us);
        if (window_us <= column_plan_us(p, batch, (size_t)tick_dtype)) *plan_out = wplan;
    }
    return CP_OK;
}

// Both entry points of the evaluation.  tables_by_kernel: the cost tables reach the device as
// kernel arguments instead of through the pinned staging ring (nothing is allocated then).
static int eval_run(const cp_graph *g, int32_t batch, int32_t k,
                    const uint8_t *assignments, int assign_layout,
                    const int64_t *speeds, const int64_t *bandwidth,
                    void *workspace, size_t workspace_bytes, void *stream,
                    int64_t *cp_out, void *blevel_out, void *tlevel_out, uint64_t *mask_out,
                    int tick_dtype, int out_layout, int plan, int32_t *status_out, cp_profile *profile,
                    bool tables_by_kernel) {
    int rc = check_eval_sizes(g, batch, k, assign_layout, plan);
    if (rc) return rc;
    if (!assignments || !speeds || !bandwidth || !workspace || !status_out) return CP_ERR_NULL;
    if (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64) return CP_ERR_ARG;
    if (out_layout != CP_OUT_VERTEX_MAJOR && out_layout != CP_OUT_PARTITION_MAJOR) return CP_ERR_ARG;
    if (mask_out && (!cp_out || !blevel_out || !tlevel_out)) return CP_ERR_ARG;
    if (!g->device_blob) return CP_ERR_STATE;
    const Packed &p = g->packed;
    if (tick_dtype == CP_TICK_I32 && p.info.min_tick_bytes > 4) return CP_ERR_OVERFLOW;
    if (((uintptr_t)workspace % kAlign) != 0) return CP_ERR_WORKSPACE;
    if (profile && profile->count >= profile->slots) return CP_ERR_STATE;

    CostTables tabs;
    try {
        rc = build_cost_tables(k, speeds, bandwidth, p.narrow, p.info.max_c, p.info.max_t, tabs);
    } catch (const std::bad_alloc &) {
        rc = CP_ERR_ALLOC;
    }
    if (rc) return rc;

    // plan
    WindowCfg cfg_b, cfg_t;
    const bool can_window = tabs.magic_ok && window_fits(p, k, (size_t)tick_dtype,
                                                         device_window_lds_limit(), &cfg_b, &cfg_t, tabs.tab4_ok);
    int use = plan;
    SharedCfg sh_b, sh_t;
    if (plan == CP_PLAN_AUTO) {
        use = CP_PLAN_WAVE_COLUMN;
        if (can_window) {
            // with a mask to write and rows per vertex (or far reads), the shared plans pay for a pass
            // of their own over b and tl (else their t sweep writes it)
            const bool sh_mask_pass = mask_out && !(out_layout == CP_OUT_PARTITION_MAJOR && tick_dtype == CP_TICK_I32 &&
                                                    p.win_t.far_cap == 0);
            const double mask_us = sh_mask_pass ? 5.0 + (double)p.n * batch * (2.0 * tick_dtype + 0.125) / kMaskPassBytesPerUs : 0.0;
            double window_us = 0.0;
            const int wplan = choose_window_plan(p, k, (size_t)tick_dtype, device_window_lds_limit(), cfg_b, cfg_t, batch,
                                                 mask_us, &sh_b, &sh_t, tabs.tab4_ok,
                                                 mask_out && !sh_mask_pass ? 1.22 : 1.0, &window_us);
            // (the mask's cost is left out of the comparison with the wave-column plan, which pays
            // for a pass of its own as well)
            if (window_us - mask_us <= column_plan_us(p, batch, (size_t)tick_dtype)) use = wplan;
        }
    }
    if (use == CP_PLAN_RESIDENT_WINDOW && !can_window) return CP_ERR_ARG;
    // several partitions per workgroup behind one graph stream
    const bool shared = use == CP_PLAN_SHARED_WINDOW_2 || use == CP_PLAN_SHARED_WINDOW_4;
    if (shared && plan != CP_PLAN_AUTO &&
        (!tabs.magic_ok || !shared_fits(p, k, (size_t)tick_dtype, use == CP_PLAN_SHARED_WINDOW_4 ? 4 : 2,
                                        device_window_lds_limit(), &sh_b, &sh_t, tabs.tab4_ok)))
        return CP_ERR_ARG;
    StreamCfg st_b, st_t, st_tm;
    const bool streamed = use == CP_PLAN_STREAMED_WINDOW;
    if (streamed && (!tabs.magic_ok || !stream_fits(p, k, (size_t)tick_dtype, device_window_lds_limit(), &st_b, &st_t)))
        return CP_ERR_ARG;
    const bool windowish = use == CP_PLAN_RESIDENT_WINDOW || shared || streamed;
    const bool columnish = !windowish;       // wave-column, or its persistent column-slice form
    if (use == CP_PLAN_COLUMN_SLICE && (!tabs.magic_ok || k > kMagicMaxK)) return CP_ERR_ARG;
    // the wave-column plan reads CP off the stored b-levels; the window sweeps keep a running maximum
    if (cp_out && !blevel_out && (!windowish || p.win_b.far_cap > 0)) return CP_ERR_ARG;

    // Device ids reach the resident-window sweep either straight from the caller's rows
    // (16-byte loads: the rows must be contiguous, and whole-buffer size and base must be
    // multiples of 16 so that no load leaves the buffer) or gathered into sweep order first.
    const bool rows_ok = assign_layout == CP_ASSIGN_PARTITION_MAJOR &&
                         ((uint64_t)p.n * (uint64_t)batch) % 16 == 0 && ((uintptr_t)assignments % 16) == 0;
    const bool direct_b = rows_ok && p.win_b.direct_ok, direct_t = rows_ok && p.win_t.direct_ok;
    const bool gather_b = windowish && (blevel_out || cp_out) && !direct_b;
    const bool gather_t = windowish && tlevel_out && !direct_t;

    // workspace: only what this call uses (cp_eval_workspace_bytes is an upper bound over
    // every way the call may go)
    const bool need_pT = columnish && assign_layout == CP_ASSIGN_PARTITION_MAJOR;
    size_t need = tables_bytes(k) + (need_pT ? align_up((size_t)p.n * (size_t)batch) : 0);
    const size_t pperm_b_bytes = gather_b ? pperm_bytes(p, p.win_b, batch) : 0;
    const size_t pperm_t_bytes = gather_t ? pperm_bytes(p, p.win_t, batch) : 0;
    need += pperm_b_bytes + pperm_t_bytes;
    const bool by_partition = out_layout == CP_OUT_PARTITION_MAJOR;
    const bool via_scratch = by_partition && columnish;
    const size_t scratch_at = need;
    if (via_scratch) need += 2 * column_scratch_bytes(p, batch, tick_dtype);
    if (workspace_bytes < need) return CP_ERR_WORKSPACE;
    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *d_tab = ws;
    uint8_t *d_pT = ws + tables_bytes(k);
    uint8_t *d_pperm_b = ws + tables_bytes(k);
    uint8_t *d_pperm_t = d_pperm_b + pperm_b_bytes;
    // vertex-major sweep results of the wave-column plan when the caller wants rows per partition
    void *col_b = via_scratch && blevel_out ? (void *)(ws + scratch_at) : blevel_out;
    void *col_t = via_scratch && tlevel_out ? (void *)(ws + scratch_at + column_scratch_bytes(p, batch, tick_dtype))
                                            : tlevel_out;

    hipStream_t st = (hipStream_t)stream;
    hipEvent_t *ev = nullptr;
    int32_t *launches = nullptr;
    if (profile) {
        ev = profile->ev.data() + (size_t)profile->count * (CP_NUM_STAGES + 1);
        launches = profile->launches.data() + (size_t)profile->count * 2;
        launches[0] = launches[1] = 0;
        profile->count++;
    }
#define CP_MARK(i)                                                              \
    do {                                                                        \
        if (ev && hipEventRecord(ev[i], st) != hipSuccess) return CP_ERR_HIP;  \
    } while (0)

    // ---- stage: prep
    CP_MARK(CP_STAGE_PREP);
    rc = launch_clear(cp_out, batch, status_out, stream);
    if (rc) return rc;
    const std::vector<uint64_t> tab_img = table_image(tabs, k);
    rc = upload_tables(tab_img.data(), tab_img.size(), d_tab, st, tables_by_kernel);
    if (rc) return rc;
    const uint8_t *pT = assignments;
    if (need_pT) {
        rc = launch_transpose(assignments, d_pT, p.n, batch, stream);
        if (rc) return rc;
        pT = d_pT;
    }
    const size_t kk = (size_t)k * k;

    SweepLaunch s;
    s.blob = (const uint8_t *)g->device_blob;
    s.c_off = p.c_off;
    s.magic = tabs.magic_ok;
    s.narrow = p.narrow;
    s.tick_bytes = tick_dtype;
    s.n = p.n; s.P = batch; s.k = k; s.L = p.L; s.max_width = p.max_width;
    const uint32_t *d_tab4 = tabs.tab4_ok ? (const uint32_t *)(d_tab + table_entries(k) * 8) : nullptr;
    s.vert_tab4 = d_tab4 ? d_tab4 + 2 * kk : nullptr;
    s.pT = pT;
    s.assign = assignments;
    if (assign_layout == CP_ASSIGN_PARTITION_MAJOR) { s.a_stride_p = p.n; s.a_stride_v = 1; }
    else { s.a_stride_p = 1; s.a_stride_v = batch; }
    s.vert_tab = d_tab + 2 * kk * 8;
    s.status = status_out;
    if (by_partition) { s.out_sv = 1; s.out_sq = p.n; }
    else { s.out_sv = batch; s.out_sq = 1; }
    // With rows per partition the t sweep can write the mask as it goes: it needs the tick's b
    // values staged like the device ids (16-byte loads that must stay inside the b array).
    WindowCfg cfg_tm;
    bool fuse_mask = use == CP_PLAN_RESIDENT_WINDOW && by_partition && mask_out && direct_t &&
                     tick_dtype == CP_TICK_I32 && ((uintptr_t)blevel_out % 16) == 0 &&
                     ((uint64_t)p.n * (uint64_t)batch * 4) % 16 == 0 &&
                     window_config(p.win_t, k, (size_t)tick_dtype, device_window_lds_limit(), cfg_tm, true);
    // the streamed kernel: the same rule without the cost model (its workgroups are small either way)
    const bool fuse_mask_st = streamed && by_partition && mask_out && direct_t && p.win_t.smax >= 4 &&
                              ((uintptr_t)blevel_out % 16) == 0 && ((uint64_t)p.n * (uint64_t)batch * 4) % 16 == 0 &&
                              stream_config(p.win_t, k, device_window_lds_limit() - kSharedStaticLds, true, st_tm);
    if (fuse_mask) {
        // The mask variant costs a little per slice (one more LDS read and a compare) and a fixed
        // amount per tick.  On wide ticks that is far less than a streaming pass over b and tl
        // afterwards (large sparse workload: +0.15 ms against 0.51 ms); on ticks of one or two
        // slices the fixed part outweighs it (5,271 vertices in 251 ticks, 16,384 partitions:
        // +0.70 ms against 0.25 ms).  The same holds where fewer partitions would fit a compute
        // unit with it.
        const double mask_pass_us = 5.0 + (double)p.n * batch * (2.0 * tick_dtype + 0.125) / kMaskPassBytesPerUs;
        fuse_mask = p.win_t.smax >= 4 &&
                    window_sweep_us(p.win_t, cfg_tm, batch) <= window_sweep_us(p.win_t, cfg_t, batch) + mask_pass_us;
    }
    // the shared-window kernel fetches b(v) from the b rows itself, a tick ahead of the comparison
    // (one slice per compute wavefront and tick is what that kernel's bookkeeping assumes)
    const bool fuse_mask_sh = shared && by_partition && mask_out && tick_dtype == CP_TICK_I32 &&
                              sh_t.nc >= p.win_t.smax && p.n < (1 << 24) && p.win_t.far_cap == 0;
    fuse_mask = fuse_mask || fuse_mask_st || fuse_mask_sh;
    // Both sweeps in one launch, a workgroup of each side by side on a compute unit: where one
    // workgroup of either sweep would have the unit to itself, the pair takes 0.66 of the two
    // sweeps' time (measured), which outweighs the mask pass it then needs.
    WindowCfg pr_b, pr_t;
    // (rows per partition only: with rows per vertex the strided stores of two sweeps at once cost
    // more than the overlap gains, 4.9 against 3.8 ms)
    bool paired = use == CP_PLAN_RESIDENT_WINDOW && (blevel_out || cp_out) && tlevel_out && tick_dtype == CP_TICK_I32 &&
                  by_partition &&
                  window_pair_config(p.win_b, p.win_t, k, device_window_lds_limit(), pr_b, pr_t);
    // ... or where every workgroup of both sweeps finds room on the chip at once (small graphs,
    // moderate batches): then the two chains simply run side by side
    const bool alone = window_wg_per_cu(cfg_b) == 1.0 && window_wg_per_cu(cfg_t) == 1.0;
    const bool roomy = paired && !alone &&
                       2.0 * std::ceil((double)batch / 256.0) <= std::min(window_wg_per_cu(pr_b), window_wg_per_cu(pr_t));
    paired = paired && (alone || roomy);
    if (paired && roomy) {
        const double mask_pass_us = mask_out ? 5.0 + (double)p.n * batch * (2.0 * tick_dtype + 0.125) / kMaskPassBytesPerUs : 0.0;
        const double b_us = window_sweep_us(p.win_b, cfg_b, batch), t_us = window_sweep_us(p.win_t, cfg_t, batch);
        const double seq_us = b_us + (fuse_mask ? window_sweep_us(p.win_t, cfg_tm, batch) * 1.06 : t_us + mask_pass_us);
        paired = 1.2 * std::max(b_us, t_us) + mask_pass_us < seq_us;
    } else if (paired) {
        const double mask_pass_us = mask_out ? 5.0 + (double)p.n * batch * (2.0 * tick_dtype + 0.125) / kMaskPassBytesPerUs : 0.0;
        const double b_us = window_sweep_us(p.win_b, cfg_b, batch), t_us = window_sweep_us(p.win_t, cfg_t, batch);
        const double seq_us = b_us + (fuse_mask ? window_sweep_us(p.win_t, cfg_tm, batch) * 1.06 : t_us + mask_pass_us);
        paired = 0.66 * (b_us + t_us) + mask_pass_us < seq_us;
    }
    if (paired) fuse_mask = false;
    if (gather_b) {
        s.win = &p.win_b;
        rc = launch_gather_assign(s, d_pperm_b, stream);
        if (rc) return rc;
    }
    if (gather_t) {
        s.win = &p.win_t;
        rc = launch_gather_assign(s, d_pperm_t, stream);
        if (rc) return rc;
    }

    // ---- stage: b-level sweep
    CP_MARK(CP_STAGE_BLEVEL);
    if (blevel_out || cp_out) {
        s.tsweep = false;
        s.dir = &p.col_b;
        s.win = &p.win_b;
        s.val = windowish ? blevel_out : col_b;
        s.edge_tab = d_tab;
        s.edge_tab4 = d_tab4;
        s.cp_out = windowish ? cp_out : nullptr;
        s.pperm = d_pperm_b;
        s.direct_ids = direct_b;
        if (paired) {
            SweepLaunch t = s;
            t.tsweep = true;
            t.dir = &p.col_t;
            t.win = &p.win_t;
            t.val = tlevel_out;
            t.edge_tab = d_tab + kk * 8;
            t.edge_tab4 = d_tab4 ? d_tab4 + kk : nullptr;
            t.cp_out = nullptr;
            t.pperm = d_pperm_t;
            t.direct_ids = direct_t;
            rc = launch_window_pair(s, t, pr_b, pr_t, stream);
            if (launches) { launches[0] = 1; launches[1] = 0; }
        } else if (shared || streamed) {
            rc = shared ? launch_window_shared(s, sh_b, stream) : launch_window_stream(s, st_b, stream);
            if (launches) launches[0] = 1;
        } else {
            if (use == CP_PLAN_COLUMN_SLICE) {
                rc = launch_column_slice(s, stream);
                if (launches) launches[0] = 1;
            } else {
                rc = use == CP_PLAN_RESIDENT_WINDOW ? launch_window_sweep(s, cfg_b, stream, launches)
                                                    : launch_column_sweep(s, stream, launches);
            }
        }
        if (rc) return rc;
    }

    // ---- stage: critical-path length
    CP_MARK(CP_STAGE_CP);
    if (cp_out && columnish) {
        rc = launch_cp_sources((const int32_t *)(s.blob + p.sources_off), p.info.num_sources,
                               col_b, batch, tick_dtype, cp_out, stream);
        if (rc) return rc;
    }
    if (via_scratch && blevel_out) {
        rc = launch_transpose_ticks(col_b, blevel_out, p.n, batch, tick_dtype, stream);
        if (rc) return rc;
    }

    // ---- stage: t-level sweep
    CP_MARK(CP_STAGE_TLEVEL);
    if (tlevel_out && !paired) {
        s.tsweep = true;
        s.dir = &p.col_t;
        s.win = &p.win_t;
        s.val = windowish ? tlevel_out : col_t;
        s.edge_tab = d_tab + kk * 8;
        s.edge_tab4 = d_tab4 ? d_tab4 + kk : nullptr;
        s.cp_out = nullptr;
        s.pperm = d_pperm_t;
        s.direct_ids = direct_t;
        if (fuse_mask) {
            // the t sweep sets the mask bits itself (tl + b = CP is known when a vertex is published)
            rc = launch_zero_words(mask_out, (int64_t)batch * (((int64_t)p.n + 63) / 64), stream);
            if (rc) return rc;
            s.mask_b = blevel_out;
            s.mask_cp = cp_out;
            s.mask_out = mask_out;
        }
        if (shared || streamed) {
            rc = shared ? launch_window_shared(s, sh_t, stream)
                        : launch_window_stream(s, fuse_mask ? st_tm : st_t, stream);
            if (launches) launches[1] = 1;
        } else {
            if (use == CP_PLAN_COLUMN_SLICE) {
                rc = launch_column_slice(s, stream);
                if (launches) launches[1] = 1;
            } else {
                rc = use == CP_PLAN_RESIDENT_WINDOW
                         ? launch_window_sweep(s, fuse_mask ? cfg_tm : cfg_t, stream, launches ? launches + 1 : nullptr)
                         : launch_column_sweep(s, stream, launches ? launches + 1 : nullptr);
            }
        }
        if (rc) return rc;
        if (via_scratch) {
            rc = launch_transpose_ticks(col_t, tlevel_out, p.n, batch, tick_dtype, stream);
            if (rc) return rc;
        }
    }

    // ---- stage: mask
    CP_MARK(CP_STAGE_MASK);
    if (mask_out && !fuse_mask) {
        rc = launch_mask(blevel_out, tlevel_out, cp_out, p.n, batch, tick_dtype, by_partition, mask_out, stream);
        if (rc) return rc;
    }
    CP_MARK(CP_NUM_STAGES);
#undef CP_MARK
    return CP_OK;
}

int cp_eval(const cp_graph *g, int32_t batch, int32_t k,
            const uint8_t *assignments, int assign_layout,
            const int64_t *speeds, const int64_t *bandwidth,
            void *workspace, size_t workspace_bytes, void *stream,
            int64_t *cp_out, void *blevel_out, void *tlevel_out, uint64_t *mask_out,
            int tick_dtype, int out_layout, int plan, int32_t *status_out, cp_profile *profile) {
    return eval_run(g, batch, k, assignments, assign_layout, speeds, bandwidth, workspace, workspace_bytes, stream,
                    cp_out, blevel_out, tlevel_out, mask_out, tick_dtype, out_layout, plan, status_out, profile,
                    /*tables_by_kernel=*/false);
}

int cp_eval_static(const cp_graph *g, int32_t batch, int32_t k,
                   const uint8_t *assignments, int assign_layout,
                   const int64_t *speeds, const int64_t *bandwidth, void *stream,
                   int64_t *cp_out, void *blevel_out, void *tlevel_out, uint64_t *mask_out,
                   int tick_dtype, int out_layout, int plan, int32_t *status_out) {
    if (k > CP_STATIC_MAX_K) return CP_ERR_SIZE;
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc) return rc;
    // eval_run answers CP_ERR_WORKSPACE when the call needs more than the array holds
    return eval_run(g, batch, k, assignments, assign_layout, speeds, bandwidth, ws, (size_t)CP_STATIC_SCRATCH_BYTES,
                    stream, cp_out, blevel_out, tlevel_out, mask_out, tick_dtype, out_layout, plan, status_out,
                    nullptr, /*tables_by_kernel=*/true);
}

int cp_critical_path(const cp_graph *g, int32_t batch, int32_t k,
                     const uint8_t *assignments, int assign_layout,
                     const int64_t *speeds, const int64_t *bandwidth,
                     const void *blevel, const int64_t *cp, int tick_dtype, int b_layout,
                     void *workspace, size_t workspace_bytes, void *stream,
                     int32_t max_len, int32_t *path_out, int32_t *len_out, int32_t *status_out) {
    int rc = check_eval_sizes(g, batch, k, assign_layout, CP_PLAN_AUTO);
    if (rc) return rc;
    if (b_layout != CP_OUT_VERTEX_MAJOR && b_layout != CP_OUT_PARTITION_MAJOR) return CP_ERR_ARG;
    if (!assignments || !speeds || !bandwidth || !blevel || !cp || !workspace || !path_out || !len_out ||
        !status_out)
        return CP_ERR_NULL;
    if (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64) return CP_ERR_ARG;
    if (!g->device_blob) return CP_ERR_STATE;
    const Packed &p = g->packed;
    if (tick_dtype == CP_TICK_I32 && p.info.min_tick_bytes > 4) return CP_ERR_OVERFLOW;
    if (max_len < p.L) return CP_ERR_SIZE;      // a path has at most one vertex per level
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < tables_bytes(k)) return CP_ERR_WORKSPACE;
    CostTables tabs;
    try {
        rc = build_cost_tables(k, speeds, bandwidth, p.narrow, p.info.max_c, p.info.max_t, tabs);
    } catch (const std::bad_alloc &) {
        rc = CP_ERR_ALLOC;
    }
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    rc = launch_clear(nullptr, 1, status_out, stream);
    if (rc) return rc;
    uint8_t *d_tab = (uint8_t *)workspace;
    const void *tab_src = tabs.magic_ok ? (const void *)tabs.magic.data() : (const void *)tabs.divisor.data();
    rc = upload_tables(tab_src, table_entries(k), d_tab, st);
    if (rc) return rc;
    SweepLaunch s;
    s.blob = (const uint8_t *)g->device_blob;
    s.dir = &p.col_b;
    s.c_off = p.c_off;
    s.magic = tabs.magic_ok;
    s.narrow = p.narrow;
    s.tick_bytes = tick_dtype;
    s.n = p.n; s.P = batch; s.k = k; s.L = p.L;
    s.assign = assignments;
    if (assign_layout == CP_ASSIGN_PARTITION_MAJOR) { s.a_stride_p = p.n; s.a_stride_v = 1; }
    else { s.a_stride_p = 1; s.a_stride_v = batch; }
    s.val = const_cast<void *>(blevel);
    if (b_layout == CP_OUT_PARTITION_MAJOR) { s.out_sv = 1; s.out_sq = p.n; }
    else { s.out_sv = batch; s.out_sq = 1; }
    s.edge_tab = d_tab;
    s.vert_tab = d_tab + 2 * (size_t)k * k * 8;
    s.status = status_out;
    return launch_critical_path(s, (const int32_t *)(s.blob + p.sources_off), p.info.num_sources, cp,
                                max_len, path_out, len_out, stream);
}

int cp_pct_order_workspace_bytes(const cp_graph *g, int32_t batch, int32_t k, int64_t max_b,
                                 size_t *out_bytes) {
    if (!out_bytes) return CP_ERR_NULL;
    PctPlan plan;
    int rc = pct_plan(g, batch, k, max_b, plan);
    if (rc) return rc;
    *out_bytes = plan.total;
    return CP_OK;
}

int cp_pct_order(const cp_graph *g, int32_t batch, int32_t k,
                 const uint8_t *assignments, int assign_layout,
                 const void *blevel, int tick_dtype, int b_layout, int64_t max_b,
                 void *workspace, size_t workspace_bytes, void *stream,
                 int32_t *order_out, int32_t *seg_out, int32_t *status_out) {
    PctPlan plan;
    if (b_layout != CP_OUT_VERTEX_MAJOR && b_layout != CP_OUT_PARTITION_MAJOR) return CP_ERR_ARG;
    int rc = pct_plan(g, batch, k, max_b, plan);
    if (rc) return rc;
    if (assign_layout != CP_ASSIGN_PARTITION_MAJOR && assign_layout != CP_ASSIGN_VERTEX_MAJOR) return CP_ERR_ARG;
    if (!assignments || !blevel || !workspace || !order_out || !seg_out || !status_out) return CP_ERR_NULL;
    if (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64) return CP_ERR_ARG;
    if (!g->device_blob) return CP_ERR_STATE;
    const Packed &p = g->packed;
    if (tick_dtype == CP_TICK_I32 && p.info.min_tick_bytes > 4) return CP_ERR_OVERFLOW;
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < plan.total) return CP_ERR_WORKSPACE;
    rc = launch_clear(nullptr, 1, status_out, stream);
    if (rc) return rc;
    uint8_t *ws = (uint8_t *)workspace;
    PctOrderLaunch s;
    s.n = p.n; s.P = batch; s.k = k;
    s.b = blevel;
    s.b_by_partition = b_layout == CP_OUT_PARTITION_MAJOR;
    s.tick_bytes = tick_dtype;
    s.assign = assignments;
    if (assign_layout == CP_ASSIGN_PARTITION_MAJOR) { s.a_stride_p = p.n; s.a_stride_v = 1; }
    else { s.a_stride_p = 1; s.a_stride_v = batch; }
    s.max_b = plan.max_b;
    s.b_bits = plan.b_bits; s.key_bits = plan.key_bits; s.key_bytes = plan.key_bytes;
    s.keys_a = ws;
    s.keys_b = ws + plan.keys_bytes;
    s.vals_tmp = (int32_t *)(ws + 2 * plan.keys_bytes);
    s.counts = (uint32_t *)(ws + 2 * plan.keys_bytes + plan.vals_bytes);
    s.order_out = order_out;
    s.seg_out = seg_out;
    s.status = status_out;
    return launch_pct_order(s, stream);
}

int cp_validate(int32_t n, int32_t batch, int32_t k, const uint8_t *assignments, int assign_layout,
                int64_t num_pairs, const int32_t *pairs, int64_t num_pins, const int32_t *pins,
                void *stream, uint8_t *valid_out, int32_t *violations_out, int32_t *status_out) {
    if (n < 1 || batch < 1 || k < 1 || k > 255 || num_pairs < 0 || num_pins < 0) return CP_ERR_SIZE;
    if (assign_layout != CP_ASSIGN_PARTITION_MAJOR && assign_layout != CP_ASSIGN_VERTEX_MAJOR) return CP_ERR_ARG;
    if (!assignments || !valid_out || !status_out || (num_pairs > 0 && !pairs) || (num_pins > 0 && !pins))
        return CP_ERR_NULL;
    int rc = launch_clear(nullptr, 1, status_out, stream);
    if (rc) return rc;
    const int64_t sp = assign_layout == CP_ASSIGN_PARTITION_MAJOR ? n : 1;
    const int64_t sv = assign_layout == CP_ASSIGN_PARTITION_MAJOR ? 1 : batch;
    return launch_validate(assignments, sp, sv, n, batch, k, num_pairs, pairs, num_pins, pins, valid_out,
                           violations_out, status_out, stream);
}

int cp_simulate_workspace_bytes(const cp_graph *g, int32_t batch, int32_t k, int policy, int with_tie,
                                size_t *out_bytes) {
    if (!out_bytes) return CP_ERR_NULL;
    SimPlan plan;
    int rc = sim_plan(g, batch, k, policy, with_tie != 0, plan);
    if (rc) return rc;
    *out_bytes = plan.total;
    return CP_OK;
}

int cp_simulate(const cp_graph *g, int32_t batch, int32_t k,
                const uint8_t *assignments, int assign_layout,
                const int64_t *speeds, const int64_t *bandwidth, int policy,
                const void *blevel, int tick_dtype, int b_layout, const int32_t *tie,
                void *workspace, size_t workspace_bytes, void *stream,
                int64_t *makespan_out, int32_t *start_out, int32_t *status_out) {
    SimPlan plan;
    int rc = sim_plan(g, batch, k, policy, tie != nullptr, plan);
    if (rc) return rc;
    if (assign_layout != CP_ASSIGN_PARTITION_MAJOR && assign_layout != CP_ASSIGN_VERTEX_MAJOR) return CP_ERR_ARG;
    if (!assignments || !speeds || !bandwidth || !workspace || !makespan_out || !status_out) return CP_ERR_NULL;
    if (plan.pct) {
        if (!blevel) return CP_ERR_NULL;
        if (b_layout != CP_OUT_VERTEX_MAJOR && b_layout != CP_OUT_PARTITION_MAJOR) return CP_ERR_ARG;
        if (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64) return CP_ERR_ARG;
    }
    if (!g->device_blob) return CP_ERR_STATE;
    const Packed &p = g->packed;
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < plan.total) return CP_ERR_WORKSPACE;
    CostTables tabs;
    try {
        rc = build_cost_tables(k, speeds, bandwidth, p.narrow, p.info.max_c, p.info.max_t, tabs);
    } catch (const std::bad_alloc &) {
        rc = CP_ERR_ALLOC;
    }
    if (rc) return rc;

    // every vertex takes a tick or more; the shortest execution and transfer times give the
    // span of decision times that may be served together.  No time may reach 2^31: at every
    // moment before the end either some device is busy (at most the summed execution times in
    // all) or every device waits for a transfer on one chain of dependent vertices (at most
    // the longest path's transfers, which the raw path bound covers, and so does L - 1 times the
    // longest transfer).
    int64_t s_min = speeds[0], s_max = speeds[0], b_min = INT64_MAX, b_max = 1;
    for (int i = 0; i < k; ++i) {
        s_min = std::min(s_min, speeds[i]);
        s_max = std::max(s_max, speeds[i]);
        for (int j = 0; j < k; ++j)
            if (i != j) {
                b_min = std::min(b_min, bandwidth[(size_t)i * k + j]);
                b_max = std::max(b_max, bandwidth[(size_t)i * k + j]);
            }
    }
    if (b_min == INT64_MAX) b_min = 1;
    uint64_t min_c = 0, min_t = 0;
    long double sum_w = 0;
    if (p.narrow) min_weights<uint32_t>(p, (uint64_t)s_min, min_c, min_t, sum_w);
    else min_weights<int64_t>(p, (uint64_t)s_min, min_c, min_t, sum_w);
    if (min_c < 1) return CP_ERR_ARG;
    auto ceil_div = [](uint64_t a, uint64_t d) { return a / d + (a % d != 0); };
    // a chain has at most one vertex per level, so L - 1 transfers of at most ceil(max t / min B)
    const long double chain = std::min<long double>(
        (long double)p.info.raw_path_bound,
        (long double)(p.L - 1) * (long double)ceil_div((uint64_t)p.info.max_t, (uint64_t)b_min));
    if (sum_w + chain >= 2147483647.0L) return CP_ERR_OVERFLOW;
    const uint64_t w_min = ceil_div(min_c, (uint64_t)s_max);
    const uint64_t x_min = (p.m == 0 || min_t == 0) ? 0 : ceil_div(min_t, (uint64_t)b_max);
    const uint64_t window = std::min<uint64_t>(w_min + x_min - 1, 1u << 30);

    hipStream_t st = (hipStream_t)stream;
    rc = launch_clear(nullptr, 1, status_out, stream);
    if (rc) return rc;
    uint8_t *ws = (uint8_t *)workspace;
    const void *tab_src = tabs.magic_ok ? (const void *)tabs.magic.data() : (const void *)tabs.divisor.data();
    rc = upload_tables(tab_src, table_entries(k), ws, st);
    if (rc) return rc;
    SimulateLaunch s;
    s.blob = (const uint8_t *)g->device_blob;
    s.succ = &p.col_b;
    s.pred = &p.col_t;
    s.c_off = p.c_off;
    s.magic = tabs.magic_ok;
    s.narrow = p.narrow;
    s.pct = plan.pct;
    s.n = p.n; s.P = batch; s.k = k;
    s.window = (uint32_t)window;
    // One partition per wavefront until the batch alone fills the GPU several times over (8,192
    // wavefronts are 8 per SIMD); past that, partitions with few devices share a wavefront.
    s.groups = (int32_t)std::max<int64_t>(1, std::min<int64_t>(kWave / k, batch / 8192));
    s.assign = assignments;
    if (assign_layout == CP_ASSIGN_PARTITION_MAJOR) { s.a_stride_p = p.n; s.a_stride_v = 1; }
    else { s.a_stride_p = 1; s.a_stride_v = batch; }
    if (plan.pct) {
        s.b = blevel;
        s.b_bytes = tick_dtype;
        if (b_layout == CP_OUT_PARTITION_MAJOR) { s.b_sv = 1; s.b_sq = p.n; }
        else { s.b_sv = batch; s.b_sq = 1; }
    }
    s.edge_tab = ws;
    s.vert_tab = ws + 2 * (size_t)k * k * 8;
    uint8_t *at = ws + plan.tab;
    if (plan.with_tie) {
        s.tie = tie;
        s.tie_inv = (int32_t *)at;
        at += plan.tie_inv;
    }
    s.ready = (int32_t *)at; at += plan.per_i32;
    s.need = (int32_t *)at; at += plan.per_i32;
    s.inbox = (int32_t *)at; at += plan.per_i32;
    s.pending = (uint64_t *)at; at += plan.per_u64;
    if (plan.pct) { s.available = (uint64_t *)at; at += plan.per_u64; }
    s.makespan = makespan_out;
    s.start = start_out;
    s.status = status_out;
    return launch_simulate(s, stream);
}

int cp_ranks_workspace_bytes(const cp_graph *g, size_t *out_bytes) {
    if (!g || !out_bytes) return CP_ERR_NULL;
    size_t eval = 0;
    int rc = cp_eval_workspace_bytes(g, 1, 1, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO, CP_OUT_VERTEX_MAJOR,
                                     g->packed.info.min_tick_bytes, &eval);
    if (rc) return rc;
    const size_t n = (size_t)g->packed.n, T = (size_t)g->packed.info.min_tick_bytes;
    *out_bytes = align_up(eval) + align_up(n) + 2 * align_up(n * T) + 2 * kAlign;
    return CP_OK;
}

int cp_ranks(const cp_graph *g, void *workspace, size_t workspace_bytes, void *stream,
             int64_t *up_out, int64_t *down_out, int64_t *total_out) {
    if (!g || !workspace) return CP_ERR_NULL;
    if (!up_out && !down_out && !total_out) return CP_ERR_NULL;
    if (!g->device_blob) return CP_ERR_STATE;
    size_t need = 0, eval = 0;
    int rc = cp_ranks_workspace_bytes(g, &need);
    if (rc) return rc;
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < need) return CP_ERR_WORKSPACE;
    rc = cp_eval_workspace_bytes(g, 1, 1, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO, CP_OUT_VERTEX_MAJOR,
                                 g->packed.info.min_tick_bytes, &eval);
    if (rc) return rc;
    const Packed &p = g->packed;
    const size_t n = (size_t)p.n, T = (size_t)p.info.min_tick_bytes;
    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *d_assign = ws + align_up(eval);
    uint8_t *d_b = d_assign + align_up(n);
    uint8_t *d_tl = d_b + align_up(n * T);
    int64_t *d_cp = (int64_t *)(d_tl + align_up(n * T));
    int32_t *d_status = (int32_t *)((uint8_t *)d_cp + kAlign);
    rc = launch_zero_bytes(d_assign, (int64_t)n, stream);
    if (rc) return rc;
    // one device of speed 1: w(v) = c(v), nothing is ever transferred
    const int64_t one = 1;
    rc = cp_eval(g, 1, 1, d_assign, CP_ASSIGN_PARTITION_MAJOR, &one, &one, ws, align_up(eval), stream, d_cp,
                 d_b, d_tl, nullptr, (int)T, CP_OUT_VERTEX_MAJOR, CP_PLAN_AUTO, d_status, nullptr);
    if (rc) return rc;
    return launch_ranks(d_b, d_tl, (const uint8_t *)g->device_blob + p.c_off, p.narrow, (int)T, p.n, up_out,
                        down_out, total_out, stream);
}

int cp_profile_create(int32_t slots, cp_profile **out) {
    if (!out) return CP_ERR_NULL;
    *out = nullptr;
    if (slots < 1 || slots > 65536) return CP_ERR_SIZE;
    cp_profile *p = new (std::nothrow) cp_profile;
    if (!p) return CP_ERR_ALLOC;
    p->slots = slots;
    try {
        p->ev.assign((size_t)slots * (CP_NUM_STAGES + 1), nullptr);
        p->launches.assign((size_t)slots * 2, 0);
    } catch (const std::bad_alloc &) {
        delete p;
        return CP_ERR_ALLOC;
    }
    for (auto &e : p->ev)
        if (hipEventCreate(&e) != hipSuccess) {
            cp_profile_destroy(p);
            return CP_ERR_HIP;
        }
    *out = p;
    return CP_OK;
}

int cp_profile_reset(cp_profile *p) {
    if (!p) return CP_ERR_NULL;
    p->count = 0;
    return CP_OK;
}

int cp_profile_count(const cp_profile *p, int32_t *out) {
    if (!p || !out) return CP_ERR_NULL;
    *out = p->count;
    return CP_OK;
}

int cp_profile_read(const cp_profile *p, int32_t slot, float ms_out[CP_NUM_STAGES],
                    int32_t sweep_launches[2]) {
    if (!p || !ms_out) return CP_ERR_NULL;
    if (slot < 0 || slot >= p->count) return CP_ERR_STATE;
    const hipEvent_t *ev = p->ev.data() + (size_t)slot * (CP_NUM_STAGES + 1);
    for (int i = 0; i < CP_NUM_STAGES; ++i)
        if (hipEventElapsedTime(&ms_out[i], ev[i], ev[i + 1]) != hipSuccess) return CP_ERR_HIP;
    if (sweep_launches) {
        sweep_launches[0] = p->launches[(size_t)slot * 2];
        sweep_launches[1] = p->launches[(size_t)slot * 2 + 1];
    }
    return CP_OK;
}

void cp_profile_destroy(cp_profile *p) {
    if (!p) return;
    for (auto e : p->ev)
        if (e) (void)hipEventDestroy(e);
    delete p;
}

int cp_cost_magic(int64_t divisor, int64_t max_dividend, uint32_t *mul, uint32_t *dm1) {
    if (!mul || !dm1) return CP_ERR_NULL;
    if (divisor < 1 || max_dividend < 0) return CP_ERR_SIZE;
    int64_t s = divisor, b[1] = {1};
    CostTables t;
    // one device of speed `divisor`: the vertex entry carries the constants
    int rc = build_cost_tables(1, &s, b, true, max_dividend, 0, t);
    if (rc) return rc;
    if (!t.magic_ok) return 0;
    *mul = t.magic[2].mul;
    *dm1 = t.magic[2].dm1;
    return 1;
}

int cp_cost_compact(int64_t divisor, int64_t max_dividend, uint32_t *entry) {
    if (!entry) return CP_ERR_NULL;
    if (divisor < 1 || max_dividend < 0) return CP_ERR_SIZE;
    int64_t s = divisor, b[1] = {1};
    CostTables t;
    int rc = build_cost_tables(1, &s, b, true, max_dividend, 0, t);
    if (rc) return rc;
    if (!t.tab4_ok) return 0;
    *entry = t.tab4[2];
    return 1;
}

int cp_window_shape(const cp_graph *g, int32_t k, int tick_dtype, int tsweep, int32_t shape[8]) {
    if (!g || !shape) return CP_ERR_NULL;
    if (k < 1 || k > kMagicMaxK || (tick_dtype != CP_TICK_I32 && tick_dtype != CP_TICK_I64)) return CP_ERR_ARG;
    const Packed &p = g->packed;
    if (!p.have_window) return CP_ERR_ARG;
    const WindowDir &d = tsweep ? p.win_t : p.win_b;
    WindowCfg c;
    if (!window_config(d, k, (size_t)tick_dtype, kWindowLdsLimit, c)) return CP_ERR_ARG;
    shape[0] = c.nl; shape[1] = c.nlw; shape[2] = c.nfw; shape[3] = c.nc; shape[4] = c.dr; shape[5] = c.groups;
    shape[6] = (d.smax + c.nc - 1) / c.nc;
    shape[7] = (int32_t)c.lds_bytes;
    return CP_OK;
}

const char *cp_error_string(int code) {
    switch (code) {
        case CP_OK: return "ok";
        case CP_ERR_NULL: return "a required pointer is NULL";
        case CP_ERR_SIZE: return "size out of range (n, m, L, batch or k)";
        case CP_ERR_CSR: return "malformed CSR arrays, or successor and predecessor arrays disagree";
        case CP_ERR_LEVELS: return "level index is not a partition of the vertices, or an edge does not go to a higher level";
        case CP_ERR_NEGATIVE: return "negative vertex complexity or edge volume";
        case CP_ERR_SPEED: return "device speed < 1";
        case CP_ERR_BANDWIDTH: return "off-diagonal bandwidth < 1";
        case CP_ERR_OVERFLOW: return "longest raw path too large for the requested tick type";
        case CP_ERR_WORKSPACE: return "workspace or blob too small or misaligned";
        case CP_ERR_HIP: return "a HIP runtime call failed";
        case CP_ERR_STATE: return "graph not uploaded, or profile full / slot not filled";
        case CP_ERR_ARG: return "bad enum value, output dependency not met, or plan not runnable";
        case CP_ERR_ALLOC: return "host allocation failed";
        default: return "unknown error code";
    }
}

}  // extern "C"
