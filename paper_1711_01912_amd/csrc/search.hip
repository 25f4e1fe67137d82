// Critical-path move search on top of cp_eval.  The paper's path-based strategies
// (section 3.2) place the critical path first because it decides the running time;
// this is the same idea as a descent over partitions: all single moves of a vertex of
// the current critical path to another device are evaluated in batches, the best one
// that meets the placement constraints (section 2) is taken while it shortens the
// critical path.  The evaluation is the library's own batched cp_eval; the kernels here
// only build the candidates, pick the minimum and apply the move.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cstdint>
#include <new>
#include <vector>

#include "cpeval_internal.hpp"
#include "device_math.hpp"
#include "launch.hpp"

namespace cpeval {

namespace {

// Candidate number j = i * (k-1) + r moves path vertex number i to the r-th device other
// than its own.  Rows first + 0 .. first + count - 1 are written, 16 bytes per thread.
__global__ __launch_bounds__(256) void neighbours_kernel(const uint8_t *__restrict__ base,
                                                         const int32_t *__restrict__ path, int32_t n, int32_t k,
                                                         int32_t first, int32_t count, uint8_t *__restrict__ out,
                                                         int vector_ok) {
    const int64_t at = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 16;
    if (at >= n) return;
    for (int32_t local = blockIdx.y; local < count; local += gridDim.y) {
        const int32_t j = first + local;
        const int32_t v = path[j / (k - 1)];
        const int32_t r = j % (k - 1);
        uint8_t *row = out + (int64_t)local * n;
        if (vector_ok) {
            uint4 x = *(const uint4 *)(base + at);
            if (v >= at && v < at + 16) {
                uint8_t *b8 = (uint8_t *)&x;
                const int32_t own = b8[v - at];
                b8[v - at] = (uint8_t)(r < own ? r : r + 1);
            }
            *(uint4 *)(row + at) = x;
        } else {
            const int64_t end = min((int64_t)n, at + 16);
            for (int64_t i = at; i < end; ++i) {
                const int32_t own = base[i];
                row[i] = i == v ? (uint8_t)(r < own ? r : r + 1) : (uint8_t)own;
            }
        }
    }
}

struct Best {
    long long value;    // smallest CP so far, LLONG_MAX = none
    long long index;    // its candidate number, -1 = none
};

__global__ void best_reset_kernel(Best *best) {
    best->value = LLONG_MAX;
    best->index = -1;
}

// Lowest-numbered minimum of cp[0..count) over the valid entries, merged into *best.
// Chunks arrive in increasing candidate order, so a tie keeps the earlier candidate.
__global__ __launch_bounds__(1024) void argmin_merge_kernel(const int64_t *__restrict__ cp,
                                                            const uint8_t *__restrict__ valid, int32_t count,
                                                            int32_t first, Best *best) {
    __shared__ long long sv[16], si[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    long long v = LLONG_MAX, idx = LLONG_MAX;
    for (int32_t i = tid; i < count; i += 1024) {
        if (valid && !valid[i]) continue;
        const long long c = cp[i];
        if (c < v) { v = c; idx = i; }          // i grows, so the first minimum stays
    }
    for (int off = 32; off > 0; off >>= 1) {
        const long long ov = __shfl_xor(v, off), oi = __shfl_xor(idx, off);
        if (ov < v || (ov == v && oi < idx)) { v = ov; idx = oi; }
    }
    if (lane == 0) { sv[wave] = v; si[wave] = idx; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 16; ++w)
            if (sv[w] < v || (sv[w] == v && si[w] < idx)) { v = sv[w]; idx = si[w]; }
        if (idx != LLONG_MAX && v < best->value) {
            best->value = v;
            best->index = (long long)first + idx;
        }
    }
}

// base[path vertex] = its new device; the move is also left in move[0..1] = {vertex, device}.
__global__ void apply_move_kernel(uint8_t *base, const int32_t *path, int32_t k, const Best *best, int32_t *move) {
    const int32_t j = (int32_t)best->index;
    const int32_t v = path[j / (k - 1)];
    const int32_t r = j % (k - 1);
    const int32_t own = base[v];
    const int32_t d = r < own ? r : r + 1;
    base[v] = (uint8_t)d;
    move[0] = v;
    move[1] = d;
}

// ---------------------------------------------------------------- Critical Path strategy (section 3.2.2)

constexpr int kSeedMaxK = 64;        // one lane per device

struct SeedArgs {
    const void *c;            // uint32 or int64 [n]
    const int32_t *path;      // device-free critical path
    const int32_t *len;
    uint8_t *assign;          // [n]
    int32_t n, k, fastest, magic;
    Magic mg[kSeedMaxK];
    int64_t speed[kSeedMaxK];
};

__global__ void seed_mark_kernel(SeedArgs a) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < a.n) a.assign[i] = 0xff;          // not placed yet
}

__global__ void seed_path_kernel(SeedArgs a) {
    const int32_t len = *a.len;
    for (int32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < len; i += gridDim.x * blockDim.x)
        a.assign[a.path[i]] = (uint8_t)a.fastest;
}

// Minimum over lanes 0 .. span-1 (span a power of two), valid in those lanes: inside a row
// of 16 by register permutations (swap neighbours, swap pairs, mirror 8, mirror 16), across
// rows by shuffles.
__device__ __forceinline__ long long min_over_lanes(long long x, int span) {
    x = min(x, dpp_i64<0xB1>(x));                     // quad_perm 1,0,3,2
    if (span > 2) x = min(x, dpp_i64<0x4E>(x));       // quad_perm 2,3,0,1
    if (span > 4) x = min(x, dpp_i64<0x141>(x));      // row_half_mirror
    if (span > 8) x = min(x, dpp_i64<0x140>(x));      // row_mirror
    if (span > 16) x = min(x, __shfl_xor(x, 16));
    if (span > 32) x = min(x, __shfl_xor(x, 32));
    return x;
}

// The same on 32-bit numbers over the first 16 lanes (WIDE: all 64), every step taken: lanes
// past the devices hold the largest number and never win.
template <bool WIDE>
__device__ __forceinline__ uint32_t min_over_lanes_u32(uint32_t x) {
    x = min(x, dpp_u32<0xB1>(x));
    x = min(x, dpp_u32<0x4E>(x));
    x = min(x, dpp_u32<0x141>(x));
    x = min(x, dpp_u32<0x140>(x));
    if (WIDE) {
        x = min(x, (uint32_t)__shfl_xor((int)x, 16));
        x = min(x, (uint32_t)__shfl_xor((int)x, 32));
    }
    return x;
}

// One batch of up to 64 vertices on relative 32-bit loads (see seed_greedy_kernel): lane j of
// `dev` holds vertex j's device (0xff: not placed yet), of `cv` its c.  No branch but the one
// that skips a placed vertex.
template <bool MAGIC, bool WIDE>
__device__ __forceinline__ void seed_batch_u32(uint32_t &rel, int32_t &dev, uint32_t cv, int cnt, bool mine,
                                               const Magic &mg, uint64_t sp, int lane) {
    for (int j = 0; j < cnt; ++j) {
        if (__builtin_amdgcn_readlane(dev, j) != 0xff) continue;            // on the critical path
        const uint32_t cj = (uint32_t)__builtin_amdgcn_readlane((int)cv, j);
        const uint32_t w = MAGIC ? magic_div(cj, mg) : (uint32_t)plain_div((uint64_t)cj, sp);
        const uint32_t val = mine ? rel + w : 0xffffffffu;
        const uint32_t best = min_over_lanes_u32<WIDE>(val);
        const int chosen = __ffsll((long long)__ballot(val == best)) - 1;  // lowest device on ties
        rel = lane == chosen ? val : rel;
        dev = lane == j ? chosen : dev;
    }
}

__device__ __forceinline__ long long lane0_i64(long long x) {
    return (long long)((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x) |
                       (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32)) << 32);
}

// The load rule is a chain: every choice changes the loads the next one sees.  One
// wavefront walks the vertices in order, lane d keeps load(d); 64 vertices are fetched
// at a time and handed round with readlane.  The chain is the wavefront's own instruction
// latency, so a batch of 64 vertices runs on 32-bit numbers where it can: loads relative
// to the smallest one, which stay below 2^32 - 1 through the batch when (largest - smallest
// load) + 64 * (largest c of the batch) does -- an execution time is at most c.  The choices
// are the same, a minimum and its ties do not move when every load loses the same amount.
template <typename WT>
__global__ __launch_bounds__(64) void seed_greedy_kernel(SeedArgs a) {
    const int lane = threadIdx.x;
    const WT *c = (const WT *)a.c;
    const bool mine = lane < a.k;
    const Magic mg = a.mg[mine ? lane : 0];
    const uint64_t sp = (uint64_t)a.speed[mine ? lane : 0];
    auto cost = [&](uint64_t cv) -> long long {
        return a.magic ? (long long)magic_div((uint32_t)cv, mg) : (long long)plain_div(cv, sp);
    };
    // the critical path is placed first: its execution times on the fastest device
    long long load = 0;
    {
        const Magic mf = a.mg[a.fastest];
        const uint64_t sf = (uint64_t)a.speed[a.fastest];
        const int32_t len = *a.len;
        long long part = 0;
        for (int32_t i = lane; i < len; i += 64) {
            const uint64_t cv = (uint64_t)c[a.path[i]];
            part += a.magic ? (long long)magic_div((uint32_t)cv, mf) : (long long)plain_div(cv, sf);
        }
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
        if (lane == a.fastest) load = part;
    }
    int span = 1;
    while (span < a.k) span <<= 1;
    for (int32_t v0 = 0; v0 < a.n; v0 += 64) {
        const int32_t v = v0 + lane;
        const uint64_t cv = v < a.n ? (uint64_t)c[v] : 0;
        int32_t dev = v < a.n ? (int32_t)a.assign[v] : 0;
        const int32_t cnt = min(64, a.n - v0);
        // smallest and largest load, largest c of the batch (the same in every lane)
        const long long low = lane0_i64(min_over_lanes(mine ? load : LLONG_MAX, span));
        const long long high = -lane0_i64(min_over_lanes(mine ? -load : LLONG_MAX, span));
        unsigned long long cmax = cv;
        for (int off = 32; off > 0; off >>= 1) cmax = max(cmax, (unsigned long long)__shfl_xor((long long)cmax, off));
        const bool narrow = cmax < (1ull << 32) && (unsigned long long)(high - low) + 64 * cmax < 0xffffffffull;
        if (narrow) {
            uint32_t rel = mine ? (uint32_t)(load - low) : 0xffffffffu;
            if (a.magic) {
                if (span <= 16) seed_batch_u32<true, false>(rel, dev, (uint32_t)cv, cnt, mine, mg, sp, lane);
                else seed_batch_u32<true, true>(rel, dev, (uint32_t)cv, cnt, mine, mg, sp, lane);
            } else {
                if (span <= 16) seed_batch_u32<false, false>(rel, dev, (uint32_t)cv, cnt, mine, mg, sp, lane);
                else seed_batch_u32<false, true>(rel, dev, (uint32_t)cv, cnt, mine, mg, sp, lane);
            }
            if (mine) load = low + (long long)rel;
        } else {
            for (int j = 0; j < cnt; ++j) {
                if (__builtin_amdgcn_readlane(dev, j) != 0xff) continue;
                const uint64_t cj = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)cv, j) |
                                    (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(cv >> 32), j) << 32;
                const long long val = mine ? load + cost(cj) : LLONG_MAX;
                // the devices sit in lanes 0 .. k-1: a reduction over the next power of two covers them
                const long long best = min_over_lanes(val, span);
                const int chosen = __ffsll((long long)__ballot(val == best)) - 1;
                if (lane == chosen) load = val;
                if (lane == j) dev = chosen;
            }
        }
        if (v < a.n) a.assign[v] = (uint8_t)dev;
    }
}

struct SearchLayout {
    size_t eval_ws = 0, cand = 0, b = 0, cp = 0, valid = 0, path = 0, small = 0, total = 0;
    size_t eval_bytes = 0;
    int plan_chunk = 0;      // plan that evaluates a chunk of candidates
    bool cp_only = false;    // ... without a b array
    int tick = 4;
};

int search_layout(const cp_graph *g, int32_t k, int32_t chunk, const int64_t *speeds, const int64_t *bandwidth,
                  SearchLayout &o) {
    cp_graph_info info;
    int rc = cp_graph_get_info(g, &info);
    if (rc) return rc;
    o.tick = info.min_tick_bytes;
    // the plan is not known without the cost model: size for the costlier case (wave-column keeps b)
    o.plan_chunk = CP_PLAN_WAVE_COLUMN;
    if (speeds && bandwidth) {
        rc = cp_eval_choose_plan(g, chunk, k, speeds, bandwidth, o.tick, &o.plan_chunk);
        if (rc) return rc;
    }
    size_t ws_chunk = 0, ws_one = 0;
    rc = cp_eval_workspace_bytes(g, chunk, k, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO, CP_OUT_VERTEX_MAJOR, o.tick,
                                 &ws_chunk);
    if (rc) return rc;
    rc = cp_eval_workspace_bytes(g, 1, k, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO, CP_OUT_VERTEX_MAJOR, o.tick,
                                 &ws_one);
    if (rc) return rc;
    const size_t n = (size_t)info.n;
    o.eval_bytes = align_up(std::max(ws_chunk, ws_one));
    // CP alone needs no b array only under the resident-window plan on a graph without far reads
    o.cp_only = o.plan_chunk != CP_PLAN_WAVE_COLUMN && info.window_far_b == 0;
    const size_t b_cols = o.cp_only ? 1 : (size_t)chunk;
    size_t at = 0;
    o.eval_ws = at; at += o.eval_bytes;
    o.cand = at;    at += align_up((size_t)chunk * n);
    o.b = at;       at += align_up(n * b_cols * (size_t)o.tick);
    o.cp = at;      at += align_up((size_t)chunk * sizeof(int64_t));
    o.valid = at;   at += align_up((size_t)chunk);
    o.path = at;    at += align_up((size_t)info.L * sizeof(int32_t));
    o.small = at;   at += kAlign;        // best (16 B), path length, status, cp of the base, move
    o.total = at;
    return CP_OK;
}

int copy_back(void *host, const void *dev, size_t bytes, hipStream_t st) {
    if (hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, st) != hipSuccess) return CP_ERR_HIP;
    return hipStreamSynchronize(st) == hipSuccess ? CP_OK : CP_ERR_HIP;
}

}  // namespace

}  // namespace cpeval

using namespace cpeval;

extern "C" {

int cp_search_workspace_bytes(const cp_graph *g, int32_t k, int32_t chunk, size_t *out_bytes) {
    if (!g || !out_bytes) return CP_ERR_NULL;
    if (k < 1 || k > 255 || chunk < 1) return CP_ERR_SIZE;
    SearchLayout lay;
    int rc = search_layout(g, k, chunk, nullptr, nullptr, lay);
    if (rc) return rc;
    *out_bytes = lay.total;
    return CP_OK;
}

int cp_search(const cp_graph *g, int32_t k, const int64_t *speeds, const int64_t *bandwidth,
              uint8_t *assignment, int64_t num_pairs, const int32_t *pairs, int64_t num_pins,
              const int32_t *pins, int32_t max_moves, int32_t chunk, void *workspace, size_t workspace_bytes,
              void *stream, int64_t *cp_trace, int32_t *moves, int32_t *num_moves, int64_t *evaluated) {
    if (!g || !speeds || !bandwidth || !assignment || !workspace || !cp_trace || !num_moves) return CP_ERR_NULL;
    if (k < 1 || k > 255 || chunk < 1 || max_moves < 0 || num_pairs < 0 || num_pins < 0) return CP_ERR_SIZE;
    if ((num_pairs > 0 && !pairs) || (num_pins > 0 && !pins)) return CP_ERR_NULL;
    SearchLayout lay;
    int rc = search_layout(g, k, chunk, speeds, bandwidth, lay);
    if (rc) return rc;
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < lay.total) return CP_ERR_WORKSPACE;
    cp_graph_info info;
    rc = cp_graph_get_info(g, &info);
    if (rc) return rc;
    if (!info.uploaded) return CP_ERR_STATE;
    const int32_t n = info.n, L = info.L;
    hipStream_t st = (hipStream_t)stream;
    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *d_cand = ws + lay.cand;
    void *d_b = ws + lay.b;
    int64_t *d_cp = (int64_t *)(ws + lay.cp);
    uint8_t *d_valid = ws + lay.valid;
    int32_t *d_path = (int32_t *)(ws + lay.path);
    Best *d_best = (Best *)(ws + lay.small);
    int32_t *d_len = (int32_t *)(ws + lay.small + 16);
    int32_t *d_status = (int32_t *)(ws + lay.small + 24);
    int64_t *d_cp_base = (int64_t *)(ws + lay.small + 32);
    int32_t *d_move = (int32_t *)(ws + lay.small + 40);
    const bool constrained = num_pairs > 0 || num_pins > 0;
    const bool vector_ok = n % 16 == 0 && ((uintptr_t)assignment % 16) == 0;     // candidate rows start at j * n
    int32_t done = 0;
    int64_t seen = 0;
    *num_moves = 0;
    for (;;) {
        // the current partition: CP, b, one critical path
        rc = cp_eval(g, 1, k, assignment, CP_ASSIGN_PARTITION_MAJOR, speeds, bandwidth, ws + lay.eval_ws,
                     lay.eval_bytes, stream, d_cp_base, d_b, nullptr, nullptr, lay.tick, CP_OUT_VERTEX_MAJOR,
                     CP_PLAN_AUTO, d_status, nullptr);
        if (rc) return rc;
        rc = cp_critical_path(g, 1, k, assignment, CP_ASSIGN_PARTITION_MAJOR, speeds, bandwidth, d_b, d_cp_base,
                              lay.tick, CP_OUT_VERTEX_MAJOR, ws + lay.eval_ws, lay.eval_bytes, stream, L, d_path,
                              d_len, d_status + 1);
        if (rc) return rc;
        struct { int32_t len; int32_t pad; int32_t status[2]; int64_t cp; } head;
        rc = copy_back(&head, d_len, sizeof(head), st);
        if (rc) return rc;
        if (head.status[0] != CP_STATUS_OK || head.status[1] != CP_STATUS_OK) return CP_ERR_ARG;   // bad device id
        cp_trace[done] = head.cp;
        if (done >= max_moves || k < 2) break;
        const int64_t total = (int64_t)head.len * (k - 1);
        hipLaunchKernelGGL(best_reset_kernel, dim3(1), dim3(1), 0, st, d_best);
        for (int64_t first = 0; first < total; first += chunk) {
            const int32_t count = (int32_t)std::min<int64_t>(chunk, total - first);
            const dim3 grid((unsigned)(((int64_t)n + 16 * 256 - 1) / (16 * 256)), (unsigned)std::min(count, 65535));
            hipLaunchKernelGGL(neighbours_kernel, grid, dim3(256), 0, st, (const uint8_t *)assignment,
                               (const int32_t *)d_path, n, k, (int32_t)first, count, d_cand, vector_ok ? 1 : 0);
            if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
            int plan = CP_PLAN_AUTO;
            rc = cp_eval_choose_plan(g, count, k, speeds, bandwidth, lay.tick, &plan);
            if (rc) return rc;
            // a short last chunk may resolve to the other plan: it needs b only if room was made for it
            void *b_arg = lay.cp_only ? nullptr : d_b;
            if (lay.cp_only && plan == CP_PLAN_WAVE_COLUMN) {
                if (count > 1) plan = CP_PLAN_RESIDENT_WINDOW;
                else b_arg = d_b;
            }
            rc = cp_eval(g, count, k, d_cand, CP_ASSIGN_PARTITION_MAJOR, speeds, bandwidth, ws + lay.eval_ws,
                         lay.eval_bytes, stream, d_cp, b_arg, nullptr, nullptr, lay.tick, CP_OUT_VERTEX_MAJOR, plan,
                         d_status, nullptr);
            if (rc) return rc;
            if (constrained) {
                rc = cp_validate(n, count, k, d_cand, CP_ASSIGN_PARTITION_MAJOR, num_pairs, pairs, num_pins, pins,
                                 stream, d_valid, nullptr, d_status + 1);
                if (rc) return rc;
            }
            hipLaunchKernelGGL(argmin_merge_kernel, dim3(1), dim3(1024), 0, st, (const int64_t *)d_cp,
                               constrained ? (const uint8_t *)d_valid : nullptr, count, (int32_t)first, d_best);
            if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
            seen += count;
        }
        Best best;
        rc = copy_back(&best, d_best, sizeof(best), st);
        if (rc) return rc;
        if (best.index < 0 || best.value >= head.cp) break;
        hipLaunchKernelGGL(apply_move_kernel, dim3(1), dim3(1), 0, st, assignment, (const int32_t *)d_path, k,
                           (const Best *)d_best, d_move);
        if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
        if (moves) {
            rc = copy_back(moves + 2 * done, d_move, 2 * sizeof(int32_t), st);
            if (rc) return rc;
        }
        ++done;
    }
    *num_moves = done;
    if (evaluated) *evaluated = seen;
    return hipStreamSynchronize(st) == hipSuccess ? CP_OK : CP_ERR_HIP;
}

int cp_seed_workspace_bytes(const cp_graph *g, size_t *out_bytes) {
    if (!g || !out_bytes) return CP_ERR_NULL;
    cp_graph_info info;
    int rc = cp_graph_get_info(g, &info);
    if (rc) return rc;
    size_t eval = 0;
    rc = cp_eval_workspace_bytes(g, 1, 1, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO, CP_OUT_VERTEX_MAJOR,
                                 info.min_tick_bytes, &eval);
    if (rc) return rc;
    *out_bytes = align_up(eval) + align_up((size_t)info.n) + align_up((size_t)info.n * (size_t)info.min_tick_bytes) +
                 align_up((size_t)info.L * sizeof(int32_t)) + kAlign;
    return CP_OK;
}

int cp_seed_partition(const cp_graph *g, int32_t k, const int64_t *speeds, void *workspace, size_t workspace_bytes,
                      void *stream, uint8_t *assignment_out, int32_t *status_out) {
    if (!g || !speeds || !workspace || !assignment_out || !status_out) return CP_ERR_NULL;
    if (k < 1 || k > kSeedMaxK) return CP_ERR_SIZE;
    size_t need = 0;
    int rc = cp_seed_workspace_bytes(g, &need);
    if (rc) return rc;
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < need) return CP_ERR_WORKSPACE;
    cp_graph_info info;
    rc = cp_graph_get_info(g, &info);
    if (rc) return rc;
    if (!info.uploaded) return CP_ERR_STATE;
    const Packed &p = g->packed;
    std::vector<int64_t> ones((size_t)k * k, 1);
    CostTables tabs;
    try {
        rc = build_cost_tables(k, speeds, ones.data(), p.narrow, p.info.max_c, p.info.max_t, tabs);
    } catch (const std::bad_alloc &) {
        rc = CP_ERR_ALLOC;
    }
    if (rc) return rc;
    size_t eval = 0;
    rc = cp_eval_workspace_bytes(g, 1, 1, CP_ASSIGN_PARTITION_MAJOR, CP_PLAN_AUTO, CP_OUT_VERTEX_MAJOR,
                                 info.min_tick_bytes, &eval);
    if (rc) return rc;
    const size_t n = (size_t)info.n;
    const int T = info.min_tick_bytes;
    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *d_one = ws + align_up(eval);
    void *d_b = d_one + align_up(n);
    int32_t *d_path = (int32_t *)((uint8_t *)d_b + align_up(n * (size_t)T));
    uint8_t *d_small = (uint8_t *)d_path + align_up((size_t)info.L * sizeof(int32_t));
    int64_t *d_cp = (int64_t *)d_small;
    int32_t *d_len = (int32_t *)(d_small + 8);
    hipStream_t st = (hipStream_t)stream;
    // the ranks know no devices: one device of speed 1, nothing is transferred
    rc = launch_zero_bytes(d_one, (int64_t)n, stream);
    if (rc) return rc;
    const int64_t unit = 1;
    rc = cp_eval(g, 1, 1, d_one, CP_ASSIGN_PARTITION_MAJOR, &unit, &unit, ws, align_up(eval), stream, d_cp, d_b,
                 nullptr, nullptr, T, CP_OUT_VERTEX_MAJOR, CP_PLAN_AUTO, status_out, nullptr);
    if (rc) return rc;
    rc = cp_critical_path(g, 1, 1, d_one, CP_ASSIGN_PARTITION_MAJOR, &unit, &unit, d_b, d_cp, T,
                          CP_OUT_VERTEX_MAJOR, ws, align_up(eval), stream, info.L, d_path, d_len, status_out);
    if (rc) return rc;
    SeedArgs a{};
    a.c = (const uint8_t *)g->device_blob + p.c_off;
    a.path = d_path;
    a.len = d_len;
    a.assign = assignment_out;
    a.n = info.n;
    a.k = k;
    a.fastest = 0;
    for (int d = 1; d < k; ++d)
        if (speeds[d] > speeds[a.fastest]) a.fastest = d;
    a.magic = tabs.magic_ok ? 1 : 0;
    for (int d = 0; d < k; ++d) {
        a.mg[d] = tabs.magic[2 * (size_t)k * k + d];
        a.speed[d] = speeds[d];
    }
    hipLaunchKernelGGL(seed_mark_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(seed_path_kernel, dim3(64), dim3(256), 0, st, a);
    if (p.narrow) hipLaunchKernelGGL(seed_greedy_kernel<uint32_t>, dim3(1), dim3(64), 0, st, a);
    else hipLaunchKernelGGL(seed_greedy_kernel<int64_t>, dim3(1), dim3(64), 0, st, a);
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
}

}  // extern "C"
