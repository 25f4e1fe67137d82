// List-scheduling simulation of one iteration for a batch of partitions: the paper's
// scheduling criteria (section 4, (1)-(6)) with its PCT rule (section 4.1) or the FIFO
// baseline (section 5.1), on the cost model of section 2 in integer ticks.  The result is
// the start time of every vertex and the makespan, the quantity the paper's evaluation
// plots (section 5).
//
// One wavefront simulates one partition, lane d being device d; with 32 devices or fewer it
// simulates 64 / k partitions side by side, k lanes each.  A device keeps the vertices
// whose predecessors have all started -- their ready time is final by then -- in a
// min-heap keyed by ready time ("pending"); under PCT the ones that are executable at the
// device's decision time move on to a second heap keyed by descending b ("available").
// Devices only interact through tensors that arrive: a vertex that starts at time T on
// one device reaches another device no earlier than T + (shortest execution time) +
// (shortest transfer time).  So with T_min the earliest decision time over all devices,
// every device whose decision time lies less than that sum after T_min already knows all
// it needs, and those lanes decide in the same step.  A lane that starts a vertex lowers
// the open-input count of each successor and raises its ready time; the lane that takes
// the last open input hands the successor to its owner's inbox, which the owner drains at
// the top of its next step.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "cpeval_internal.hpp"
#include "device_math.hpp"
#include "launch.hpp"

namespace cpeval {

namespace {

constexpr uint32_t kNever = 0xffffffffu;
constexpr int kWideRow = 32;      // out-edges from which a started vertex's row is shared out over the wavefront

// All lanes of a partition sit in one wavefront, so everything they exchange passes through
// one compute unit's vector L1 and one L2; no fence wider than the workgroup is ever needed (a
// release at device scope would write the L2 back on every step).  Ready times and open-input
// counts are only changed by read-modify-write atomics, which execute in the L2 and leave the
// L1 stale: a ready time is read back with a load of device scope, which goes past the L1.
// Inbox slots are written once with ordinary stores and read afterwards by another lane of
// the wavefront.
__device__ __forceinline__ int32_t l2_read(int32_t *p) {
    // a device-scope load goes past the L1 like the atomics do, and unlike an atomic it writes nothing
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t inbox_load(const int32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}
__device__ __forceinline__ void inbox_store(int32_t *p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}
// Every memory operation of the wavefront issued so far has completed.
__device__ __forceinline__ void step_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
}

// Four-ary min-heaps of 64-bit keys (children of i: 4i+1 .. 4i+4): half the levels of a binary
// heap, and the four children of a node are loaded together.  A lane's heap is touched by that
// lane only.  A heap never holds more keys than its device has vertices, so 16 levels bound
// every loop.
__device__ __forceinline__ void heap_push(uint64_t *h, int32_t &size, uint64_t key) {
    int32_t i = size++;
    for (int depth = 0; depth < 16 && i > 0; ++depth) {
        const int32_t up = (i - 1) >> 2;
        const uint64_t uk = h[up];
        if (uk <= key) break;
        h[i] = uk;
        i = up;
    }
    h[i] = key;
}

__device__ __forceinline__ uint64_t heap_pop(uint64_t *h, int32_t &size) {
    const uint64_t top = h[0];
    const int32_t left = --size;
    if (left > 0) {
        const uint64_t last = h[left];
        int32_t i = 0;
        for (int depth = 0; depth < 16; ++depth) {
            const int32_t c0 = 4 * i + 1;
            if (c0 >= left) break;
            uint64_t ck[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) ck[j] = h[min(c0 + j, left - 1)];     // in range; masked below
            uint64_t best = ck[0];
            int32_t at = c0;
#pragma unroll
            for (int j = 1; j < 4; ++j) {
                if (c0 + j < left && ck[j] < best) {
                    best = ck[j];
                    at = c0 + j;
                }
            }
            if (last <= best) break;
            h[i] = best;
            i = at;
        }
        h[i] = last;
    }
    return top;
}

// A queue = its smallest key in a register + the heap above in memory for the rest.  Device
// queues are short most of the time (a handful of executable vertices), so most pushes and
// pops never touch memory, and the decision time is read from the register.
struct Queue {
    uint64_t top = 0;
    int32_t size = 0;          // keys held, the one in the register included
};

__device__ __forceinline__ void queue_push(uint64_t *h, Queue &q, uint64_t key) {
    if (q.size == 0) {
        q.top = key;
    } else {
        const uint64_t keep = min(q.top, key), spill = max(q.top, key);
        q.top = keep;
        int32_t in_memory = q.size - 1;
        heap_push(h, in_memory, spill);
    }
    ++q.size;
}

// Taking the smallest key and bringing the next one into the register are two calls, so that
// the caller can start the loads that depend on the key before the heap in memory is put in
// order again.  Nothing else may touch the queue in between.
__device__ __forceinline__ uint64_t queue_take(Queue &q) {
    --q.size;
    return q.top;
}

__device__ __forceinline__ void queue_refill(uint64_t *h, Queue &q) {
    if (q.size > 0) {
        int32_t in_memory = q.size;
        q.top = heap_pop(h, in_memory);
    }
}

__device__ __forceinline__ uint64_t queue_pop(uint64_t *h, Queue &q) {
    const uint64_t out = queue_take(q);
    queue_refill(h, q);
    return out;
}

// b(z) of the lane's partition; a value outside [0, 2^31) is reported and replaced by 0.
__device__ __forceinline__ long long load_b(const uint8_t *bq, int32_t z, int64_t bsv, int32_t b_bytes, bool &bad) {
    long long bz = b_bytes == 4 ? (long long)*(const int32_t *)(bq + (int64_t)z * bsv * 4)
                                : *(const long long *)(bq + (int64_t)z * bsv * 8);
    if (bz < 0 || bz > 0x7fffffffll) { bad = true; bz = 0; }
    return bz;
}

struct SimArgs {
    const int32_t *ptr;        // successor CSR over original ids
    const int32_t *idx;
    const void *wt;            // t(e) in that order
    const void *c;
    const int32_t *pred_ptr;   // predecessor CSR row bounds: the in-degrees
    const uint8_t *assign;
    int64_t a_stride_p, a_stride_v;
    const void *b;             // PCT: ticks, b(v, q) at v * b_sv + q * b_sq
    int64_t b_sv, b_sq;
    int32_t b_bytes;
    const int32_t *tie;        // FIFO: rank of a vertex among equal ready times, null = its number
    const int32_t *tie_inv;    //       vertex of a rank
    const void *edge_tab;      // row = device of the edge's source vertex
    const void *vert_tab;
    int32_t *ready;            // [P][n] latest arrival so far
    int32_t *need;             // [P][n] inputs whose producer has not started
    int32_t *inbox;            // [P][n], one segment per device
    uint64_t *pending;         // [P][n], one segment per device
    uint64_t *available;       // [P][n], PCT only
    long long *makespan;       // [P]
    int32_t *start;            // [P][n] or null
    int32_t *status;
    int32_t n, P, k;
    int32_t groups;            // partitions per wavefront, <= 64 / k
    uint32_t window;           // lanes with T - T_min <= window decide together
};

template <typename WT, bool MAGIC, bool PCT>
__global__ __launch_bounds__(64) void simulate_kernel(SimArgs a) {
    __shared__ int32_t count[64];      // vertices per device, then vertices handed to the device so far
    __shared__ int32_t seg[64];        // first slot of the device's segment
    __shared__ int32_t gbad[64];       // per group: a device id >= k was seen
    const int lane = threadIdx.x;
    const int32_t n = a.n, k = a.k;
    // with k <= 32 devices a wavefront can hold up to 64 / k partitions side by side: group g =
    // lanes g*k .. g*k + k-1.  Lanes past the last group, and groups past the batch, idle.
    const int groups = a.groups;
    const int grp = lane / k, dev = lane - grp * k;
    const int first = grp * k;
    const int64_t q = (int64_t)blockIdx.x * groups + grp;
    bool alive = grp < groups && q < a.P;
    const int64_t qq = alive ? q : 0;          // idle lanes never load or store, but keep their pointers in range
    const uint8_t *row = a.assign + qq * a.a_stride_p;
    const int64_t asv = a.a_stride_v;
    const WT *wt = (const WT *)a.wt;
    const WT *cw = (const WT *)a.c;
    const Magic *etab_m = (const Magic *)a.edge_tab, *vtab_m = (const Magic *)a.vert_tab;
    const int64_t *etab_g = (const int64_t *)a.edge_tab, *vtab_g = (const int64_t *)a.vert_tab;
    int32_t *ready = a.ready + qq * n;
    int32_t *need = a.need + qq * n;
    int32_t *start = a.start ? a.start + qq * n : nullptr;

    if (*a.status & CP_STATUS_BAD_TIE) {          // set by the check of the tie ranks, same stream
        if (alive && dev == 0) a.makespan[q] = -1;
        return;
    }

    // ---- set-up: vertices per device, state of every vertex
    count[lane] = 0;
    gbad[lane] = 0;
    __syncthreads();
    if (alive) {
        for (int32_t v = dev; v < n; v += k) {
            const uint32_t d = row[(int64_t)v * asv];
            if (d >= (uint32_t)k) { gbad[grp] = 1; continue; }
            atomicAdd(&count[first + d], 1);
            ready[v] = 0;
            need[v] = a.pred_ptr[v + 1] - a.pred_ptr[v];
        }
    }
    __syncthreads();
    if (alive && gbad[grp]) {
        alive = false;
        if (dev == 0) {
            atomicOr(a.status, CP_STATUS_BAD_DEVICE_ID);
            a.makespan[q] = -1;
        }
    }
    {
        const int32_t mine = alive ? count[lane] : 0;
        int32_t incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t other = __shfl_up(incl, off);
            if (lane >= off) incl += other;
        }
        const int32_t below = __shfl(incl, first > 0 ? first - 1 : 0);   // total of the groups before this one
        __syncthreads();
        seg[lane] = incl - mine - (first > 0 ? below : 0);
        count[lane] = 0;
    }
    step_fence();
    int32_t *inbox = a.inbox + qq * n;
    if (alive) {
        for (int32_t v = dev; v < n; v += k) {
            if (a.pred_ptr[v + 1] == a.pred_ptr[v]) {
                const uint32_t d = row[(int64_t)v * asv];
                const int32_t pos = atomicAdd(&count[first + d], 1);
                inbox_store(inbox + seg[first + d] + pos, v);
            }
        }
    }
    step_fence();

    // ---- the event loop
    const int32_t base = seg[lane];
    uint64_t *hp = a.pending + qq * n + base;
    uint64_t *ha = PCT ? a.available + qq * n + base : nullptr;
    const int32_t *my_inbox = inbox + base;
    const int64_t bsv = a.b_sv;
    const uint8_t *bq = (const uint8_t *)a.b + (PCT ? qq * a.b_sq * a.b_bytes : 0);
    const int last_lane = min(first + k - 1, 63);
    Queue pending, available;
    int32_t taken = 0, done = 0;
    uint32_t free_at = 0;
    bool b_bad = false;
    // every step with work left starts at least one vertex in every unfinished group, so
    // n + 1 steps always suffice
    for (int64_t step = 0; step <= n; ++step) {
        if (alive) {   // vertices handed to this device since its last step, four loads in flight at a time
            const int32_t have = count[lane];
            while (taken < have) {
                const int32_t cnt = min(4, have - taken);
                int32_t z[4];
                uint32_t rz[4], low[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) z[j] = inbox_load(my_inbox + taken + min(j, cnt - 1));
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    rz[j] = (uint32_t)l2_read(ready + z[j]);
                    low[j] = PCT ? (uint32_t)z[j] : (a.tie ? (uint32_t)a.tie[z[j]] : (uint32_t)z[j]);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (j < cnt) {
                        if (PCT && rz[j] <= free_at) {
                            // executable at every decision this device has still to take
                            const long long bz = load_b(bq, z[j], bsv, a.b_bytes, b_bad);
                            queue_push(ha, available, ((uint64_t)(0x7fffffffu - (uint32_t)bz) << 32) | (uint32_t)z[j]);
                        } else {
                            queue_push(hp, pending, ((uint64_t)rz[j] << 32) | low[j]);
                        }
                    }
                }
                taken += cnt;
            }
        }
        uint32_t T = kNever;
        if (PCT && available.size > 0) T = free_at;
        else if (pending.size > 0) T = max(free_at, (uint32_t)(pending.top >> 32));
        // the group's earliest decision time (several groups: a running minimum over each
        // group's lanes, read from its last lane)
        uint32_t tmin = T;
        if (groups == 1) {
            // one partition in the wavefront: the minimum of each row of 16 lanes by register
            // permutations, then the four rows' minima through scalar registers
            tmin = min(tmin, dpp_u32<0xB1>(tmin));      // swap neighbours
            tmin = min(tmin, dpp_u32<0x4E>(tmin));      // swap pairs
            tmin = min(tmin, dpp_u32<0x141>(tmin));     // mirror halves of 8
            tmin = min(tmin, dpp_u32<0x140>(tmin));     // mirror the row
            tmin = min(min((uint32_t)__builtin_amdgcn_readlane((int)tmin, 0),
                           (uint32_t)__builtin_amdgcn_readlane((int)tmin, 16)),
                       min((uint32_t)__builtin_amdgcn_readlane((int)tmin, 32),
                           (uint32_t)__builtin_amdgcn_readlane((int)tmin, 48)));
        } else {
            for (int off = 1; off < k; off <<= 1) {
                const uint32_t other = (uint32_t)__shfl_up((int)tmin, off);
                if (dev >= off) tmin = min(tmin, other);
            }
            tmin = (uint32_t)__shfl((int)tmin, last_lane);
        }
        if (__all(tmin == kNever)) break;
        int32_t wide_e0 = 0, wide_e1 = 0;     // a long row is left to the whole wavefront below
        if (T != kNever && T - tmin <= a.window) {
            int32_t v;
            if (PCT) {
                for (int32_t moved = 0; pending.size > 0 && (uint32_t)(pending.top >> 32) <= T && moved < n;
                     ++moved) {
                    const int32_t z = (int32_t)(uint32_t)queue_pop(hp, pending);
                    const long long bz = load_b(bq, z, bsv, a.b_bytes, b_bad);
                    queue_push(ha, available, ((uint64_t)(0x7fffffffu - (uint32_t)bz) << 32) | (uint32_t)z);
                }
                v = (int32_t)(uint32_t)queue_take(available);
            } else {
                const uint32_t low = (uint32_t)queue_take(pending);
                v = a.tie_inv ? a.tie_inv[low] : (int32_t)low;
            }
            // what the vertex needs from the graph is on its way while the queue is put in order
            const WT cv = cw[v];
            const int32_t e0 = a.ptr[v], e1 = a.ptr[v + 1];
            if (PCT) queue_refill(ha, available);
            else queue_refill(hp, pending);
            if (start) start[v] = (int32_t)T;
            ++done;
            const uint32_t w = MAGIC ? magic_div((uint32_t)cv, vtab_m[dev])
                                     : (uint32_t)plain_div((uint64_t)cv, (uint64_t)vtab_g[dev]);
            free_at = T + w;
            // the out-edges four at a time, so that the dependent loads of four edges (successor,
            // its device, the table entry) and their atomics overlap; slots past the row's end
            // repeat its last edge for the loads and take no part in the atomics
            int32_t e_end = e1;
            if (e1 - e0 >= kWideRow) {
                wide_e0 = e0;
                wide_e1 = e1;
                e_end = e0;
            }
            for (int32_t e = e0; e < e_end; e += 4) {
                const int32_t cnt = min(4, e_end - e);
                int32_t z[4], before[4];
                WT te[4];
                uint32_t dz[4], arrive[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t ej = e + min(j, cnt - 1);
                    z[j] = a.idx[ej];
                    te[j] = wt[ej];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) dz[j] = row[(int64_t)z[j] * asv];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t x = MAGIC ? magic_div((uint32_t)te[j], etab_m[dev * k + dz[j]])
                                             : (uint32_t)plain_div((uint64_t)te[j],
                                                                       (uint64_t)etab_g[dev * k + dz[j]]);
                    arrive[j] = free_at + x;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (j < cnt)
                        __hip_atomic_fetch_max(ready + z[j], (int32_t)arrive[j], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    before[j] = 0;
                    if (j < cnt)
                        before[j] = __hip_atomic_fetch_add(need + z[j], -1, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (before[j] == 1) {
                        const int32_t pos = atomicAdd(&count[first + dz[j]], 1);
                        inbox_store(inbox + seg[first + dz[j]] + pos, z[j]);
                    }
                }
            }
        }
        // long rows (hubs), one after the other, 64 edges at a time: every lane of the wavefront,
        // whatever its own partition, works for the lane that started the hub
        for (unsigned long long wide = __ballot(wide_e1 > wide_e0); wide; wide &= wide - 1) {
            const int src = __ffsll((long long)wide) - 1;
            const int32_t he0 = __shfl(wide_e0, src), he1 = __shfl(wide_e1, src);
            const uint32_t hfree = (uint32_t)__shfl((int)free_at, src);
            const int hdev = __shfl(dev, src), hfirst = __shfl(first, src);
            const int64_t hq = ((int64_t)__shfl((int)(qq >> 32), src) << 32) | (uint32_t)__shfl((int)(uint32_t)qq, src);
            const uint8_t *hrow = a.assign + hq * a.a_stride_p;
            int32_t *hready = a.ready + hq * n, *hneed = a.need + hq * n, *hinbox = a.inbox + hq * n;
            for (int32_t e = he0 + lane; e < he1; e += 64) {
                const int32_t z = a.idx[e];
                const WT te = wt[e];
                const uint32_t dz = hrow[(int64_t)z * asv];
                const uint32_t x = MAGIC ? magic_div((uint32_t)te, etab_m[hdev * k + dz])
                                         : (uint32_t)plain_div((uint64_t)te, (uint64_t)etab_g[hdev * k + dz]);
                __hip_atomic_fetch_max(hready + z, (int32_t)(hfree + x), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                const int32_t before = __hip_atomic_fetch_add(hneed + z, -1, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_WORKGROUP);
                if (before == 1) {
                    const int32_t pos = atomicAdd(&count[hfirst + dz], 1);
                    inbox_store(hinbox + seg[hfirst + dz] + pos, z);
                }
            }
        }
        step_fence();     // everything this step wrote is in place before the next step reads it
    }
    uint32_t last = free_at;
    int32_t total = done;
    for (int off = 1; off < k; off <<= 1) {
        const uint32_t o1 = (uint32_t)__shfl_up((int)last, off);
        const int32_t o2 = __shfl_up(total, off);
        if (dev >= off) {
            last = max(last, o1);
            total += o2;
        }
    }
    if (__any(b_bad) && lane == 0) atomicOr(a.status, CP_STATUS_B_OUT_OF_RANGE);
    if (alive && dev == k - 1) {
        if (total != n) {
            atomicOr(a.status, CP_STATUS_INCOMPLETE);
            a.makespan[q] = -1;
        } else {
            a.makespan[q] = (long long)last;
        }
    }
}

// tie_inv[tie[v]] = v; a rank outside [0, n) is reported.  tie_inv starts at -1.
__global__ __launch_bounds__(256) void tie_scatter_kernel(const int32_t *tie, int32_t n, int32_t *tie_inv,
                                                          int32_t *status) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n) return;
    const int32_t r = tie[v];
    if (r < 0 || r >= n) atomicOr(status, CP_STATUS_BAD_TIE);
    else tie_inv[r] = (int32_t)v;
}

// A rank nobody has means another rank was given twice: not a permutation.
__global__ __launch_bounds__(256) void tie_check_kernel(const int32_t *tie_inv, int32_t n, int32_t *status) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r < n && tie_inv[r] < 0) atomicOr(status, CP_STATUS_BAD_TIE);
}

__global__ __launch_bounds__(256) void fill_minus_one_kernel(int32_t *dst, int32_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = -1;
}

}  // namespace

int launch_simulate(const SimulateLaunch &s, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (s.n < 1 || s.P < 1 || s.k < 1 || s.k > kWave) return CP_ERR_SIZE;
    if (s.tie) {
        const dim3 grid((unsigned)((s.n + 255) / 256)), block(256);
        hipLaunchKernelGGL(fill_minus_one_kernel, grid, block, 0, st, s.tie_inv, s.n);
        hipLaunchKernelGGL(tie_scatter_kernel, grid, block, 0, st, s.tie, s.n, s.tie_inv, s.status);
        hipLaunchKernelGGL(tie_check_kernel, grid, block, 0, st, s.tie_inv, s.n, s.status);
    }
    SimArgs a{};
    a.ptr = (const int32_t *)(s.blob + s.succ->ptr_off);
    a.idx = (const int32_t *)(s.blob + s.succ->idx_off);
    a.wt = s.blob + s.succ->wt_off;
    a.c = s.blob + s.c_off;
    a.pred_ptr = (const int32_t *)(s.blob + s.pred->ptr_off);
    a.assign = s.assign;
    a.a_stride_p = s.a_stride_p;
    a.a_stride_v = s.a_stride_v;
    a.b = s.b;
    a.b_sv = s.b_sv;
    a.b_sq = s.b_sq;
    a.b_bytes = s.b_bytes;
    a.tie = s.tie;
    a.tie_inv = s.tie ? s.tie_inv : nullptr;
    a.edge_tab = s.edge_tab;
    a.vert_tab = s.vert_tab;
    a.ready = s.ready;
    a.need = s.need;
    a.inbox = s.inbox;
    a.pending = s.pending;
    a.available = s.available;
    a.makespan = (long long *)s.makespan;
    a.start = s.start;
    a.status = s.status;
    a.n = s.n; a.P = s.P; a.k = s.k;
    a.window = s.window;
    const int groups = std::max(1, std::min(s.groups, kWave / s.k));      // partitions per wavefront
    a.groups = groups;
    const dim3 grid((unsigned)((s.P + groups - 1) / groups)), block(64);
#define CP_SIM(WT, MAGIC)                                                                      \
    do {                                                                                       \
        if (s.pct) hipLaunchKernelGGL((simulate_kernel<WT, MAGIC, true>), grid, block, 0, st, a);  \
        else hipLaunchKernelGGL((simulate_kernel<WT, MAGIC, false>), grid, block, 0, st, a);       \
    } while (0)
    if (s.magic) CP_SIM(uint32_t, true);
    else if (s.narrow) CP_SIM(uint32_t, false);
    else CP_SIM(int64_t, false);
#undef CP_SIM
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
}

}  // namespace cpeval
