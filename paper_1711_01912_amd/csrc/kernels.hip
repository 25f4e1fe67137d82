// HIP kernels for gfx950 and their launchers.
//
// Two kernel families evaluate the same recurrences (b-level: the PCT equation of
// section 4.1; t-level: the downward rank of section 3.2 without the own term):
//
//  * wave-column: distances live in HBM as [vertex][partition]; one wavefront
//    relaxes one vertex for 64 consecutive partitions, so every gather of a
//    neighbour is one contiguous 64-tick segment.  One launch per level; rows of
//    kHubDegree edges or more get a whole workgroup whose wavefronts split the
//    row and fold their maxima through LDS.
//
//  * resident-window: one workgroup owns one partition and walks all levels in a
//    single launch, lanes across the vertices of a level.  The distances and
//    device ids of the recent levels stay in an LDS ring, so the level-to-level
//    dependency never leaves the compute unit.
#include <hip/hip_runtime.h>

#include "launch.hpp"

namespace cpeval {
namespace {

// ---------------------------------------------------------------- cost policies

__device__ __forceinline__ uint32_t magic_div(uint32_t a, Magic mg) {
    uint32_t nn = a + mg.dm1;
    return (uint32_t)(((uint64_t)nn * mg.mul + nn) >> 32);
}

__device__ __forceinline__ uint64_t plain_div(uint64_t a, uint64_t d) {
    return d ? (a + d - 1) / d : 0;
}

template <typename T>
__device__ __forceinline__ T wave_bcast(T v, int src_lane);

template <>
__device__ __forceinline__ int32_t wave_bcast<int32_t>(int32_t v, int src_lane) {
    return __builtin_amdgcn_readlane(v, src_lane);
}
template <>
__device__ __forceinline__ uint32_t wave_bcast<uint32_t>(uint32_t v, int src_lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, src_lane);
}
template <>
__device__ __forceinline__ int64_t wave_bcast<int64_t>(int64_t v, int src_lane) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, src_lane);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), src_lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// ---------------------------------------------------------------- small kernels

__global__ void clear_kernel(int64_t *cp_out, int32_t batch, int32_t *status) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (cp_out && i < batch) cp_out[i] = 0;
    if (i == 0) *status = CP_STATUS_OK;
}

// assignments[P][n] -> pT[n][P], 64 x 64 byte tiles through LDS
__global__ __launch_bounds__(256) void transpose_kernel(const uint8_t *__restrict__ in,
                                                        uint8_t *__restrict__ out, int32_t n,
                                                        int32_t P) {
    __shared__ uint8_t tile[64][65];
    const int64_t v0 = (int64_t)blockIdx.x * 64, p0 = (int64_t)blockIdx.y * 64;
    const int lane = threadIdx.x & 63, row0 = threadIdx.x >> 6;
    for (int r = row0; r < 64; r += 4) {
        int64_t p = p0 + r, v = v0 + lane;
        if (p < P && v < n) tile[r][lane] = in[p * n + v];
    }
    __syncthreads();
    for (int r = row0; r < 64; r += 4) {
        int64_t v = v0 + r, p = p0 + lane;
        if (v < n && p < P) out[v * P + p] = tile[lane][r];
    }
}

// ---------------------------------------------------------------- wave-column sweep

struct ColumnArgs {
    const int32_t *ptr;
    const int32_t *idx;
    const void *wt;
    const void *c;
    const int32_t *order;   // already offset to the first vertex of this launch
    const uint8_t *pT;      // [n][P]
    void *val;              // [n][P] ticks: b (b sweep) or tl (t sweep)
    const void *edge_tab;   // Magic[k*k] or int64[k*k] for this sweep
    const void *vert_tab;   // Magic[k] or int64[k]
    int32_t *status;
    int32_t P, ncol, k, count;
};

template <typename Tick, typename WT, bool MAGIC, bool TSWEEP, bool HUB>
__global__ __launch_bounds__(HUB ? kHubWaves * 64 : 256) void column_level_kernel(ColumnArgs a) {
    extern __shared__ uint64_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = a.k;
    const int ntab = MAGIC ? k * k + k : 0;
    if (MAGIC) {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
        for (int i = tid; i < k * k; i += blockDim.x) lds[i] = e[i];
        for (int i = tid; i < k; i += blockDim.x) lds[k * k + i] = v[i];
        __syncthreads();
    }
    const Magic *etab_m = (const Magic *)lds;
    const Magic *vtab_m = etab_m + k * k;
    const int64_t *etab_g = (const int64_t *)a.edge_tab;
    const int64_t *vtab_g = (const int64_t *)a.vert_tab;

    const int64_t task = HUB ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
    const int64_t ntasks = (int64_t)a.count * a.ncol;
    const bool task_live = task < ntasks;
    const int32_t vi = task_live ? (int32_t)(task / a.ncol) : 0;
    const int32_t col = task_live ? (int32_t)(task % a.ncol) : 0;
    const int32_t v = a.order[vi];
    const int32_t q = col * 64 + lane;
    const int32_t P = a.P;
    const bool live = task_live && q < P;
    const uint8_t *pT = a.pT + q;
    Tick *val = (Tick *)a.val + q;
    const WT *wt = (const WT *)a.wt;
    const WT *cw = (const WT *)a.c;

    uint32_t pv = 0;
    if (live) {
        pv = pT[(size_t)v * P];
        if (pv >= (uint32_t)k) { *a.status = CP_STATUS_BAD_DEVICE_ID; pv = 0; }
    }

    int32_t e0 = a.ptr[v], e1 = a.ptr[v + 1];
    if (HUB) {  // this wavefront's share of the row
        int32_t len = e1 - e0, chunk = (len + kHubWaves - 1) / kHubWaves;
        e0 = min(e1, e0 + wave * chunk);
        e1 = min(e1, e0 + chunk);
    }
    if (!task_live) e1 = e0;

    Tick acc = 0;
    for (int32_t base = e0; base < e1; base += 64) {
        const int32_t cnt = min(64, e1 - base);
        int32_t my_u = 0;
        WT my_t = 0;
        if (lane < cnt) { my_u = a.idx[base + lane]; my_t = wt[base + lane]; }
        for (int j = 0; j < cnt; ++j) {
            const int32_t u = wave_bcast<int32_t>(my_u, j);
            const WT te = wave_bcast<WT>(my_t, j);
            if (live) {
                uint32_t pu = pT[(size_t)u * P];
                pu = min(pu, (uint32_t)(k - 1));
                Tick vu = val[(size_t)u * P];
                if (TSWEEP) {   // neighbour is a predecessor: its finish time is tl(u) + w(u)
                    const WT cu = cw[u];
                    vu += MAGIC ? (Tick)magic_div((uint32_t)cu, vtab_m[pu])
                                : (Tick)plain_div((uint64_t)cu, (uint64_t)vtab_g[pu]);
                }
                const Tick x = MAGIC ? (Tick)magic_div((uint32_t)te, etab_m[pv * k + pu])
                                     : (Tick)plain_div((uint64_t)te, (uint64_t)etab_g[pv * k + pu]);
                acc = max(acc, (Tick)(vu + x));
            }
        }
    }

    if (HUB) {  // fold the wavefronts' maxima
        Tick *part = (Tick *)(lds + ntab);
        part[wave * 64 + lane] = acc;
        __syncthreads();
        if (wave != 0) return;
        for (int w2 = 1; w2 < kHubWaves; ++w2) acc = max(acc, part[w2 * 64 + lane]);
    }
    if (live) {
        const WT cv = cw[v];
        const Tick w = MAGIC ? (Tick)magic_div((uint32_t)cv, vtab_m[pv])
                             : (Tick)plain_div((uint64_t)cv, (uint64_t)vtab_g[pv]);
        val[(size_t)v * P] = TSWEEP ? acc : (Tick)(acc + w);
    }
}

// CP[q] = max over sources of b: b never decreases against the edge direction
// (b(u) >= b(v) for u -> v since all costs are >= 0), so the column maximum is
// attained at a vertex without predecessors.
template <typename Tick>
__global__ __launch_bounds__(256) void cp_sources_kernel(const int32_t *__restrict__ sources,
                                                         int32_t nsrc, const Tick *__restrict__ b,
                                                         int32_t P, int64_t *cp_out) {
    __shared__ long long part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int32_t q = blockIdx.x * 64 + lane;
    long long best = 0;
    if (q < P)
        for (int32_t i = blockIdx.y * 4 + wave; i < nsrc; i += gridDim.y * 4)
            best = max(best, (long long)b[(size_t)sources[i] * P + q]);
    part[wave][lane] = best;
    __syncthreads();
    if (wave == 0 && q < P) {
        best = max(max(part[0][lane], part[1][lane]), max(part[2][lane], part[3][lane]));
        atomicMax((long long *)cp_out + q, best);
    }
}

// mask[v][word] bit i = (tl + b == CP) for partition 64*word + i
template <typename Tick>
__global__ __launch_bounds__(256) void mask_kernel(const Tick *__restrict__ b,
                                                   const Tick *__restrict__ tl,
                                                   const int64_t *__restrict__ cp, int32_t n,
                                                   int32_t P, int32_t ncol, uint64_t *mask) {
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t ntasks = (int64_t)n * ncol;
    for (int64_t task = wave0; task < ntasks; task += nwaves) {
        const int64_t v = task / ncol;
        const int32_t col = (int32_t)(task % ncol);
        const int32_t q = col * 64 + lane;
        bool on = false;
        if (q < P) {
            const size_t at = (size_t)v * P + q;
            on = (int64_t)tl[at] + (int64_t)b[at] == cp[q];
        }
        const uint64_t word = __ballot(on);
        if (lane == 0) mask[task] = word;
    }
}

// ---------------------------------------------------------------- resident-window sweep

struct WindowArgs {
    const int32_t *vtx;        // [n] original id per position
    const uint32_t *c;         // [n]
    const int32_t *deg;        // [n]
    const int32_t *lvl;        // [L+1][2]
    const uint32_t *slice_off; // [slices+1]
    const uint2 *ent;          // {slot, t}
    const uint8_t *assign;     // [P][n] or [n][P]
    int64_t a_stride_p, a_stride_v;   // element strides of `assign`
    void *out;                 // [n][P] ticks, or NULL
    int64_t *cp_out;           // [P] or NULL: receives max of the values written to the ring
    const Magic *edge_tab;
    const Magic *vert_tab;
    int32_t *status;
    int32_t P, L, k, slots;
};

template <typename Tick, bool TSWEEP>
__global__ __launch_bounds__(kWindowMaxThreads) void window_sweep_kernel(WindowArgs a) {
    extern __shared__ uint64_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int k = a.k;
    Magic *etab = (Magic *)lds;
    Magic *vtab = etab + k * k;
    Tick *ring = (Tick *)(vtab + k);                    // 8-byte aligned: a table entry is 8 bytes
    uint8_t *pdev = (uint8_t *)(ring + a.slots);
    {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
        for (int i = tid; i < k * k; i += nt) lds[i] = e[i];
        for (int i = tid; i < k; i += nt) lds[k * k + i] = v[i];
    }
    __syncthreads();

    // partition of this workgroup; neighbours in a 128-byte output line share an XCD
    const int32_t q = blockIdx.x;
    const uint8_t *assign = a.assign + (int64_t)q * a.a_stride_p;
    Tick *out = a.out ? (Tick *)a.out + q : nullptr;
    const int32_t R = a.slots, P = a.P;
    long long best = 0;

    for (int32_t s = 0; s < a.L; ++s) {
        const int32_t pa = a.lvl[2 * s], sl0 = a.lvl[2 * s + 1], pb = a.lvl[2 * s + 2];
        for (int32_t i0 = pa; i0 < pb; i0 += nt) {
            const int32_t i = i0 + tid;
            if (i < pb) {
                const int32_t v = a.vtx[i];
                uint32_t pv = assign[(int64_t)v * a.a_stride_v];
                if (pv >= (uint32_t)k) { *a.status = CP_STATUS_BAD_DEVICE_ID; pv = 0; }
                const int32_t dg = a.deg[i];
                const uint32_t cv = a.c[i];
                const uint32_t slice = sl0 + ((i - pa) >> 6);
                const uint2 *ent = a.ent + a.slice_off[slice] + lane;
                Tick acc = 0;
                for (int32_t j = 0; j < dg; ++j) {
                    const uint2 en = ent[(size_t)j * 64];
                    const uint32_t pu = pdev[en.x];
                    const Tick vu = ring[en.x];
                    const Tick x = (Tick)magic_div(en.y, etab[pv * k + pu]);
                    acc = max(acc, (Tick)(vu + x));
                }
                const Tick w = (Tick)magic_div(cv, vtab[pv]);
                const Tick fin = acc + w;             // b(v), or tl(v) + w(v)
                const int32_t slot = i % R;
                ring[slot] = fin;
                pdev[slot] = (uint8_t)pv;
                if (out) out[(size_t)v * P] = TSWEEP ? acc : fin;
                best = max(best, (long long)fin);
            }
        }
        __syncthreads();
    }

    if (a.cp_out) {   // workgroup maximum of everything written
        __shared__ long long red[kWindowMaxThreads / 64];
        for (int off = 32; off > 0; off >>= 1) best = max(best, __shfl_xor(best, off));
        if (lane == 0) red[tid >> 6] = best;
        __syncthreads();
        if (tid == 0) {
            for (int w2 = 1; w2 < (nt + 63) / 64; ++w2) best = max(best, red[w2]);
            a.cp_out[q] = best;
        }
    }
}

// ---------------------------------------------------------------- launch helpers

inline int hip_ok(hipError_t e) { return e == hipSuccess ? CP_OK : CP_ERR_HIP; }

template <typename Tick, typename WT, bool MAGIC, bool TSWEEP>
int launch_column_sweep_t(const SweepLaunch &s, hipStream_t st, int32_t *launches) {
    const ColumnDir &dir = *s.dir;
    const int L = (int)dir.lvl_begin.size();
    const int ncol = (s.P + 63) / 64;
    const size_t tab_bytes = MAGIC ? sizeof(Magic) * ((size_t)s.k * s.k + s.k) : 0;
    ColumnArgs a{};
    a.ptr = (const int32_t *)(s.blob + dir.ptr_off);
    a.idx = (const int32_t *)(s.blob + dir.idx_off);
    a.wt = s.blob + dir.wt_off;
    a.c = s.blob + s.c_off;
    a.pT = s.pT;
    a.val = s.val;
    a.edge_tab = s.edge_tab;
    a.vert_tab = s.vert_tab;
    a.status = s.status;
    a.P = s.P; a.ncol = ncol; a.k = s.k;
    const int32_t *order = (const int32_t *)(s.blob + dir.order_off);
    int32_t count = 0;
    for (int l = 0; l < L; ++l) {
        const int32_t hubs = dir.lvl_hubs[l], total = dir.lvl_count[l];
        if (hubs > 0) {
            a.order = order + dir.lvl_begin[l];
            a.count = hubs;
            const int64_t blocks = (int64_t)hubs * ncol;
            const size_t lds_bytes = tab_bytes + sizeof(Tick) * 64 * kHubWaves;
            hipLaunchKernelGGL((column_level_kernel<Tick, WT, MAGIC, TSWEEP, true>),
                               dim3((unsigned)blocks), dim3(kHubWaves * 64), lds_bytes, st, a);
            ++count;
        }
        if (total > hubs) {
            a.order = order + dir.lvl_begin[l] + hubs;
            a.count = total - hubs;
            const int64_t tasks = (int64_t)(total - hubs) * ncol;
            hipLaunchKernelGGL((column_level_kernel<Tick, WT, MAGIC, TSWEEP, false>),
                               dim3((unsigned)((tasks + 3) / 4)), dim3(256), tab_bytes, st, a);
            ++count;
        }
    }
    if (launches) *launches = count;
    return hip_ok(hipGetLastError());
}

template <typename Tick, bool TSWEEP>
int launch_window_sweep_t(const SweepLaunch &s, hipStream_t st, int32_t *launches) {
    const WindowDir &dir = *s.win;
    WindowArgs a{};
    a.vtx = (const int32_t *)(s.blob + dir.vtx_off);
    a.c = (const uint32_t *)(s.blob + dir.c_off);
    a.deg = (const int32_t *)(s.blob + dir.deg_off);
    a.lvl = (const int32_t *)(s.blob + dir.lvl_off);
    a.slice_off = (const uint32_t *)(s.blob + dir.slice_off);
    a.ent = (const uint2 *)(s.blob + dir.ent_off);
    a.assign = s.assign;
    a.a_stride_p = s.a_stride_p;
    a.a_stride_v = s.a_stride_v;
    a.out = s.val;
    a.cp_out = s.cp_out;
    a.edge_tab = (const Magic *)s.edge_tab;
    a.vert_tab = (const Magic *)s.vert_tab;
    a.status = s.status;
    a.P = s.P; a.L = s.L; a.k = s.k; a.slots = dir.slots;
    const size_t lds_bytes = window_lds_bytes(s.k, dir.slots, sizeof(Tick));
    auto kern = window_sweep_kernel<Tick, TSWEEP>;
    if (lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return CP_ERR_HIP;
    }
    int threads = std::min<int>(kWindowMaxThreads, (s.max_width + 63) / 64 * 64);
    hipLaunchKernelGGL(kern, dim3((unsigned)s.P), dim3(threads), lds_bytes, st, a);
    if (launches) *launches = 1;
    return hip_ok(hipGetLastError());
}

}  // namespace

size_t window_lds_bytes(int32_t k, int32_t slots, size_t tick_bytes) {
    size_t tab = sizeof(Magic) * ((size_t)k * k + k);
    return align_up(tab + (tick_bytes + 1) * (size_t)slots, 16);
}

int launch_clear(int64_t *cp_out, int32_t batch, int32_t *status, void *stream) {
    hipLaunchKernelGGL(clear_kernel, dim3((batch + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       cp_out, batch, status);
    return hip_ok(hipGetLastError());
}

int launch_transpose(const uint8_t *in, uint8_t *out, int32_t n, int32_t P, void *stream) {
    dim3 grid((unsigned)((n + 63) / 64), (unsigned)((P + 63) / 64));
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, (hipStream_t)stream, in, out, n, P);
    return hip_ok(hipGetLastError());
}

int launch_column_sweep(const SweepLaunch &s, void *stream, int32_t *launches) {
    hipStream_t st = (hipStream_t)stream;
#define CP_COL(TICK, WT, MAGIC)                                                              \
    return s.tsweep ? launch_column_sweep_t<TICK, WT, MAGIC, true>(s, st, launches)          \
                    : launch_column_sweep_t<TICK, WT, MAGIC, false>(s, st, launches)
    if (s.tick_bytes == 4) {
        if (s.magic) { CP_COL(int32_t, uint32_t, true); }
        if (s.narrow) { CP_COL(int32_t, uint32_t, false); }
        CP_COL(int32_t, int64_t, false);
    } else {
        if (s.magic) { CP_COL(int64_t, uint32_t, true); }
        if (s.narrow) { CP_COL(int64_t, uint32_t, false); }
        CP_COL(int64_t, int64_t, false);
    }
#undef CP_COL
}

int launch_window_sweep(const SweepLaunch &s, void *stream, int32_t *launches) {
    hipStream_t st = (hipStream_t)stream;
    if (s.tick_bytes == 4)
        return s.tsweep ? launch_window_sweep_t<int32_t, true>(s, st, launches)
                        : launch_window_sweep_t<int32_t, false>(s, st, launches);
    return s.tsweep ? launch_window_sweep_t<int64_t, true>(s, st, launches)
                    : launch_window_sweep_t<int64_t, false>(s, st, launches);
}

int launch_cp_sources(const int32_t *sources, int32_t nsrc, const void *b, int32_t P,
                      int tick_bytes, int64_t *cp_out, void *stream) {
    const int ncol = (P + 63) / 64;
    int chunks = std::max(1, std::min(1024, (nsrc + 63) / 64));
    dim3 grid((unsigned)ncol, (unsigned)chunks);
    if (tick_bytes == 4)
        hipLaunchKernelGGL(cp_sources_kernel<int32_t>, grid, dim3(256), 0, (hipStream_t)stream,
                           sources, nsrc, (const int32_t *)b, P, cp_out);
    else
        hipLaunchKernelGGL(cp_sources_kernel<int64_t>, grid, dim3(256), 0, (hipStream_t)stream,
                           sources, nsrc, (const int64_t *)b, P, cp_out);
    return hip_ok(hipGetLastError());
}

int launch_mask(const void *b, const void *tl, const int64_t *cp, int32_t n, int32_t P,
                int tick_bytes, uint64_t *mask, void *stream) {
    const int ncol = (P + 63) / 64;
    const int64_t tasks = (int64_t)n * ncol;
    const unsigned blocks = (unsigned)std::max<int64_t>(1, std::min<int64_t>((tasks + 3) / 4, 256 * 64));
    if (tick_bytes == 4)
        hipLaunchKernelGGL(mask_kernel<int32_t>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const int32_t *)b, (const int32_t *)tl, cp, n, P, ncol, mask);
    else
        hipLaunchKernelGGL(mask_kernel<int64_t>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const int64_t *)b, (const int64_t *)tl, cp, n, P, ncol, mask);
    return hip_ok(hipGetLastError());
}

}  // namespace cpeval
