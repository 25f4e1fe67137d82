// Column-slice sweep: the wave-column layout walked by persistent workgroups.
//
// Distances live in HBM as [vertex][partition] and one wavefront relaxes one vertex for 64
// consecutive partitions, exactly as in the wave-column plan; but one workgroup owns a slice
// of 64 partitions and walks all levels in a single launch.  A slice never reads another
// slice's columns, so the only synchronisation between levels is the workgroup's own barrier
// (with the level's stores made visible to the whole GPU and the compute unit's vector cache
// invalidated, since the next level's gathers are served by L2).  The recurrences are those
// of the other plans (b-level: the PCT equation of section 4.1; t-level: the downward rank of
// section 3.2 without the own term).
#include <hip/hip_runtime.h>

#include "device_math.hpp"
#include "launch.hpp"

namespace cpeval {
namespace {

constexpr int kSliceWaves = 16;

struct SliceArgs {
    const int32_t *ptr;
    const int32_t *idx;
    const uint32_t *wt;
    const uint32_t *c;
    const int32_t *order;   // vertices in sweep order
    const int32_t *lvl;     // [L][4] {first position, hub rows, rows, 0}
    const uint8_t *pT;      // [n][P]
    void *val;              // [n][P] ticks
    const Magic *edge_tab;  // [k*k] for this sweep
    const Magic *vert_tab;  // [k]
    int32_t *status;
    int32_t P, k, L;
};

__device__ __forceinline__ int32_t bcast(int32_t v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

template <typename Tick, bool TSWEEP>
__global__ __launch_bounds__(kSliceWaves * 64) void column_slice_kernel(SliceArgs a) {
    extern __shared__ uint64_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = a.k;
    {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
        for (int i = tid; i < k * k; i += blockDim.x) lds[i] = e[i];
        for (int i = tid; i < k; i += blockDim.x) lds[k * k + i] = v[i];
    }
    const Magic *etab = (const Magic *)lds;
    const Magic *vtab = etab + k * k;
    Tick *part = (Tick *)(lds + k * k + k);          // [kSliceWaves][64] partial maxima of a hub row
    __syncthreads();

    const int32_t P = a.P;
    const int32_t q = (int32_t)blockIdx.x * 64 + lane;
    const bool live = q < P;
    const size_t qq = live ? (size_t)q : 0;          // lanes past the batch read column 0 and store nothing
    const uint8_t *pT = a.pT + qq;
    Tick *val = (Tick *)a.val + qq;
    bool bad = false;

    // the edges base .. base+cnt-1 of vertex v's row, four at a time: all gathers first, then
    // the arithmetic; a short last group repeats its last edge (the maximum does not notice)
    auto relax = [&](int32_t e0, int32_t e1, uint32_t pv) -> Tick {
        Tick acc = 0;
        for (int32_t base = e0; base < e1; base += 64) {
            const int32_t cnt = min(64, e1 - base);
            int32_t my_u = 0, my_t = 0;
            if (lane < cnt) { my_u = a.idx[base + lane]; my_t = (int32_t)a.wt[base + lane]; }
            for (int j = 0; j < cnt; j += 4) {
                int32_t u[4], te[4];
                uint32_t pu[4], cu[4];
                Tick vu[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int jj = min(j + i, cnt - 1);
                    u[i] = bcast(my_u, jj);
                    te[i] = bcast(my_t, jj);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pu[i] = pT[(size_t)u[i] * P];
                    vu[i] = val[(size_t)u[i] * P];
                    if (TSWEEP) cu[i] = a.c[u[i]];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t d = min(pu[i], (uint32_t)(k - 1));
                    Tick x = vu[i];
                    if (TSWEEP) x += (Tick)magic_div(cu[i], vtab[d]);   // the tail's finish time tl + w
                    x += (Tick)magic_div((uint32_t)te[i], etab[pv * k + d]);
                    acc = max(acc, x);
                }
            }
        }
        return acc;
    };

    for (int32_t l = 0; l < a.L; ++l) {
        const int32_t begin = a.lvl[4 * l], hubs = a.lvl[4 * l + 1], count = a.lvl[4 * l + 2];
        // rows of kHubDegree edges or more: the workgroup's wavefronts split the row
        for (int32_t i = 0; i < hubs; ++i) {
            const int32_t v = a.order[begin + i];
            uint32_t pv = pT[(size_t)v * P];
            if (pv >= (uint32_t)k) { bad = true; pv = 0; }
            const int32_t r0 = a.ptr[v], r1 = a.ptr[v + 1];
            const int32_t chunk = (r1 - r0 + kSliceWaves - 1) / kSliceWaves;
            const int32_t e0 = min(r1, r0 + wave * chunk), e1 = min(r1, e0 + chunk);
            part[wave * 64 + lane] = relax(e0, e1, pv);
            __syncthreads();
            if (wave == 0) {
                Tick acc = 0;
                for (int w2 = 0; w2 < kSliceWaves; ++w2) acc = max(acc, part[w2 * 64 + lane]);
                const Tick w = (Tick)magic_div(a.c[v], vtab[pv]);
                if (live) val[(size_t)v * P] = TSWEEP ? acc : (Tick)(acc + w);
            }
            __syncthreads();
        }
        for (int32_t i = hubs + wave; i < count; i += kSliceWaves) {
            const int32_t v = a.order[begin + i];
            uint32_t pv = pT[(size_t)v * P];
            if (pv >= (uint32_t)k) { bad = true; pv = 0; }
            const Tick acc = relax(a.ptr[v], a.ptr[v + 1], pv);
            const Tick w = (Tick)magic_div(a.c[v], vtab[pv]);
            if (live) val[(size_t)v * P] = TSWEEP ? acc : (Tick)(acc + w);
        }
        // the level's values are in L2 before any wavefront of the slice reads them
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    if (bad && live) *a.status = CP_STATUS_BAD_DEVICE_ID;
}

}  // namespace

int launch_column_slice(const SweepLaunch &s, void *stream) {
    if (!s.magic || !s.narrow || s.k > kMagicMaxK) return CP_ERR_ARG;
    const ColumnDir &dir = *s.dir;
    SliceArgs a{};
    a.ptr = (const int32_t *)(s.blob + dir.ptr_off);
    a.idx = (const int32_t *)(s.blob + dir.idx_off);
    a.wt = (const uint32_t *)(s.blob + dir.wt_off);
    a.c = (const uint32_t *)(s.blob + s.c_off);
    a.order = (const int32_t *)(s.blob + dir.order_off);
    a.lvl = (const int32_t *)(s.blob + dir.lvl_off);
    a.pT = s.pT;
    a.val = s.val;
    a.edge_tab = (const Magic *)s.edge_tab;
    a.vert_tab = (const Magic *)s.vert_tab;
    a.status = s.status;
    a.P = s.P; a.k = s.k; a.L = (int32_t)dir.lvl_begin.size();
    const size_t lds = sizeof(Magic) * ((size_t)s.k * s.k + s.k) + (size_t)s.tick_bytes * 64 * kSliceWaves;
    const dim3 grid((unsigned)((s.P + 63) / 64)), block(kSliceWaves * 64);
    hipStream_t st = (hipStream_t)stream;
    if (s.tick_bytes == 4) {
        if (s.tsweep) hipLaunchKernelGGL((column_slice_kernel<int32_t, true>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((column_slice_kernel<int32_t, false>), grid, block, lds, st, a);
    } else {
        if (s.tsweep) hipLaunchKernelGGL((column_slice_kernel<int64_t, true>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((column_slice_kernel<int64_t, false>), grid, block, lds, st, a);
    }
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
}

}  // namespace cpeval
