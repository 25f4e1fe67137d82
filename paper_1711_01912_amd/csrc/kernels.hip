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

#include <type_traits>

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

// Barrier that orders LDS traffic only: global loads issued by the loader
// wavefronts stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Device ids gathered into sweep order, one padded row of L*wpad bytes per
// partition, so that the sweep kernel streams them like the graph packets.
// Ids >= k are reported and replaced by 0.
__global__ __launch_bounds__(256) void gather_assign_kernel(const int32_t *__restrict__ gmap,
                                                            int64_t row_len,
                                                            const uint8_t *__restrict__ assign,
                                                            int64_t a_stride_p, int64_t a_stride_v,
                                                            int32_t k, uint8_t *__restrict__ out,
                                                            int32_t *status) {
    const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;   // row_len is a multiple of 64
    if (i4 >= row_len) return;
    const int64_t q = blockIdx.y;
    const int4 v = *(const int4 *)(gmap + i4);
    const uint8_t *row = assign + q * a_stride_p;
    uint32_t p0 = v.x >= 0 ? row[(int64_t)v.x * a_stride_v] : 0;
    uint32_t p1 = v.y >= 0 ? row[(int64_t)v.y * a_stride_v] : 0;
    uint32_t p2 = v.z >= 0 ? row[(int64_t)v.z * a_stride_v] : 0;
    uint32_t p3 = v.w >= 0 ? row[(int64_t)v.w * a_stride_v] : 0;
    if (max(max(p0, p1), max(p2, p3)) >= (uint32_t)k) {
        *status = CP_STATUS_BAD_DEVICE_ID;
        if (p0 >= (uint32_t)k) p0 = 0;
        if (p1 >= (uint32_t)k) p1 = 0;
        if (p2 >= (uint32_t)k) p2 = 0;
        if (p3 >= (uint32_t)k) p3 = 0;
    }
    *(uint32_t *)(out + q * row_len + i4) = p0 | (p1 << 8) | (p2 << 16) | (p3 << 24);
}

struct WindowArgs {
    const uint4 *stream;       // level packets
    const uint32_t *pkt_off;   // [L+1] first chunk of each packet
    const uint8_t *pperm;      // [P][L*wpad] device ids in sweep order
    void *out;                 // [n][P] ticks, or NULL
    int64_t *cp_out;           // [P] or NULL: receives the maximum of b over the partition
    const Magic *edge_tab;
    const Magic *vert_tab;
    int32_t P, L, k, slots, wpad;
    int32_t nc, nlw;           // compute and loader wavefronts per workgroup
    int32_t pgroups;           // partitions per XCD-sized group (blockIdx -> partition map)
};

template <typename Tick, bool PACKED> struct Ring;

// {value, device id} in one 8-byte element: one LDS read per relaxation
template <> struct Ring<int32_t, true> {
    uint2 *e;
    __device__ void init(uint8_t *base, int) { e = (uint2 *)base; }
    __device__ void put(int slot, int32_t val, uint32_t p) { e[slot] = make_uint2((uint32_t)val, p); }
    __device__ void get(int slot, int32_t &val, uint32_t &p) const {
        const uint2 x = e[slot];
        val = (int32_t)x.x;
        p = x.y;
    }
};
// separate arrays: 5 (or 9) bytes per slot when the window is large
template <typename Tick> struct Ring<Tick, false> {
    Tick *v;
    uint8_t *d;
    __device__ void init(uint8_t *base, int slots) {
        v = (Tick *)base;
        d = base + sizeof(Tick) * ((size_t)slots + 1);
    }
    __device__ void put(int slot, Tick val, uint32_t p) { v[slot] = val; d[slot] = (uint8_t)p; }
    __device__ void get(int slot, Tick &val, uint32_t &p) const { val = v[slot]; p = d[slot]; }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // stays in registers when indexed statically
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;   // uniform reads become scalar loads

// LDS layout: [tables][ring][stage slot 0][stage slot 1]; a stage slot is
// [wpad bytes of device ids][packet], NL*nlw*1024 bytes in all.
//
// Wavefronts 0..nc-1 compute, wavefronts nc..nc+nlw-1 load.  Tick t: after the
// barrier the compute wavefronts relax level t out of stage slot t&1 while the
// loaders copy packet t+1 (which they requested DR ticks earlier and hold in
// registers) into the other slot and request packet t+1+DR.  The only traffic on
// the level-to-level dependency is LDS.
template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4, int NL, int DR>
__global__ __launch_bounds__(kWindowMaxWaves * 64) void window_sweep_kernel(WindowArgs a) {
    extern __shared__ uint4 lds16[];
    __shared__ long long red[kWindowMaxWaves];
    uint8_t *lds = (uint8_t *)lds16;
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = a.k, L = a.L;

    // blockIdx -> partition: blocks are dealt round-robin to the 8 XCDs; give each
    // XCD a run of consecutive partitions so that the 4-byte stores of one output
    // line meet in one L2
    const int32_t q = (int32_t)(blockIdx.x % 8) * a.pgroups + (int32_t)(blockIdx.x / 8);
    if (q >= a.P) return;      // whole workgroup: no barrier has been reached yet

    Magic *etab = (Magic *)lds;
    Magic *vtab = etab + k * k;
    const size_t tab_bytes = (sizeof(Magic) * ((size_t)k * k + k) + 15) & ~(size_t)15;
    const size_t ring_bytes = (((size_t)a.slots + 1) * (PACKED ? 8 : sizeof(Tick) + 1) + 15) & ~(size_t)15;
    Ring<Tick, PACKED> ring;
    ring.init(lds + tab_bytes, a.slots);
    const int slot_chunks = NL * a.nlw * 64;
    uint4 *stage = (uint4 *)(lds + tab_bytes + ring_bytes);
    {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
        uint64_t *t64 = (uint64_t *)lds;
        for (int i = tid; i < k * k; i += nt) t64[i] = e[i];
        for (int i = tid; i < k; i += nt) t64[k * k + i] = v[i];
        if (tid == 0) ring.put(a.slots, 0, 0);     // the constant-zero slot padding entries point at
    }

    const int Lpad = (L + DR - 1) / DR * DR;
    const int wp16 = a.wpad / 16;
    long long best = 0;

    if (wave >= a.nc) {
        // ------------------------------------------------ loader wavefronts
        const int lw = wave - a.nc;
        const uint4 *pp = (const uint4 *)(a.pperm + (size_t)q * L * a.wpad);
        const_u32_ptr pkt_off = (const_u32_ptr)a.pkt_off;
        u32x4 buf[DR][NL];
        // every lane always loads: chunks past the packet's end re-read its last chunk
#define CP_ISSUE(R, S)                                                                          \
    do {                                                                                        \
        const int s_ = min((S), L - 1);                                                         \
        const uint32_t o0_ = pkt_off[s_], o1_ = pkt_off[s_ + 1];                                \
        const int nchunks_ = wp16 + (int)(o1_ - o0_);                                           \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                     \
            const int c_ = min((i_ * a.nlw + lw) * 64 + lane, nchunks_ - 1);                    \
            const uint4 *src_ = c_ < wp16 ? pp + (size_t)s_ * wp16 + c_                         \
                                          : a.stream + (size_t)o0_ + (c_ - wp16);               \
            buf[R][i_] = *(const u32x4 *)src_;                                                  \
        }                                                                                       \
    } while (0)
#define CP_STORE(R, SLOT)                                                                       \
    do {                                                                                        \
        u32x4 *dst_ = (u32x4 *)(stage + (size_t)(SLOT) * slot_chunks);                          \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_)                                       \
            dst_[(i_ * a.nlw + lw) * 64 + lane] = buf[R][i_];                                   \
    } while (0)
#pragma unroll
        for (int r = 0; r < DR; ++r) CP_ISSUE(r, r);
        CP_STORE(0, 0);
        CP_ISSUE(0, DR);
        for (int t0 = 0; t0 < Lpad; t0 += DR) {
#pragma unroll
            for (int r = 0; r < DR; ++r) {
                const int t = t0 + r;
                lds_barrier();
                CP_STORE((r + 1) % DR, (t + 1) & 1);
                CP_ISSUE((r + 1) % DR, t + 1 + DR);
            }
        }
#undef CP_ISSUE
#undef CP_STORE
    } else {
        // ------------------------------------------------ compute wavefronts
        typedef typename std::conditional<ENT4, uint32_t, uint2>::type Ent;
        Tick *out = a.out ? (Tick *)a.out + q : nullptr;
        const int32_t P = a.P, R = a.slots;
        for (int t = 0; t < Lpad; ++t) {
            lds_barrier();
            if (t >= L) continue;
            const uint8_t *st = (const uint8_t *)(stage + (size_t)(t & 1) * slot_chunks);
            const uint8_t *pk = st + a.wpad;
            const uint4 hdr = *(const uint4 *)pk;
            const int npos = __builtin_amdgcn_readfirstlane((int)hdr.x);
            const int nsl = __builtin_amdgcn_readfirstlane((int)hdr.y);
            const int rbase = __builtin_amdgcn_readfirstlane((int)hdr.z);
            const uint2 *slice_tab = (const uint2 *)(pk + 16);
            const uint2 *rec = (const uint2 *)(pk + 16 + ((8 * nsl + 15) & ~15));
            const Ent *ent_all = (const Ent *)(rec + (size_t)64 * nsl);
            for (int j = wave; j < nsl; j += a.nc) {
                const uint2 sl = slice_tab[j];
                const int ebase = __builtin_amdgcn_readfirstlane((int)sl.x);
                const int width = __builtin_amdgcn_readfirstlane((int)(sl.y & 0xffffffu));
                const int lsh = __builtin_amdgcn_readfirstlane((int)(sl.y >> 24));   // log2 lanes per row
                const int p = j * 64 + (lane >> lsh);
                const uint2 rc = rec[p];
                const uint32_t pv = st[p];
                const Ent *ent = ent_all + ebase + lane;
                const Magic *erow = etab + pv * k;
                Tick acc = 0;
#pragma unroll 4
                for (int jj = 0; jj < width; ++jj) {
                    uint32_t slot, te;
                    if constexpr (ENT4) {
                        const uint32_t en = ent[jj * 64];
                        slot = en & 0xffffu;
                        te = en >> 16;
                    } else {
                        const uint2 en = ent[jj * 64];
                        slot = en.x;
                        te = en.y;
                    }
                    Tick vu;
                    uint32_t pu;
                    ring.get((int)slot, vu, pu);
                    const Tick x = (Tick)magic_div(te, erow[pu]);
                    acc = max(acc, (Tick)(vu + x));
                }
                for (int off = (1 << lsh) >> 1; off > 0; off >>= 1)   // fold the lanes of a row
                    acc = max(acc, __shfl_xor(acc, off));
                if (p < npos && (lane & ((1 << lsh) - 1)) == 0) {
                    const Tick fin = acc + (Tick)magic_div(rc.y, vtab[pv]);   // b(v), or tl(v) + w(v)
                    int rs = rbase + p;
                    if (rs >= R) rs -= R;
                    ring.put(rs, fin, pv);
                    if (out) out[(size_t)rc.x * P] = TSWEEP ? acc : fin;
                    best = max(best, (long long)fin);
                }
            }
        }
    }

    if (a.cp_out) {   // workgroup maximum
        for (int off = 32; off > 0; off >>= 1) best = max(best, __shfl_xor(best, off));
        if (lane == 0) red[wave] = best;
        lds_barrier();
        if (tid == 0) {
            for (int w2 = 1; w2 < a.nc; ++w2) best = max(best, red[w2]);
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

template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4, int NL, int DR>
int launch_window_sweep_k(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    const WindowDir &dir = *s.win;
    WindowArgs a{};
    a.stream = (const uint4 *)(s.blob + dir.stream_off);
    a.pkt_off = (const uint32_t *)(s.blob + dir.pkt_off);
    a.pperm = s.pperm;
    a.out = s.val;
    a.cp_out = s.cp_out;
    a.edge_tab = (const Magic *)s.edge_tab;
    a.vert_tab = (const Magic *)s.vert_tab;
    a.P = s.P; a.L = s.L; a.k = s.k; a.slots = dir.slots; a.wpad = dir.wpad;
    a.nc = cfg.nc; a.nlw = cfg.nlw;
    a.pgroups = (s.P + 7) / 8;
    auto kern = window_sweep_kernel<Tick, TSWEEP, PACKED, ENT4, NL, DR>;
    if (cfg.lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)cfg.lds_bytes);
        if (e != hipSuccess) return CP_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * a.pgroups)), dim3((cfg.nc + cfg.nlw) * 64),
                       cfg.lds_bytes, st, a);
    return hip_ok(hipGetLastError());
}

template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4>
int launch_window_sweep_e(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    switch (cfg.nl) {   // loads per loader lane per level x levels in flight: 64 registers at most
        case 1: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 1, 8>(s, cfg, st);
        case 2: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 2, 8>(s, cfg, st);
        case 4: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 4, 4>(s, cfg, st);
        case 8: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 8, 2>(s, cfg, st);
        default: return CP_ERR_ARG;
    }
}

template <typename Tick, bool TSWEEP, bool PACKED>
int launch_window_sweep_p(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    return s.win->ent4 ? launch_window_sweep_e<Tick, TSWEEP, PACKED, true>(s, cfg, st)
                       : launch_window_sweep_e<Tick, TSWEEP, PACKED, false>(s, cfg, st);
}

template <bool TSWEEP>
int launch_window_sweep_d(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    if (s.tick_bytes == 4)
        return cfg.packed ? launch_window_sweep_p<int32_t, TSWEEP, true>(s, cfg, st)
                          : launch_window_sweep_p<int32_t, TSWEEP, false>(s, cfg, st);
    return launch_window_sweep_p<int64_t, TSWEEP, false>(s, cfg, st);
}

}  // namespace

bool window_config(const WindowDir &d, int32_t k, size_t tick_bytes, size_t lds_limit, WindowCfg &out) {
    const int64_t need = d.wpad / 16 + (int64_t)d.max_chunks;     // 16-byte chunks per stage slot
    const size_t tab = (sizeof(Magic) * ((size_t)k * k + k) + 15) & ~(size_t)15;
    static const int kNl[4] = {1, 2, 4, 8};
    for (int nl : kNl) {
        const int64_t nlw = (need + 64 * nl - 1) / (64 * nl);
        if (nlw > 8) continue;
        out.nl = nl;
        out.nlw = (int)nlw;
        out.dr = nl <= 2 ? 8 : (nl == 4 ? 4 : 2);
        out.nc = std::max(1, std::min(d.smax, kWindowMaxWaves - (int)nlw));
        const size_t stage = (size_t)2 * nl * nlw * 1024;
        const size_t packed = (8 * ((size_t)d.slots + 1) + 15) & ~(size_t)15;
        const size_t split = ((tick_bytes + 1) * ((size_t)d.slots + 1) + 15) & ~(size_t)15;
        if (tick_bytes == 4 && tab + packed + stage <= lds_limit) {
            out.packed = true;
            out.lds_bytes = tab + packed + stage;
            return true;
        }
        if (tab + split + stage <= lds_limit) {
            out.packed = false;
            out.lds_bytes = tab + split + stage;
            return true;
        }
        return false;
    }
    return false;
}

int launch_gather_assign(const SweepLaunch &s, uint8_t *out, void *stream) {
    const WindowDir &dir = *s.win;
    const int64_t row_len = (int64_t)s.L * dir.wpad;
    const int64_t chunks = (row_len + 1023) / 1024;
    if (chunks > 65535) return CP_ERR_SIZE;
    hipLaunchKernelGGL(gather_assign_kernel, dim3((unsigned)chunks, (unsigned)s.P), dim3(256), 0,
                       (hipStream_t)stream, (const int32_t *)(s.blob + dir.gmap_off), row_len,
                       s.assign, s.a_stride_p, s.a_stride_v, s.k, out, s.status);
    return hip_ok(hipGetLastError());
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

int launch_window_sweep(const SweepLaunch &s, const WindowCfg &cfg, void *stream, int32_t *launches) {
    if (launches) *launches = 1;
    return s.tsweep ? launch_window_sweep_d<true>(s, cfg, (hipStream_t)stream)
                    : launch_window_sweep_d<false>(s, cfg, (hipStream_t)stream);
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
