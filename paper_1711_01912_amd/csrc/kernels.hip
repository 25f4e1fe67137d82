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

#include "device_math.hpp"
#include "launch.hpp"

namespace cpeval {
namespace {

// ---------------------------------------------------------------- cost policies

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

__global__ void zero_words_kernel(uint64_t *dst, int64_t words) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = 0;
}

__global__ void zero_bytes_kernel(uint8_t *dst, int64_t bytes) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < bytes) dst[i] = 0;
}

// Ranks of section 3.2 from the one-device, unit-speed evaluation: upRank = b,
// downRank = tl + c (the rank equation adds the vertex's own c), totalRank = their sum.
template <typename Tick, typename WT>
__global__ void ranks_kernel(const Tick *__restrict__ b, const Tick *__restrict__ tl,
                             const WT *__restrict__ c, int32_t n, int64_t *__restrict__ up,
                             int64_t *__restrict__ down, int64_t *__restrict__ total) {
    int32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    const int64_t u = (int64_t)b[v], d = (int64_t)tl[v] + (int64_t)c[v];
    if (up) up[v] = u;
    if (down) down[v] = d;
    if (total) total[v] = u + d;
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

// The same with four ids per load and per store, for n and P multiples of four and 4-byte
// aligned arrays: a tile of 64 partitions x 256 vertices, a row of it read as 64 words, a
// vertex's 64 ids written as 16 words, each put together from four rows of the tile.
__global__ __launch_bounds__(256) void transpose4_kernel(const uint8_t *__restrict__ in, uint8_t *__restrict__ out,
                                                         int32_t n, int32_t P) {
    __shared__ uint32_t tile[64][65];
    const int64_t v0 = (int64_t)blockIdx.x * 256, p0 = (int64_t)blockIdx.y * 64;
    const int lane = threadIdx.x & 63, row0 = threadIdx.x >> 6;
    for (int r = row0; r < 64; r += 4) {
        const int64_t p = p0 + r, v = v0 + 4 * lane;
        if (p < P && v < n) tile[r][lane] = *(const uint32_t *)(in + p * n + v);
    }
    __syncthreads();
    const uint8_t *bytes = (const uint8_t *)&tile[0][0];
    for (int it = 0; it < 16; ++it) {
        const int idx = it * 256 + threadIdx.x;
        const int vl = idx >> 4, pq = idx & 15;
        const int64_t v = v0 + vl, p = p0 + 4 * pq;
        if (v < n && p < P) {
            const uint32_t w = (uint32_t)bytes[(4 * pq + 0) * 260 + vl] | (uint32_t)bytes[(4 * pq + 1) * 260 + vl] << 8 |
                               (uint32_t)bytes[(4 * pq + 2) * 260 + vl] << 16 |
                               (uint32_t)bytes[(4 * pq + 3) * 260 + vl] << 24;
            *(uint32_t *)(out + v * P + p) = w;
        }
    }
}

// ---------------------------------------------------------------- wave-column sweep

struct ColumnArgs {
    const int32_t *idx;
    const void *wt;
    const void *c;
    const int4 *rows;       // {vertex, first edge, end of edges, 0} per position, offset to this launch's first
    const uint8_t *pT;      // [n][P]
    void *val;              // [n][P] ticks: b (b sweep) or tl (t sweep)
    const void *edge_tab;   // Magic[k*k] or int64[k*k] for this sweep
    const void *vert_tab;   // Magic[k] or int64[k]
    int32_t *status;
    int32_t P, ncol, k, count;
};

constexpr int kColumnUnroll = 4;      // neighbours whose loads are in flight together
template <typename Tick, typename WT, bool MAGIC, bool TSWEEP, bool HUB>
__global__ __launch_bounds__(HUB ? kHubWaves * 64 : 256) void column_level_kernel(ColumnArgs a) {
    extern __shared__ uint64_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = a.k;
    const int ntab = MAGIC ? k * k + k : 0;
    const Magic *etab_m = (const Magic *)lds;
    const Magic *vtab_m = etab_m + k * k;
    const int64_t *etab_g = (const int64_t *)a.edge_tab;
    const int64_t *vtab_g = (const int64_t *)a.vert_tab;

    // What the wavefront needs to start (its row's record, its vertex's device ids, the first 64
    // neighbours) is asked for before the cost tables are copied into LDS, so that the copy and
    // its barrier overlap those round trips instead of preceding them.
    const int64_t task = HUB ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
    const int64_t ntasks = (int64_t)a.count * a.ncol;
    const bool task_live = task < ntasks;
    const int32_t vi = task_live ? (int32_t)(task / a.ncol) : 0;
    const int32_t col = task_live ? (int32_t)(task % a.ncol) : 0;
    const int4 rec = a.rows[vi];          // one load instead of the vertex number and then its row bounds
    const int32_t v = rec.x;
    const int32_t q = col * 64 + lane;
    const int32_t P = a.P;
    const bool live = task_live && q < P;
    const uint8_t *pT = a.pT + q;
    Tick *val = (Tick *)a.val + q;
    const WT *wt = (const WT *)a.wt;
    const WT *cw = (const WT *)a.c;

    uint32_t pv = 0;
    if (live) pv = pT[(size_t)v * P];

    int32_t e0 = rec.y, e1 = rec.z;
    if (HUB) {  // this wavefront's share of the row
        int32_t len = e1 - e0, chunk = (len + kHubWaves - 1) / kHubWaves;
        e0 = min(e1, e0 + wave * chunk);
        e1 = min(e1, e0 + chunk);
    }
    if (!task_live) e1 = e0;
    int32_t first_u = 0;
    WT first_t = 0;
    if (e0 + lane < e1) { first_u = a.idx[e0 + lane]; first_t = wt[e0 + lane]; }

    if (MAGIC) {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *vt = (const uint64_t *)a.vert_tab;
        for (int i = tid; i < k * k; i += blockDim.x) lds[i] = e[i];
        for (int i = tid; i < k; i += blockDim.x) lds[k * k + i] = vt[i];
        __syncthreads();
    }
    if (live && pv >= (uint32_t)k) { *a.status = CP_STATUS_BAD_DEVICE_ID; pv = 0; }

    Tick acc = 0;
    for (int32_t base = e0; base < e1; base += 64) {
        const int32_t cnt = min(64, e1 - base);
        int32_t my_u = first_u;
        WT my_t = first_t;
        if (base != e0) {
            my_u = 0;
            my_t = 0;
            if (lane < cnt) { my_u = a.idx[base + lane]; my_t = wt[base + lane]; }
        }
        // four neighbours at a time: their device ids and values are four independent pairs of
        // loads in flight per lane (one pair at a time leaves the memory system a third busy);
        // slots past the row's end repeat its last neighbour and are left out of the maximum
        for (int j = 0; j < cnt; j += kColumnUnroll) {
            int32_t u[kColumnUnroll];
            WT te[kColumnUnroll], cu[kColumnUnroll];
            uint32_t pu[kColumnUnroll];
            Tick vu[kColumnUnroll];
#pragma unroll
            for (int i = 0; i < kColumnUnroll; ++i) {
                const int jj = min(j + i, cnt - 1);
                u[i] = wave_bcast<int32_t>(my_u, jj);
                te[i] = wave_bcast<WT>(my_t, jj);
            }
            if (live) {
#pragma unroll
                for (int i = 0; i < kColumnUnroll; ++i) {
                    pu[i] = pT[(size_t)u[i] * P];
                    vu[i] = val[(size_t)u[i] * P];
                    if (TSWEEP) cu[i] = cw[u[i]];
                }
#pragma unroll
                for (int i = 0; i < kColumnUnroll; ++i) {
                    const uint32_t pd = min(pu[i], (uint32_t)(k - 1));
                    Tick t = vu[i];
                    if (TSWEEP)   // neighbour is a predecessor: its finish time is tl(u) + w(u)
                        t += MAGIC ? (Tick)magic_div((uint32_t)cu[i], vtab_m[pd])
                                   : (Tick)plain_div((uint64_t)cu[i], (uint64_t)vtab_g[pd]);
                    const Tick x = MAGIC ? (Tick)magic_div((uint32_t)te[i], etab_m[pv * k + pd])
                                         : (Tick)plain_div((uint64_t)te[i], (uint64_t)etab_g[pv * k + pd]);
                    if (j + i < cnt) acc = max(acc, (Tick)(t + x));
                }
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

// Vertex-major (BY_PARTITION = false): b, tl are [n][P] and mask[v][word] bit i =
// (tl + b == CP) for partition 64*word + i.  Partition-major: b, tl are [P][n] and
// mask[q][word] bit i belongs to vertex 64*word + i.  Either way rows x cols ticks are
// read row by row; a wavefront takes four (row, word) tasks per trip so that eight
// loads are in flight.
template <typename Tick, bool BY_PARTITION>
__global__ __launch_bounds__(256) void mask_kernel(const Tick *__restrict__ b,
                                                   const Tick *__restrict__ tl,
                                                   const int64_t *__restrict__ cp, int32_t rows,
                                                   int32_t cols, int32_t ncol, uint64_t *mask) {
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t ntasks = (int64_t)rows * ncol;
    for (int64_t task0 = wave0 * 4; task0 < ntasks; task0 += nwaves * 4) {
        Tick vb[4], vt[4];
        int64_t c[4];
        bool live[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t task = task0 + u;
            const int64_t r = task / ncol;
            const int32_t i = (int32_t)(task % ncol) * 64 + lane;
            live[u] = task < ntasks && i < cols;
            vb[u] = 0; vt[u] = 0; c[u] = -1;
            if (live[u]) {
                const size_t at = (size_t)r * cols + i;
                vt[u] = __builtin_nontemporal_load(tl + at);      // read once, far larger than the caches
                vb[u] = __builtin_nontemporal_load(b + at);
                c[u] = cp[BY_PARTITION ? r : (int64_t)i];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t word = __ballot(live[u] && (int64_t)vt[u] + (int64_t)vb[u] == c[u]);
            if (lane == 0 && task0 + u < ntasks) mask[task0 + u] = word;
        }
    }
}

// The same for rows of 32-bit ticks that start on 16-byte boundaries (a row length that is a
// multiple of 4), rows per partition or per vertex: a lane takes four consecutive columns with
// one 16-byte load from either array, a wavefront kMaskTrips x 256 columns.  The four match
// bits of a lane are bits 4 (lane mod 16) .. +3 of mask word (lane / 16) of the trip's four
// words; the sixteen lanes of a word fold with shuffles.  Both arrays are read once and far
// exceed the caches: the loads carry the non-temporal hint, and a wavefront takes one trip
// (6.2 TB/s on the large sparse batch; 5.1 TB/s with plain loads and four trips).
constexpr int kMaskTrips = 1;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool BY_PARTITION>
__global__ __launch_bounds__(256) void mask_rows_kernel(const int32_t *__restrict__ b, const int32_t *__restrict__ tl,
                                                        const int64_t *__restrict__ cp, int32_t n, int32_t ncol,
                                                        uint64_t *mask) {
    // n: the length of a row (vertices with rows per partition, else partitions).  The row's
    // number sits in whichever grid dimension takes it: there may be millions of vertices.
    const int lane = threadIdx.x & 63;
    const int32_t r = BY_PARTITION ? blockIdx.y : blockIdx.x;
    const int64_t wave = (int64_t)(BY_PARTITION ? blockIdx.x : blockIdx.y) * 4 + (threadIdx.x >> 6);
    const int64_t v0 = wave * (256 * kMaskTrips);                    // first column of this wavefront
    if (v0 >= n) return;
    const int64_t c_row = BY_PARTITION ? cp[r] : 0;
    const uint4 *b4 = (const uint4 *)(b + (size_t)r * n), *t4 = (const uint4 *)(tl + (size_t)r * n);
    uint4 vb[kMaskTrips], vt[kMaskTrips];
    int64_t c[kMaskTrips][4];
#pragma unroll
    for (int u = 0; u < kMaskTrips; ++u) {
        const int64_t v = v0 + 256 * u + 4 * lane;
        vb[u] = make_uint4(0, 0, 0, 0);
        vt[u] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) c[u][j] = c_row;
        if (v < n) {                                                 // n is a multiple of 4: all four or none
            const u32x4 xt = __builtin_nontemporal_load((const u32x4 *)t4 + (v >> 2));
            const u32x4 xb = __builtin_nontemporal_load((const u32x4 *)b4 + (v >> 2));
            vt[u] = make_uint4(xt.x, xt.y, xt.z, xt.w);
            vb[u] = make_uint4(xb.x, xb.y, xb.z, xb.w);
            if (!BY_PARTITION) {                                     // a column is a partition: its own CP
#pragma unroll
                for (int j = 0; j < 4; ++j) c[u][j] = cp[v + j];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kMaskTrips; ++u) {
        const int64_t v = v0 + 256 * u + 4 * lane;
        uint32_t nib = 0;
        if (v < n) {
            nib = (uint32_t)((int64_t)(int32_t)vt[u].x + (int32_t)vb[u].x == c[u][0]) |
                  (uint32_t)((int64_t)(int32_t)vt[u].y + (int32_t)vb[u].y == c[u][1]) << 1 |
                  (uint32_t)((int64_t)(int32_t)vt[u].z + (int32_t)vb[u].z == c[u][2]) << 2 |
                  (uint32_t)((int64_t)(int32_t)vt[u].w + (int32_t)vb[u].w == c[u][3]) << 3;
        }
        uint64_t word = (uint64_t)nib << (4 * (lane & 15));
        word |= __shfl_xor(word, 1);
        word |= __shfl_xor(word, 2);
        word |= __shfl_xor(word, 4);
        word |= __shfl_xor(word, 8);
        const int64_t w = (v0 + 256 * u) / 64 + (lane >> 4);
        if ((lane & 15) == 0 && w < ncol) mask[(size_t)r * ncol + w] = word;
    }
}

// in[rows][cols] -> out[cols][rows], 64 x 64 tiles through LDS
template <typename T>
__global__ __launch_bounds__(256) void transpose_ticks_kernel(const T *__restrict__ in, T *__restrict__ out,
                                                              int32_t rows, int32_t cols) {
    __shared__ T tile[64][65];
    const int lane = threadIdx.x & 63, row0 = threadIdx.x >> 6;
    const int64_t r0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
    for (int r = row0; r < 64; r += 4)
        if (r0 + r < rows && c0 + lane < cols) tile[r][lane] = in[(r0 + r) * cols + c0 + lane];
    __syncthreads();
    for (int c = row0; c < 64; c += 4)
        if (c0 + c < cols && r0 + lane < rows) out[(c0 + c) * rows + r0 + lane] = tile[lane][c];
}

// ---------------------------------------------------------------- one critical path

struct PathArgs {
    const int32_t *ptr;      // successor CSR over original ids
    const int32_t *idx;
    const void *wt;
    const void *c;
    const int32_t *sources;
    int32_t nsrc;
    const uint8_t *assign;
    int64_t a_stride_p, a_stride_v;
    const void *b;           // ticks; b(v, q) sits at v * b_sv + q * b_sq
    int64_t b_sv, b_sq;
    const int64_t *cp;       // [P]
    const void *edge_tab;    // b-sweep orientation: row = device of the edge's source vertex
    const void *vert_tab;
    int32_t *path;           // [P][max_len]
    int32_t *len;            // [P]
    int32_t *status;
    int32_t P, k, max_len;
};

// One wavefront walks one partition's critical path (section 3.2.2, read as: the
// lexicographically smallest source-to-sink vertex sequence of cost CP).  It starts at
// the lowest-numbered source whose b equals CP; from v it moves to the lowest-numbered
// successor u with b(v) = w(v) + x(v->u) + b(u), lanes across the successors.
// With LDS_TAB the k*k + k table entries are staged in LDS first (one dependent
// global load less per step of the walk).
template <typename Tick, typename WT, bool MAGIC, bool LDS_TAB>
__global__ __launch_bounds__(64) void critical_path_kernel(PathArgs a) {
    extern __shared__ __align__(16) uint64_t path_lds[];
    const int lane = threadIdx.x;
    const int32_t q = blockIdx.x;
    const int32_t k = a.k;
    const Tick *b = (const Tick *)a.b + (int64_t)q * a.b_sq;
    const int64_t bsv = a.b_sv;
    const uint8_t *row = a.assign + (int64_t)q * a.a_stride_p;
    const WT *wt = (const WT *)a.wt;
    const WT *cw = (const WT *)a.c;
    const void *etab = a.edge_tab, *vtab = a.vert_tab;
    if (LDS_TAB) {
        const uint64_t *ge = (const uint64_t *)a.edge_tab, *gv = (const uint64_t *)a.vert_tab;
        for (int i = lane; i < k * k; i += 64) path_lds[i] = ge[i];
        for (int i = lane; i < k; i += 64) path_lds[k * k + i] = gv[i];
        __syncthreads();
        etab = path_lds;
        vtab = path_lds + k * k;
    }
    const Magic *etab_m = (const Magic *)etab, *vtab_m = (const Magic *)vtab;
    const int64_t *etab_g = (const int64_t *)etab, *vtab_g = (const int64_t *)vtab;
    int32_t *path = a.path + (int64_t)q * a.max_len;
    for (int i = lane; i < a.max_len; i += 64) path[i] = -1;

    const long long cpq = a.cp[q];
    int32_t v = 0x7fffffff;
    for (int32_t i = lane; i < a.nsrc; i += 64) {
        const int32_t s = a.sources[i];
        if ((long long)b[(int64_t)s * bsv] == cpq) v = min(v, s);
    }
    for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off));

    // What the walk needs of the current vertex: its device, c, b and row bounds.  For the
    // start they are loaded here; afterwards every lane fetches them for the successor it
    // examines, together with that successor's b and device, and the winner's copy is
    // broadcast: two dependent rounds of loads per path vertex instead of three.
    uint32_t pv = 0;
    WT cv = 0;
    Tick bv = 0;
    int32_t e0 = 0, e1 = 0;
    if (v != 0x7fffffff) {
        pv = row[(int64_t)v * a.a_stride_v];
        cv = cw[v];
        bv = b[(int64_t)v * bsv];
        e0 = a.ptr[v];
        e1 = a.ptr[v + 1];
    }
    bool bad_id = false;
    int32_t len = 0;
    while (v != 0x7fffffff && len < a.max_len) {
        if (lane == 0) path[len] = v;
        ++len;
        if (pv >= (uint32_t)k) { bad_id = true; pv = 0; }
        const Tick wv = MAGIC ? (Tick)magic_div((uint32_t)cv, vtab_m[pv])
                              : (Tick)plain_div((uint64_t)cv, (uint64_t)vtab_g[pv]);
        const Tick rest = bv - wv;
        int32_t next = 0x7fffffff;          // this lane's best successor and what it fetched for it
        uint32_t n_p = 0;
        WT n_c = 0;
        Tick n_b = 0;
        int32_t n_e0 = 0, n_e1 = 0;
        for (int32_t e = e0 + lane; e < e1; e += 64) {
            const int32_t u = a.idx[e];
            const WT te = wt[e];
            const uint32_t pu_raw = row[(int64_t)u * a.a_stride_v];
            const Tick bu = b[(int64_t)u * bsv];
            const WT cu = cw[u];
            const int32_t u0 = a.ptr[u], u1 = a.ptr[u + 1];
            const uint32_t pu = min(pu_raw, (uint32_t)(k - 1));
            const Tick x = MAGIC ? (Tick)magic_div((uint32_t)te, etab_m[pv * k + pu])
                                 : (Tick)plain_div((uint64_t)te, (uint64_t)etab_g[pv * k + pu]);
            if (x + bu == rest && u < next) {
                next = u; n_p = pu_raw; n_c = cu; n_b = bu; n_e0 = u0; n_e1 = u1;
            }
        }
        int32_t best = next;
        for (int off = 32; off > 0; off >>= 1) best = min(best, __shfl_xor(best, off));
        if (best != 0x7fffffff) {
            const int from = __ffsll((long long)__ballot(next == best)) - 1;
            pv = __shfl(n_p, from);
            cv = (WT)__shfl(n_c, from);
            bv = (Tick)__shfl(n_b, from);
            e0 = __shfl(n_e0, from);
            e1 = __shfl(n_e1, from);
        }
        v = best;
    }
    if (bad_id) *a.status = CP_STATUS_BAD_DEVICE_ID;
    if (lane == 0) a.len[q] = len;
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
// Ids >= k are reported and replaced by 0.  One thread fills 16 positions.
__global__ __launch_bounds__(256) void gather_assign_kernel(const int32_t *__restrict__ gmap,
                                                            int64_t row_len,
                                                            const uint8_t *__restrict__ assign,
                                                            int64_t a_stride_p, int64_t a_stride_v,
                                                            int32_t k, uint8_t *__restrict__ out,
                                                            int32_t *status) {
    const int64_t i16 = ((int64_t)blockIdx.y * 256 + threadIdx.x) * 16;   // row_len is a multiple of 64
    if (i16 >= row_len) return;
    const int64_t q = blockIdx.x;
    const uint8_t *row = assign + q * a_stride_p;
    int4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = *(const int4 *)(gmap + i16 + 4 * j);
    uint32_t w[4];
    uint32_t worst = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t p0 = v[j].x >= 0 ? row[(int64_t)v[j].x * a_stride_v] : 0;
        uint32_t p1 = v[j].y >= 0 ? row[(int64_t)v[j].y * a_stride_v] : 0;
        uint32_t p2 = v[j].z >= 0 ? row[(int64_t)v[j].z * a_stride_v] : 0;
        uint32_t p3 = v[j].w >= 0 ? row[(int64_t)v[j].w * a_stride_v] : 0;
        const uint32_t m = max(max(p0, p1), max(p2, p3));
        if (m >= (uint32_t)k) {
            if (p0 >= (uint32_t)k) p0 = 0;
            if (p1 >= (uint32_t)k) p1 = 0;
            if (p2 >= (uint32_t)k) p2 = 0;
            if (p3 >= (uint32_t)k) p3 = 0;
        }
        worst = max(worst, m);
        w[j] = p0 | (p1 << 8) | (p2 << 16) | (p3 << 24);
    }
    if (worst >= (uint32_t)k) *status = CP_STATUS_BAD_DEVICE_ID;
    *(uint4 *)(out + q * row_len + i16) = make_uint4(w[0], w[1], w[2], w[3]);
}

// The same for rows of at most kGatherLdsRow device ids that lie one byte apart: a workgroup
// copies its partition's row into LDS once and gathers from there (64 scattered one-byte
// loads from memory per instruction are what bounds the kernel above).
constexpr int32_t kGatherLdsRow = 60 * 1024;
__global__ __launch_bounds__(256) void gather_assign_lds_kernel(const int32_t *__restrict__ gmap, int64_t row_len,
                                                                const uint8_t *__restrict__ assign,
                                                                int64_t a_stride_p, int32_t n, int32_t k,
                                                                uint8_t *__restrict__ out, int32_t *status) {
    extern __shared__ __align__(16) uint8_t ids_lds[];
    const int64_t q = blockIdx.x;
    const uint8_t *row = assign + q * a_stride_p;
    const int tid = threadIdx.x;
    if (((uintptr_t)row & 15) == 0) {
        const int32_t n16 = n / 16;
        for (int32_t i = tid; i < n16; i += 256) ((uint4 *)ids_lds)[i] = ((const uint4 *)row)[i];
        for (int32_t i = n16 * 16 + tid; i < n; i += 256) ids_lds[i] = row[i];
    } else {
        for (int32_t i = tid; i < n; i += 256) ids_lds[i] = row[i];
    }
    __syncthreads();
    uint32_t worst = 0;
    for (int64_t i16 = (int64_t)tid * 16; i16 < row_len; i16 += 256 * 16) {     // row_len is a multiple of 64
        int4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = *(const int4 *)(gmap + i16 + 4 * j);
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t p0 = v[j].x >= 0 ? ids_lds[v[j].x] : 0;
            uint32_t p1 = v[j].y >= 0 ? ids_lds[v[j].y] : 0;
            uint32_t p2 = v[j].z >= 0 ? ids_lds[v[j].z] : 0;
            uint32_t p3 = v[j].w >= 0 ? ids_lds[v[j].w] : 0;
            const uint32_t m = max(max(p0, p1), max(p2, p3));
            if (m >= (uint32_t)k) {
                if (p0 >= (uint32_t)k) p0 = 0;
                if (p1 >= (uint32_t)k) p1 = 0;
                if (p2 >= (uint32_t)k) p2 = 0;
                if (p3 >= (uint32_t)k) p3 = 0;
            }
            worst = max(worst, m);
            w[j] = p0 | (p1 << 8) | (p2 << 16) | (p3 << 24);
        }
        *(uint4 *)(out + q * row_len + i16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (worst >= (uint32_t)k) *status = CP_STATUS_BAD_DEVICE_ID;
}

struct WindowArgs {
    const uint4 *stream;       // tick packets
    const uint32_t *tick_tab;  // [L+1][4] {first chunk, chunks, lowest vertex id, id span} per tick
    const uint8_t *ids;        // direct: the caller's assignments[P][n]; else [P][L*wpad] ids in sweep order
    int64_t ids_row;           // bytes from one partition's row of `ids` to the next
    void *out;                 // [n][P] ticks, or NULL
    int64_t *cp_out;           // [P] or NULL: receives the maximum of b over the partition
    const Magic *edge_tab;
    const Magic *vert_tab;
    int32_t P, L, k, slots, wpad, smax;   // L counts ticks
    int32_t idpad;             // bytes of a stage slot set aside for device ids
    int32_t direct;            // 1: ids are staged straight from the caller's rows
    int32_t *status;
    int32_t nc, nlw;           // compute and loader wavefronts per workgroup
    int32_t pgroups;           // partitions per XCD-sized group (blockIdx -> partition map)
    int32_t out32;             // 1 if every byte offset inside a partition's outputs fits 32 bits
    int64_t out_sq;            // output index of (v, q) = v * out_sv + q * out_sq
    uint32_t out_sv;
    // t sweep that also writes the critical-vertex mask (partition-major rows only)
    const void *bvals;         // b [P][n]
    const int64_t *cp_in;      // [P]
    uint32_t *mask32;          // mask rows as 32-bit words, zeroed by the caller
    int64_t mask_row32;        // 32-bit words per mask row
    int64_t n;                 // vertices (row length of bvals)
    int32_t bpad;              // bytes a stage slot reserves for the tick's b values (0: no mask)
    // far reads: neighbours computed many ticks earlier are fetched from the output array
    const uint2 *far_list;     // [ticks][far_cap] {vertex, c}
    const uint8_t *far_assign; // caller's assignments, device of (v, q) at v * far_a_sv + q * far_a_sp
    int64_t far_a_sp, far_a_sv;
    int32_t far_cap;           // far reads per tick (multiple of 64), 0 = none
    int32_t nfw;               // far wavefronts (after the loaders)
    int32_t stores_per_tick;   // output stores one compute wavefront issues per tick
    // several partitions per workgroup (they share the cost tables in LDS)
    int32_t groups;            // partitions per workgroup
    int32_t wgs;               // workgroups that have partitions
    uint32_t sub_bytes;        // LDS of one partition: ring, far pairs, two stage slots
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // stays in registers when indexed statically
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;   // uniform reads become scalar loads

// LDS layout: per partition of the workgroup [ring][far pairs][2 stage slots], then the cost
// tables, which the partitions share; a stage slot is
// [wpad bytes of device ids][packet], NL*nlw*1024 bytes in all.  The ring is
// either (slots+1) x {value, device*8} (PACKED: one 8-byte read per relaxation, and
// an entry's ring field is the byte offset itself) or (slots+1) values followed by
// (slots+1) device bytes.
//
// Of a partition's wavefronts, 0..nc-1 compute and nc..nc+nlw-1 load.  A workgroup holds
// `groups` partitions side by side (small workgroups with large cost tables: more partitions
// per compute unit); they run tick by tick together, which costs nothing since the graph, and
// so the number of ticks, is the same for all.  Tick t: after the
// barrier the compute wavefronts relax level t out of stage slot t&1 while the
// loaders copy packet t+1 (requested DR ticks earlier, held in registers) into
// the other slot and request packet t+1+DR.  Nothing on the level-to-level
// dependency touches memory beyond LDS.
//
// `block` is the workgroup's number within its sweep (the pair kernel below runs both sweeps in
// one launch).  Wavefronts the sweep's shape does not use end at once.
template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4, int NL, int DR, bool MASK, bool FAR>
__device__ __forceinline__ void window_sweep_body(const WindowArgs &a, const uint32_t block) {
    extern __shared__ uint4 lds16[];
    __shared__ long long red[kWindowMaxWaves];
    // MASK: bits of the tick's critical vertices, by (v - (lo & ~31)) / 32; two ticks in flight
    __shared__ uint32_t mbits[MASK ? 2 : 1][MASK ? kMaskWords : 1];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wps = a.nc + a.nlw + a.nfw;                 // wavefronts of one partition
    const int nt = a.groups * wps * 64;                   // threads at work
    if (tid >= nt) return;                                // (whole wavefronts, before any barrier)
    // which of the workgroup's partitions (the variant that writes the mask runs one per
    // workgroup: its addresses stay compile-time constants)
    const int sub = MASK ? 0 : wave_all / wps;
    const int wave = wave_all - sub * wps;                // role index inside it
    uint8_t *lds = (uint8_t *)lds16 + (size_t)sub * a.sub_bytes;
    const int k = a.k, L = a.L, R = a.slots;

    // blockIdx -> partition: blocks are dealt round-robin to the 8 XCDs; give each
    // XCD a run of consecutive partitions so that the 4-byte stores of one output
    // line meet in one L2
    const int32_t wg = (int32_t)(block % 8) * a.pgroups + (int32_t)(block / 8);
    if (wg >= a.wgs) return;   // whole workgroup: no barrier has been reached yet
    // a last workgroup that is not full repeats its last partition (same values to the same
    // places) so that every wavefront meets every barrier
    const int32_t q = min(wg * a.groups + sub, a.P - 1);

    const uint32_t ring_bytes = (uint32_t)((((size_t)R + 1) * (PACKED ? 8 : sizeof(Tick) + 1) + 15) & ~(size_t)15);
    const uint32_t tab_bytes = (uint32_t)((sizeof(Magic) * ((size_t)k * k + k) + 15) & ~(size_t)15);
    Tick *ring_val = (Tick *)lds;                                  // split layout
    uint8_t *ring_dev = lds + sizeof(Tick) * ((size_t)R + 1);
    const uint32_t far_bytes = FAR ? 8u * (uint32_t)a.far_cap : 0u;   // per tick parity, behind the ring
    // byte offsets from this partition's LDS: the shared tables lie behind the last partition
    const uint32_t etab_off = (uint32_t)(a.groups - sub) * a.sub_bytes;
    const uint32_t vtab_off = etab_off + 8u * (uint32_t)(k * k);
    const int slot_bytes = NL * a.nlw * 1024;
    uint8_t *stage = lds + ring_bytes + 2u * far_bytes;
    (void)tab_bytes;
    {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
        uint64_t *t64 = (uint64_t *)(lds + etab_off);
        for (int i = tid; i < k * k; i += nt) t64[i] = e[i];
        for (int i = tid; i < k; i += nt) t64[k * k + i] = v[i];
        if constexpr (MASK)
            for (int i = tid; i < 2 * kMaskWords; i += nt) (&mbits[0][0])[i] = 0;
        if (wave == 0 && lane == 0) {        // the constant-zero slot padding entries point at
            if (PACKED) {
                ((uint2 *)lds)[R] = make_uint2(0, 0);
            } else {
                ring_val[R] = 0;
                ring_dev[R] = 0;
            }
        }
    }

    // ticks rounded up so that the loaders' and the far wavefronts' unrolled loops end together
    constexpr int kStep = !FAR ? DR : (DR % kWindowFarLead == 0 ? DR : DR * kWindowFarLead / (DR % 2 == 0 ? 2 : 1));
    static_assert(kStep % DR == 0 && (!FAR || kStep % kWindowFarLead == 0), "tick padding");
    const int Lpad = (L + kStep - 1) / kStep * kStep;
    const int id16 = a.idpad / 16;               // 16-byte chunks of a slot that hold device ids
    const int b16 = MASK ? a.bpad / 16 : 0;      // ... and the tick's b values
    const int head = a.idpad + (MASK ? a.bpad : 0);   // bytes of a slot before the packet
    Tick best = 0;

    if (FAR && wave >= a.nc + a.nlw) {
        // ------------------------------------------------ far wavefronts
        // Lane f of far wavefront fw owns far read number fw*64 + f of every tick.  For tick
        // tau its {vertex, c} is loaded 2*X + 1 steps ahead, the value and device of that vertex
        // X + 1 steps ahead (from the output array: the vertex was published at least
        // kWindowFarTicks ticks before tau, and the compute wavefronts wait for their older
        // stores before each barrier), and the pair is written one step ahead.
        constexpr int X = kWindowFarLead;
        const int f = (wave - a.nc - a.nlw) * 64 + lane;
        const Tick *outq = (const Tick *)a.out + (size_t)q * (size_t)a.out_sq;
        const uint8_t *arow = a.far_assign + (size_t)q * (size_t)a.far_a_sp;
        const Magic *vtab = (const Magic *)(lds + vtab_off);
        bool bad = false;
        auto list_load = [&](int tau) -> uint2 {
            return a.far_list[(size_t)min(tau, L - 1) * (size_t)a.far_cap + f];
        };
        auto fetch = [&](uint2 e) -> uint2 {
            // the value left this compute unit through its write-through cache: read it from L2
            Tick val = __hip_atomic_load(outq + (size_t)e.x * a.out_sv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint32_t dev = arow[(size_t)e.x * (size_t)a.far_a_sv];
            if (dev >= (uint32_t)k) { bad = true; dev = (uint32_t)k - 1; }
            if (TSWEEP) val += (Tick)magic_div(e.y, vtab[dev]);      // the ring holds tl + w
            return make_uint2((uint32_t)val, 8u * dev);
        };
        uint2 lst[X], got[X];
#pragma unroll
        for (int j = 1; j <= X; ++j) {
            lst[j % X] = list_load(j + X);
            got[j % X] = make_uint2(0, 0);
        }
        lds_barrier();                       // pairs with "packet 0 is staged"
        for (int t0 = 0; t0 < Lpad; t0 += X) {
#pragma unroll
            for (int r = 0; r < X; ++r) {
                const int t = t0 + r;
                lds_barrier();
                const int sl = (r + 1) % X;
                *(uint2 *)(lds + ring_bytes + (uint32_t)((t + 1) & 1) * far_bytes + 8u * (uint32_t)f) = got[sl];
                got[sl] = fetch(lst[sl]);                 // for tick t + 1 + X
                lst[sl] = list_load(t + 1 + 2 * X);
            }
        }
        if (MASK) lds_barrier();
        if (bad) *a.status = CP_STATUS_BAD_DEVICE_ID;
    } else if (wave >= a.nc) {
        // ------------------------------------------------ loader wavefronts
        const int lw = wave - a.nc;
        const_u32_ptr tick_tab = (const_u32_ptr)a.tick_tab;
        // chunk ids of this lane are fixed; whether one is a device-id chunk (the first
        // id16 of a slot) or a packet chunk is therefore fixed too
        int cid[NL];
        const uint4 *base[NL];
        bool is_id[NL], is_b[NL];
        const uint8_t *row = a.ids + (size_t)q * a.ids_row;
        // direct staging starts at the 16-byte boundary below the tick's lowest id
        const uint32_t row_mis = (uint32_t)((uintptr_t)row & 15);
        const uint8_t *brow = MASK ? (const uint8_t *)a.bvals + (size_t)q * (size_t)a.n * sizeof(Tick) : nullptr;
        const uint32_t brow_mis = (uint32_t)((uintptr_t)brow & 15);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            cid[i] = (i * a.nlw + lw) * 64 + lane;
            is_id[i] = cid[i] < id16;
            is_b[i] = MASK && !is_id[i] && cid[i] < id16 + b16;
            base[i] = is_id[i] ? (const uint4 *)(row - row_mis)
                               : (is_b[i] ? (const uint4 *)(brow - brow_mis) : a.stream);
        }
        u32x4 buf[DR][NL];
        // every lane always loads: chunks past the end of the ids or of the packet re-read
        // the last chunk of that part
#define CP_ISSUE(R_, S_)                                                                        \
    do {                                                                                        \
        const int s_ = min((S_), L - 1);                                                        \
        const u32x4 tt_ = *(const u32x4 __attribute__((address_space(4))) *)(tick_tab + 4 * s_); \
        const uint32_t o0_ = tt_.x, oc_ = tt_.y, lo_ = tt_.z, span_ = tt_.w;                    \
        int id_first_, id_last_;                                                                \
        if (a.direct) {                                                                         \
            id_first_ = (int)((row_mis + lo_) >> 4);                                            \
            id_last_ = (int)((row_mis + lo_ + span_ - 1) >> 4) - id_first_;                     \
        } else {                                                                                \
            id_first_ = s_ * (a.wpad / 16);                                                     \
            id_last_ = a.wpad / 16 - 1;                                                         \
        }                                                                                       \
        const int pk_last_ = id16 + b16 + (int)oc_ - 1, off_pk_ = (int)o0_ - id16 - b16;        \
        int b_first_ = 0, b_last_ = 0;                                                          \
        if (MASK) {                                                                             \
            b_first_ = (int)((brow_mis + (uint32_t)sizeof(Tick) * lo_) >> 4);                   \
            b_last_ = (int)((brow_mis + (uint32_t)sizeof(Tick) * (lo_ + span_) - 1) >> 4) - b_first_; \
        }                                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                     \
            int c_ = is_id[i_] ? min(cid[i_], id_last_) + id_first_                             \
                               : min(cid[i_], pk_last_) + off_pk_;                              \
            if (MASK && is_b[i_]) c_ = min(cid[i_] - id16, b_last_) + b_first_;                 \
            buf[R_][i_] = *(const u32x4 *)(base[i_] + c_);                                      \
        }                                                                                       \
    } while (0)
#define CP_STORE(R_, SLOT_)                                                                     \
    do {                                                                                        \
        u32x4 *dst_ = (u32x4 *)(stage + (size_t)(SLOT_) * slot_bytes);                          \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) dst_[cid[i_]] = buf[R_][i_];          \
    } while (0)
        // the critical vertices of tick s, collected in LDS while it ran, go to the mask row
        auto flush_mask = [&](int s_) {
            const u32x4 tt = *(const u32x4 __attribute__((address_space(4))) *)(tick_tab + 4 * s_);
            const uint32_t lo = tt.z, span = tt.w;
            const int words = (int)(((lo & 31u) + span + 31u) >> 5);
            uint32_t *dst = a.mask32 + (size_t)q * (size_t)a.mask_row32 + (lo >> 5);
            for (int w = lane; w < words; w += 64) {
                const uint32_t bits = mbits[MASK ? (s_ & 1) : 0][MASK ? w : 0];
                if (bits) {
                    atomicOr(dst + w, bits);
                    mbits[MASK ? (s_ & 1) : 0][MASK ? w : 0] = 0;
                }
            }
        };
        (void)flush_mask;
#pragma unroll
        for (int r = 0; r < DR; ++r) CP_ISSUE(r, r);
        CP_STORE(0, 0);
        CP_ISSUE(0, DR);
        lds_barrier();                       // packet 0 is staged
        for (int t0 = 0; t0 < Lpad; t0 += DR) {
#pragma unroll
            for (int r = 0; r < DR; ++r) {
                const int t = t0 + r;
                lds_barrier();
                // the compute wavefronts now read slot t&1, which packet t-1 has left
                CP_STORE((r + 1) % DR, (t + 1) & 1);
                CP_ISSUE((r + 1) % DR, t + 1 + DR);
                if (MASK && lw == 0 && t >= 1 && t <= L) flush_mask(t - 1);
            }
        }
        if (MASK) {
            lds_barrier();                   // the last tick's bits are set
            if (lw == 0 && Lpad == L) flush_mask(L - 1);
        }
#undef CP_ISSUE
#undef CP_STORE
    } else {
        // ------------------------------------------------ compute wavefronts
        // They carry the sweep's critical chain (LDS round trips per relaxation); the loaders
        // only have to stay a few ticks ahead.  Issue priority over the loaders and far
        // wavefronts: 4 % off the b sweep of the large sparse workload.
        __builtin_amdgcn_s_setprio(1);
        typedef typename std::conditional<ENT4, uint32_t, uint2>::type Ent;
        Tick *out = a.out ? (Tick *)a.out + (size_t)q * (size_t)a.out_sq : nullptr;
        const uint32_t out_sv = a.out_sv;
        const uint32_t k8 = 8u * (uint32_t)k;
        const uint32_t rec_off = (uint32_t)head + 16u * (uint32_t)a.smax;   // records, from the slot base
        const uint32_t brow_mis = MASK ? (uint32_t)(((uintptr_t)a.bvals + (size_t)q * (size_t)a.n * sizeof(Tick)) & 15)
                                       : 0u;
        const Tick cpq = MASK ? (Tick)a.cp_in[q] : 0;     // tl + b <= CP: no overflow in Tick
        int cur_tick = 0;
        const uint32_t row_mis = (uint32_t)((uintptr_t)(a.ids + (size_t)q * a.ids_row) & 15);
        uint32_t worst = 0;                  // largest device id seen

        auto ent_field = [](Ent e) -> uint32_t {
            if constexpr (ENT4) return e & 0xffffu; else return e.x;
        };
        auto ent_t = [](Ent e) -> uint32_t {
            if constexpr (ENT4) return e >> 16; else return e.y;
        };
        // value and 8 * device of the vertex behind ring field f
        auto ring_get = [&](uint32_t f, Tick &vu, uint32_t &pu8) {
            if constexpr (PACKED) {
                const uint2 x = *(const uint2 *)(lds + f);
                vu = (Tick)x.x;
                pu8 = x.y;
            } else {
                vu = ring_val[f];
                pu8 = 8u * ring_dev[f];
            }
        };
        // fold the lanes of a row; afterwards the row's first lane holds the row's maximum
        auto fold = [&](Tick acc, int lsh) -> Tick {
            if (lsh == 0) return acc;
            if (lsh >= 1) acc = max(acc, __shfl_xor(acc, 1));
            if (lsh >= 2) acc = max(acc, __shfl_xor(acc, 2));
            if (lsh >= 3) acc = max(acc, __shfl_xor(acc, 4));
            if (lsh >= 4) acc = max(acc, __shfl_xor(acc, 8));
            if (lsh >= 5) acc = max(acc, __shfl_xor(acc, 16));
            if (lsh >= 6) acc = max(acc, __shfl_xor(acc, 32));
            return acc;
        };
        // the row's first lane publishes the vertex: ring, output, running maximum
        auto publish = [&](Tick acc, Tick w, int lsh, int rows, int rbase, uint32_t v, uint32_t pv, Tick bv,
                           uint32_t lo) {
            const int row = lane >> lsh;
            const bool first = lsh == 0 || (lane & ((1 << lsh) - 1)) == 0;
            if (row < rows && first) {
                const Tick fin = acc + w;            // b(v), or tl(v) + w(v)
                int rs = rbase + row;
                if (rs >= R) rs -= R;
                if constexpr (PACKED) {
                    ((uint2 *)lds)[rs] = make_uint2((uint32_t)fin, 8u * pv);
                } else {
                    ring_val[rs] = fin;
                    ring_dev[rs] = (uint8_t)pv;
                }
                if (out) {
                    // (a 32-bit byte offset beside the row's uniform address where that fits)
                    if (a.out32) *(Tick *)((char *)out + __umul24(v, out_sv) * (uint32_t)sizeof(Tick)) = TSWEEP ? acc : fin;
                    else out[(size_t)v * out_sv] = TSWEEP ? acc : fin;
                }
                best = max(best, fin);
                if constexpr (MASK) {        // tl(v) + b(v) = CP marks a critical vertex
                    if ((Tick)(acc + bv) == cpq) {
                        const uint32_t rel = v - (lo & ~31u);
                        atomicOr(&mbits[cur_tick & 1][rel >> 5], 1u << (rel & 31u));
                    }
                }
            }
        };
        // one slice of the current level out of its stage slot
        auto slice_direct = [&](const uint8_t *st, int j) {
            // the descriptor is the same for all lanes; only what steers control flow
            // (width, lanes per row) is moved to scalars, the rest stays in vector registers
            const uint4 d = ((const uint4 *)(st + head))[j];
            const uint32_t ent_off = d.x;
            const int width = __builtin_amdgcn_readfirstlane((int)(d.y & 0xffffu));
            const int lsh = __builtin_amdgcn_readfirstlane((int)(d.y >> 24));
            const int rows = (int)((d.y >> 16) & 0xffu);
            const uint32_t lo = d.z;
            const int rbase = (int)d.w;
            if (width == 0 && lsh == 0 && __builtin_amdgcn_readfirstlane(rows) == 0) return;
            const int p = j * 64 + (lane >> lsh);
            const uint2 *rec = (const uint2 *)(st + rec_off) + p;
            const Ent *ent = (const Ent *)(st + head + ent_off) + lane;
            const uint32_t id_bias = a.direct ? ((row_mis + lo) & 15u) - lo : 0u;
            uint2 rc;
            uint32_t pv;
            Magic mv;
            Tick acc = 0, bv = 0;
            // byte (v - lo) * sizeof(Tick) of the staged b range, which starts at a 16-byte boundary
            const uint32_t b_bias = ((brow_mis + (uint32_t)sizeof(Tick) * lo) & 15u) - (uint32_t)sizeof(Tick) * lo;
            // The vertex's own reads (record, then its device id, then its cost-table entry)
            // and the first N relaxations (entries, then ring, then transfer-table entries)
            // are two chains of three dependent LDS reads; issued side by side they cost
            // three round trips together.  Device id: position p of the gathered row, or
            // byte (v - lo) of the staged id range (padding rows carry v = lo, so every lane
            // reads a byte that was staged); it is checked against k once, after the sweep.
#define CP_HEAD(N)                                                                              \
    do {                                                                                        \
        Ent en_[N + 1];                                                                         \
        Tick vu_[N + 1];                                                                        \
        uint32_t pu8_[N + 1];                                                                   \
        Magic mg_[N + 1];                                                                       \
        rc = *rec;                                                                              \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) en_[i_] = ent[i_ * 64];                \
        pv = st[a.direct ? rc.x + id_bias : (uint32_t)p];                                       \
        if (MASK) bv = *(const Tick *)(st + a.idpad + (uint32_t)sizeof(Tick) * rc.x + b_bias);  \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) ring_get(ent_field(en_[i_]), vu_[i_], pu8_[i_]); \
        worst = max(worst, pv);                                                                 \
        pv = min(pv, (uint32_t)(k - 1));                                                        \
        erow = etab_off + __umul24(pv, k8);                                                     \
        mv = *(const Magic *)(lds + vtab_off + 8u * pv);                                        \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) mg_[i_] = *(const Magic *)(lds + erow + pu8_[i_]); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_)                                        \
            acc = max(acc, (Tick)(vu_[i_] + (Tick)magic_div(ent_t(en_[i_]), mg_[i_])));         \
    } while (0)
            // N further relaxations as one straight-line block: N entry reads, N ring reads,
            // N cost-table reads, then the arithmetic -- three LDS round trips whatever N is
#define CP_BLOCK(N)                                                                             \
    do {                                                                                        \
        Ent en_[N];                                                                             \
        Tick vu_[N];                                                                            \
        uint32_t pu8_[N];                                                                       \
        Magic mg_[N];                                                                           \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) en_[i_] = ent[(jj + i_) * 64];         \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) ring_get(ent_field(en_[i_]), vu_[i_], pu8_[i_]); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) mg_[i_] = *(const Magic *)(lds + erow + pu8_[i_]); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_)                                        \
            acc = max(acc, (Tick)(vu_[i_] + (Tick)magic_div(ent_t(en_[i_]), mg_[i_])));         \
    } while (0)
            uint32_t erow;
            switch (min(width, 8)) {
                case 0: CP_HEAD(0); break;
                case 1: CP_HEAD(1); break;
                case 2: CP_HEAD(2); break;
                case 3: CP_HEAD(3); break;
                case 4: CP_HEAD(4); break;
                case 5: CP_HEAD(5); break;
                case 6: CP_HEAD(6); break;
                case 7: CP_HEAD(7); break;
                default: CP_HEAD(8); break;
            }
            int jj = 8;
            for (; jj + 8 <= width; jj += 8) CP_BLOCK(8);
            switch (width - jj) {
                case 1: CP_BLOCK(1); break;
                case 2: CP_BLOCK(2); break;
                case 3: CP_BLOCK(3); break;
                case 4: CP_BLOCK(4); break;
                case 5: CP_BLOCK(5); break;
                case 6: CP_BLOCK(6); break;
                case 7: CP_BLOCK(7); break;
                default: break;
            }
#undef CP_BLOCK
#undef CP_HEAD
            acc = fold(acc, lsh);
            publish(acc, (Tick)magic_div(rc.y, mv), lsh, rows, rbase, rc.x, pv, bv, lo);
        };

        lds_barrier();                       // packet 0 is staged
        for (int t = 0; t < Lpad; ++t) {
            if constexpr (FAR) {
                // far reads take values from the output array kWindowFarTicks ticks later:
                // keep at most two ticks' worth of stores in flight
                if (a.stores_per_tick == 1) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                else if (a.stores_per_tick == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            lds_barrier();
            if (t >= L) continue;
            cur_tick = t;
            const uint8_t *st = stage + (size_t)(t & 1) * slot_bytes;
            for (int j = wave; j < a.smax; j += a.nc) slice_direct(st, j);
        }
        if (worst >= (uint32_t)k) *a.status = CP_STATUS_BAD_DEVICE_ID;
        if (MASK) lds_barrier();             // pairs with the loaders' barrier before the last flush
    }

    if (a.cp_out) {   // the partition's maximum
        long long b64 = (long long)best;
        for (int off = 32; off > 0; off >>= 1) b64 = max(b64, __shfl_xor(b64, off));
        if (lane == 0) red[wave_all] = b64;
        lds_barrier();
        if (wave == 0 && lane == 0) {
            for (int w2 = 1; w2 < a.nc; ++w2) b64 = max(b64, red[sub * wps + w2]);
            a.cp_out[q] = b64;
        }
    }
}

template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4, int NL, int DR, bool MASK, bool FAR>
__global__ __launch_bounds__(kWindowMaxWaves * 64) void window_sweep_kernel(WindowArgs a) {
    window_sweep_body<Tick, TSWEEP, PACKED, ENT4, NL, DR, MASK, FAR>(a, blockIdx.x);
}

// Both sweeps in one launch: even workgroups run the b-level sweep, odd ones the t-level sweep
// (nb of each).  A sweep of one workgroup per compute unit leaves the unit's LDS pipe and vector ALUs
// more than half idle (its tick is a chain of dependent steps); the two sweeps are independent,
// and a workgroup of each fits a unit side by side when they are shaped for it: 4 loads per
// loader lane held for 2 ticks (64 registers per lane in all, so eight wavefronts fit a SIMD)
// and at most 16 wavefronts and half the LDS each.  Large sparse workload, 256 partitions:
// 2.07 ms for both sweeps against 1.47 + 1.75 ms one after the other.
constexpr int kPairNl = 4, kPairDr = 2;
template <bool ENT4>
__global__ __launch_bounds__(kWindowMaxWaves * 64) void window_pair_kernel(WindowArgs ab, WindowArgs at, uint32_t nb) {
    (void)nb;
    if ((blockIdx.x & 1) == 0) window_sweep_body<int32_t, false, true, ENT4, kPairNl, kPairDr, false, false>(ab, blockIdx.x >> 1);
    else window_sweep_body<int32_t, true, true, ENT4, kPairNl, kPairDr, false, false>(at, blockIdx.x >> 1);
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
    a.idx = (const int32_t *)(s.blob + dir.idx_off);
    a.wt = s.blob + dir.wt_off;
    a.c = s.blob + s.c_off;
    a.pT = s.pT;
    a.val = s.val;
    a.edge_tab = s.edge_tab;
    a.vert_tab = s.vert_tab;
    a.status = s.status;
    a.P = s.P; a.ncol = ncol; a.k = s.k;
    const int4 *rows = (const int4 *)(s.blob + dir.rows_off);
    int32_t count = 0;
    for (int l = 0; l < L; ++l) {
        const int32_t hubs = dir.lvl_hubs[l], total = dir.lvl_count[l];
        if (hubs > 0) {
            a.rows = rows + dir.lvl_begin[l];
            a.count = hubs;
            const int64_t blocks = (int64_t)hubs * ncol;
            const size_t lds_bytes = tab_bytes + sizeof(Tick) * 64 * kHubWaves;
            hipLaunchKernelGGL((column_level_kernel<Tick, WT, MAGIC, TSWEEP, true>),
                               dim3((unsigned)blocks), dim3(kHubWaves * 64), lds_bytes, st, a);
            ++count;
        }
        if (total > hubs) {
            a.rows = rows + dir.lvl_begin[l] + hubs;
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

// What both forms of launch hand the kernel for one sweep (no mask, no far reads).
WindowArgs window_args(const SweepLaunch &s, const WindowCfg &cfg) {
    const WindowDir &dir = *s.win;
    WindowArgs a{};
    a.stream = (const uint4 *)(s.blob + dir.stream_off);
    a.tick_tab = (const uint32_t *)(s.blob + dir.tick_off);
    a.direct = s.direct_ids ? 1 : 0;
    a.ids = s.direct_ids ? s.assign : s.pperm;
    a.ids_row = s.direct_ids ? s.a_stride_p : (int64_t)dir.ticks * dir.wpad;
    a.idpad = dir.idpad;
    a.status = s.status;
    a.out = s.val;
    a.cp_out = s.cp_out;
    a.edge_tab = (const Magic *)s.edge_tab;
    a.vert_tab = (const Magic *)s.vert_tab;
    a.P = s.P; a.L = dir.ticks; a.k = s.k; a.slots = dir.slots; a.wpad = dir.wpad; a.smax = dir.smax;
    a.nc = cfg.nc; a.nlw = cfg.nlw;
    // every byte offset of a vertex inside a partition's row of outputs fits 32 bits (and both factors 24)
    a.out32 = s.n < (1 << 24) && s.out_sv < (1 << 24) &&
              (uint64_t)s.n * (uint64_t)s.out_sv * (uint64_t)s.tick_bytes < (1ull << 32);
    a.out_sq = s.out_sq;
    a.out_sv = (uint32_t)s.out_sv;
    a.groups = std::max(1, cfg.groups);
    a.wgs = (s.P + a.groups - 1) / a.groups;
    a.pgroups = (a.wgs + 7) / 8;
    a.sub_bytes = (uint32_t)cfg.sub_bytes;
    a.nfw = 0;
    return a;
}

template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4, int NL, int DR, bool MASK, bool FAR>
int launch_window_sweep_k(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    const WindowDir &dir = *s.win;
    WindowArgs a = window_args(s, cfg);
    if (MASK) {
        a.bvals = s.mask_b;
        a.cp_in = s.mask_cp;
        a.mask32 = (uint32_t *)s.mask_out;
        a.mask_row32 = 2 * (((int64_t)s.n + 63) / 64);
        a.n = s.n;
        a.bpad = window_mask_bpad(dir);
    }
    if (FAR) {
        if (!s.val) return CP_ERR_ARG;       // far reads come out of the output array
        a.far_list = (const uint2 *)(s.blob + dir.far_off);
        a.far_assign = s.assign;
        a.far_a_sp = s.a_stride_p;
        a.far_a_sv = s.a_stride_v;
        a.far_cap = dir.far_cap;
        a.nfw = cfg.nfw;
        a.stores_per_tick = (dir.smax + cfg.nc - 1) / cfg.nc;
    }
    auto kern = window_sweep_kernel<Tick, TSWEEP, PACKED, ENT4, NL, DR, MASK, FAR>;
    if (cfg.lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)cfg.lds_bytes);
        if (e != hipSuccess) return CP_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * a.pgroups)),
                       dim3(a.groups * (cfg.nc + cfg.nlw + (FAR ? cfg.nfw : 0)) * 64), cfg.lds_bytes, st, a);
    return hip_ok(hipGetLastError());
}

template <typename Tick, bool TSWEEP, bool PACKED, bool ENT4, bool MASK, bool FAR>
int launch_window_sweep_e(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    switch (cfg.nl) {   // loads per loader lane per level x levels in flight: 64 registers at most
        case 1: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 1, 8, MASK, FAR>(s, cfg, st);
        case 2: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 2, 8, MASK, FAR>(s, cfg, st);
        case 3: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 3, 5, MASK, FAR>(s, cfg, st);
        case 4: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 4, 4, MASK, FAR>(s, cfg, st);
        case 8: return launch_window_sweep_k<Tick, TSWEEP, PACKED, ENT4, 8, 2, MASK, FAR>(s, cfg, st);
        default: return CP_ERR_ARG;
    }
}

template <typename Tick, bool TSWEEP, bool PACKED, bool MASK, bool FAR = false>
int launch_window_sweep_p(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    return s.win->ent4 ? launch_window_sweep_e<Tick, TSWEEP, PACKED, true, MASK, FAR>(s, cfg, st)
                       : launch_window_sweep_e<Tick, TSWEEP, PACKED, false, MASK, FAR>(s, cfg, st);
}

template <bool TSWEEP>
int launch_window_sweep_d(const SweepLaunch &s, const WindowCfg &cfg, hipStream_t st) {
    if (s.mask_out) {    // the t sweep that also writes the mask: 32-bit ticks in a packed ring only
        if (!TSWEEP || s.tick_bytes != 4 || !s.win->packed || !s.direct_ids) return CP_ERR_ARG;
        return launch_window_sweep_p<int32_t, true, true, true>(s, cfg, st);
    }
    if (s.win->far_cap > 0) {   // far reads exist only beside a packed ring of 32-bit ticks
        if (s.tick_bytes != 4 || !s.win->packed) return CP_ERR_ARG;
        return launch_window_sweep_p<int32_t, TSWEEP, true, false, true>(s, cfg, st);
    }
    if (s.tick_bytes == 4)
        return s.win->packed ? launch_window_sweep_p<int32_t, TSWEEP, true, false>(s, cfg, st)
                             : launch_window_sweep_p<int32_t, TSWEEP, false, false>(s, cfg, st);
    if (s.win->packed) return CP_ERR_ARG;      // packed rings hold 32-bit ticks only
    return launch_window_sweep_p<int64_t, TSWEEP, false, false>(s, cfg, st);
}

}  // namespace

int32_t window_mask_bpad(const WindowDir &d) { return 4 * d.idpad + 16; }

bool window_config(const WindowDir &d, int32_t k, size_t tick_bytes, size_t lds_limit, WindowCfg &out,
                   bool with_mask) {
    if (d.packed && tick_bytes != 4) return false;
    if (with_mask && d.far_cap > 0) return false;
    // the mask variant's static LDS: the bits of two ticks
    const size_t mask_static = with_mask ? (size_t)2 * kMaskWords * 4 : 0;
    if (lds_limit <= mask_static) return false;
    lds_limit -= mask_static;
    const int nfw = d.far_cap / kWave;                  // far wavefronts, 64 far reads per tick each
    // a tick's id range may touch (31 + span + 31) / 32 mask words
    if (with_mask && (!d.packed || !d.direct_ok || (d.idpad + 62) / 32 > kMaskWords)) return false;
    // 16-byte chunks per stage slot: device ids, the tick's b values (mask), the packet
    const int64_t need = d.idpad / 16 + (with_mask ? window_mask_bpad(d) / 16 : 0) + (int64_t)d.max_chunks;
    const size_t tab = (sizeof(Magic) * ((size_t)k * k + k) + 15) & ~(size_t)15;
    const size_t ring = ((((size_t)d.slots + 1) * (d.packed ? 8 : tick_bytes + 1) + 15) & ~(size_t)15) +
                        2 * 8 * (size_t)d.far_cap;      // the far pairs of two ticks sit behind the ring
    static const int kNl[5] = {1, 2, 3, 4, 8};
    bool found = false;
    for (int nl : kNl) {
        const int64_t nlw = (need + 64 * nl - 1) / (64 * nl);
        if (nlw > 8 || nlw + nfw > kWindowMaxWaves - 1) continue;
        WindowCfg c;
        c.nl = nl;
        c.nlw = (int)nlw;
        c.nfw = nfw;
        c.dr = nl <= 2 ? 8 : (nl == 3 ? 5 : (nl == 4 ? 4 : 2));
        c.nc = std::max(1, std::min(d.smax, kWindowMaxWaves - (int)nlw - nfw));
        c.packed = d.packed;
        c.sub_bytes = ring + (size_t)2 * nl * nlw * 1024;
        c.groups = 1;
        c.lds_bytes = c.sub_bytes + tab;
        if (c.lds_bytes > lds_limit) continue;
        // The first shape that fits (most ticks of prefetch) is the one for a workgroup that
        // fills a compute unit.  A small workgroup shares the unit with others: there fewer
        // wavefronts per workgroup mean more workgroups, as long as the loaders still run
        // four ticks ahead.
        if (!found) {
            out = c;
            found = true;
            if (c.lds_bytes > 40 * 1024) break;
        } else if (c.lds_bytes <= 40 * 1024 && c.dr >= 4 && c.nc + c.nlw + c.nfw < out.nc + out.nlw + out.nfw) {
            out = c;
        }
    }
    if (!found) return false;
    // Several partitions per workgroup share one copy of the cost tables.  That pays when the
    // tables are a large part of a small workgroup's LDS (many devices, a narrow graph): more
    // partitions fit a compute unit.  Taken when it raises that number by a quarter or more
    // (never by the variant that writes the mask, which is for wide ticks).
    const int wps = out.nc + out.nlw + out.nfw;
    auto per_cu = [&](int g) {
        const size_t lds = (size_t)g * out.sub_bytes + tab + mask_static + 512;
        const size_t by_lds = kLdsBudget / lds, by_waves = (size_t)(32 / (g * wps));
        return (size_t)g * std::min(by_lds, by_waves);
    };
    size_t best = per_cu(1);
    for (int g = 2; !with_mask && g <= kWindowMaxGroups && g * wps <= kWindowMaxWaves; g *= 2) {
        if ((size_t)g * out.sub_bytes + tab > lds_limit) break;
        const size_t here = per_cu(g);
        if (4 * here >= 5 * best) {
            best = here;
            out.groups = g;
        }
    }
    out.lds_bytes = (size_t)out.groups * out.sub_bytes + tab;
    return true;
}

int launch_gather_assign(const SweepLaunch &s, uint8_t *out, void *stream) {
    const WindowDir &dir = *s.win;
    const int64_t row_len = (int64_t)dir.ticks * dir.wpad;
    if (s.a_stride_v == 1 && s.n <= kGatherLdsRow) {
        hipLaunchKernelGGL(gather_assign_lds_kernel, dim3((unsigned)s.P), dim3(256), (size_t)((s.n + 15) & ~15),
                           (hipStream_t)stream, (const int32_t *)(s.blob + dir.gmap_off), row_len, s.assign,
                           s.a_stride_p, s.n, s.k, out, s.status);
        return hip_ok(hipGetLastError());
    }
    const int64_t chunks = (row_len + 4095) / 4096;
    if (chunks > 65535) return CP_ERR_SIZE;
    hipLaunchKernelGGL(gather_assign_kernel, dim3((unsigned)s.P, (unsigned)chunks), dim3(256), 0,
                       (hipStream_t)stream, (const int32_t *)(s.blob + dir.gmap_off), row_len,
                       s.assign, s.a_stride_p, s.a_stride_v, s.k, out, s.status);
    return hip_ok(hipGetLastError());
}

int launch_clear(int64_t *cp_out, int32_t batch, int32_t *status, void *stream) {
    hipLaunchKernelGGL(clear_kernel, dim3((batch + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       cp_out, batch, status);
    return hip_ok(hipGetLastError());
}

int launch_zero_bytes(uint8_t *dst, int64_t bytes, void *stream) {
    if (bytes <= 0) return CP_OK;
    hipLaunchKernelGGL(zero_bytes_kernel, dim3((unsigned)((bytes + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, dst, bytes);
    return hip_ok(hipGetLastError());
}

int launch_zero_words(uint64_t *dst, int64_t words, void *stream) {
    if (words <= 0) return CP_OK;
    const unsigned blocks = (unsigned)std::min<int64_t>((words + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(zero_words_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, dst, words);
    return hip_ok(hipGetLastError());
}

int launch_ranks(const void *b, const void *tl, const void *c, bool narrow, int tick_bytes, int32_t n,
                 int64_t *up, int64_t *down, int64_t *total, void *stream) {
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipStream_t st = (hipStream_t)stream;
#define CP_RANKS(TICK, WT)                                                                         \
    hipLaunchKernelGGL((ranks_kernel<TICK, WT>), grid, block, 0, st, (const TICK *)b, (const TICK *)tl, \
                       (const WT *)c, n, up, down, total)
    if (tick_bytes == 4) {
        if (narrow) CP_RANKS(int32_t, uint32_t); else CP_RANKS(int32_t, int64_t);
    } else {
        if (narrow) CP_RANKS(int64_t, uint32_t); else CP_RANKS(int64_t, int64_t);
    }
#undef CP_RANKS
    return hip_ok(hipGetLastError());
}

int launch_transpose(const uint8_t *in, uint8_t *out, int32_t n, int32_t P, void *stream) {
    if (n % 4 == 0 && P % 4 == 0 && ((uintptr_t)in & 3) == 0 && ((uintptr_t)out & 3) == 0) {
        const dim3 grid4((unsigned)((n + 255) / 256), (unsigned)((P + 63) / 64));
        hipLaunchKernelGGL(transpose4_kernel, grid4, dim3(256), 0, (hipStream_t)stream, in, out, n, P);
        return hip_ok(hipGetLastError());
    }
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

// Shapes for the two sweeps of one graph run side by side by window_pair_kernel, or false where
// that form does not apply: packed rings of 32-bit ticks, no far reads, the same entry format
// both ways, and a workgroup of each within one compute unit's LDS and wavefront slots.
bool window_pair_config(const WindowDir &db, const WindowDir &dt, int32_t k, size_t lds_limit, WindowCfg &out_b,
                        WindowCfg &out_t) {
    if (!db.packed || !dt.packed || db.far_cap > 0 || dt.far_cap > 0 || db.ent4 != dt.ent4) return false;
    const size_t tab = (sizeof(Magic) * ((size_t)k * k + k) + 15) & ~(size_t)15;
    auto shape = [&](const WindowDir &d, WindowCfg &c) {
        const int64_t need = d.idpad / 16 + (int64_t)d.max_chunks;
        const int64_t nlw = (need + 64 * kPairNl - 1) / (64 * kPairNl);
        if (nlw > 8) return false;
        const size_t ring = ((((size_t)d.slots + 1) * 8 + 15) & ~(size_t)15);
        c = WindowCfg{};
        c.nl = kPairNl;
        c.nlw = (int)nlw;
        c.nfw = 0;
        c.dr = kPairDr;
        c.nc = std::max(1, std::min(d.smax, kWindowMaxWaves - (int)nlw));
        c.packed = true;
        c.groups = 1;
        c.sub_bytes = ring + (size_t)2 * kPairNl * nlw * 1024;
        c.lds_bytes = c.sub_bytes + tab;
        return true;
    };
    WindowCfg b, t;
    if (!shape(db, b) || !shape(dt, t)) return false;
    // one launch: both kinds of workgroup get the larger of the two LDS sizes
    const size_t lds = std::max(b.lds_bytes, t.lds_bytes);
    if (lds > lds_limit || 2 * (lds + 512) > kLdsBudget) return false;
    if (b.nc + b.nlw + t.nc + t.nlw > 32) return false;
    b.lds_bytes = t.lds_bytes = lds;
    out_b = b;
    out_t = t;
    return true;
}

int launch_window_pair(const SweepLaunch &sb, const SweepLaunch &st, const WindowCfg &cfg_b, const WindowCfg &cfg_t,
                       void *stream) {
    if (sb.tick_bytes != 4 || st.tick_bytes != 4 || sb.tsweep || !st.tsweep || sb.mask_out || st.mask_out)
        return CP_ERR_ARG;
    if (cfg_b.nl != kPairNl || cfg_t.nl != kPairNl || cfg_b.groups != 1 || cfg_t.groups != 1 ||
        cfg_b.lds_bytes != cfg_t.lds_bytes || sb.win->ent4 != st.win->ent4 || sb.win->far_cap > 0 || st.win->far_cap > 0)
        return CP_ERR_ARG;
    const WindowArgs ab = window_args(sb, cfg_b), at = window_args(st, cfg_t);
    const uint32_t nb = (uint32_t)(8 * ab.pgroups), nt = (uint32_t)(8 * at.pgroups);
    if (nb != nt) return CP_ERR_ARG;         // (the same batch both ways)
    const int waves = std::max(cfg_b.nc + cfg_b.nlw, cfg_t.nc + cfg_t.nlw);
    auto launch = [&](auto kern) {
        if (cfg_b.lds_bytes > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)cfg_b.lds_bytes);
            if (e != hipSuccess) return CP_ERR_HIP;
        }
        hipLaunchKernelGGL(kern, dim3(nb + nt), dim3(waves * 64), cfg_b.lds_bytes, (hipStream_t)stream, ab, at, nb);
        return hip_ok(hipGetLastError());
    };
    return sb.win->ent4 ? launch(window_pair_kernel<true>) : launch(window_pair_kernel<false>);
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

int launch_critical_path(const SweepLaunch &s, const int32_t *sources, int32_t nsrc, const int64_t *cp,
                         int32_t max_len, int32_t *path, int32_t *len, void *stream) {
    const ColumnDir &dir = *s.dir;
    PathArgs a{};
    a.ptr = (const int32_t *)(s.blob + dir.ptr_off);
    a.idx = (const int32_t *)(s.blob + dir.idx_off);
    a.wt = s.blob + dir.wt_off;
    a.c = s.blob + s.c_off;
    a.sources = sources;
    a.nsrc = nsrc;
    a.assign = s.assign;
    a.a_stride_p = s.a_stride_p;
    a.a_stride_v = s.a_stride_v;
    a.b = s.val;
    a.b_sv = s.out_sv;
    a.b_sq = s.out_sq;
    a.cp = cp;
    a.edge_tab = s.edge_tab;
    a.vert_tab = s.vert_tab;
    a.path = path;
    a.len = len;
    a.status = s.status;
    a.P = s.P; a.k = s.k; a.max_len = max_len;
    hipStream_t st = (hipStream_t)stream;
    const bool lds_tab = s.k <= kMagicMaxK;
    const size_t lds = lds_tab ? ((size_t)s.k * s.k + s.k) * 8 : 0;
#define CP_PATH(TICK, WT, MAGIC)                                                                           \
    do {                                                                                                   \
        if (lds_tab)                                                                                       \
            hipLaunchKernelGGL((critical_path_kernel<TICK, WT, MAGIC, true>), dim3((unsigned)s.P), dim3(64), \
                               lds, st, a);                                                                \
        else                                                                                               \
            hipLaunchKernelGGL((critical_path_kernel<TICK, WT, MAGIC, false>), dim3((unsigned)s.P),        \
                               dim3(64), 0, st, a);                                                        \
    } while (0)
    if (s.tick_bytes == 4) {
        if (s.magic) CP_PATH(int32_t, uint32_t, true);
        else if (s.narrow) CP_PATH(int32_t, uint32_t, false);
        else CP_PATH(int32_t, int64_t, false);
    } else {
        if (s.magic) CP_PATH(int64_t, uint32_t, true);
        else if (s.narrow) CP_PATH(int64_t, uint32_t, false);
        else CP_PATH(int64_t, int64_t, false);
    }
#undef CP_PATH
    return hip_ok(hipGetLastError());
}

int launch_mask(const void *b, const void *tl, const int64_t *cp, int32_t n, int32_t P,
                int tick_bytes, bool by_partition, uint64_t *mask, void *stream) {
    const int32_t rows = by_partition ? P : n, cols = by_partition ? n : P;
    const int ncol = (cols + 63) / 64;
    const int64_t tasks = (int64_t)rows * ncol;
    const dim3 grid((unsigned)std::max<int64_t>(1, std::min<int64_t>((tasks + 15) / 16, 256 * 32))), block(256);
    hipStream_t st = (hipStream_t)stream;
    // rows of 32-bit ticks that start on 16-byte boundaries: 16 bytes per load
    if (tick_bytes == 4 && cols % 4 == 0 && ((uintptr_t)b % 16) == 0 && ((uintptr_t)tl % 16) == 0) {
        const int64_t per_block = 4 * 256 * kMaskTrips;
        const int64_t chunks = (cols + per_block - 1) / per_block;
        if (by_partition && rows <= 65535) {
            hipLaunchKernelGGL(mask_rows_kernel<true>, dim3((unsigned)chunks, (unsigned)rows), block, 0, st,
                               (const int32_t *)b, (const int32_t *)tl, cp, cols, ncol, mask);
            return hip_ok(hipGetLastError());
        }
        if (!by_partition && cols >= 256 && chunks <= 65535) {      // (a wavefront per 256 partitions of a vertex)
            hipLaunchKernelGGL(mask_rows_kernel<false>, dim3((unsigned)rows, (unsigned)chunks), block, 0, st,
                               (const int32_t *)b, (const int32_t *)tl, cp, cols, ncol, mask);
            return hip_ok(hipGetLastError());
        }
    }
#define CP_MASK(TICK, BYP)                                                                              \
    hipLaunchKernelGGL((mask_kernel<TICK, BYP>), grid, block, 0, st, (const TICK *)b, (const TICK *)tl, cp, \
                       rows, cols, ncol, mask)
    if (tick_bytes == 4) {
        if (by_partition) CP_MASK(int32_t, true); else CP_MASK(int32_t, false);
    } else {
        if (by_partition) CP_MASK(int64_t, true); else CP_MASK(int64_t, false);
    }
#undef CP_MASK
    return hip_ok(hipGetLastError());
}

int launch_transpose_ticks(const void *in, void *out, int32_t rows, int32_t cols, int tick_bytes, void *stream) {
    const dim3 grid((unsigned)((rows + 63) / 64), (unsigned)((cols + 63) / 64)), block(256);
    if (tick_bytes == 4)
        hipLaunchKernelGGL(transpose_ticks_kernel<int32_t>, grid, block, 0, (hipStream_t)stream,
                           (const int32_t *)in, (int32_t *)out, rows, cols);
    else
        hipLaunchKernelGGL(transpose_ticks_kernel<int64_t>, grid, block, 0, (hipStream_t)stream,
                           (const int64_t *)in, (int64_t *)out, rows, cols);
    return hip_ok(hipGetLastError());
}

}  // namespace cpeval
