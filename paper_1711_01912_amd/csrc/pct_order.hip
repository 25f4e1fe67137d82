// PCT priority lists (paper, section 4.1): per partition, the vertices grouped by
// device and, inside a device, ordered by descending PCT = b, equal values by
// ascending vertex number.  That is a segmented sort under the key
// (device, -b, vertex), done here as a least-significant-digit radix sort with one
// segment per partition:
//
//   key(v) = device(v) << bb | (max_b - b(v))        bb = bit length of max_b
//
// Sorting keys ascending with a stable sort whose input is in vertex order yields the
// list; the vertex number never enters the key.  Each digit (8 bits, or 9 where that
// saves a pass) takes three launches: per-tile digit counts, an exclusive scan of the counts per partition in
// (digit, tile) order, and a stable scatter.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "cpeval_internal.hpp"
#include "launch.hpp"

namespace cpeval {

namespace {

constexpr int kMaxRadix = 512;
constexpr int kSortRounds = 16;                           // items per thread
// Items per workgroup = threads x 16.  Long partitions take 1024 threads: 16384 items, so a
// digit's run in a tile averages 64 items and leaves as full lines; short ones take 256
// threads (4096 items) so that several workgroups share a partition.
constexpr int kSortThreadsLong = 1024, kSortThreadsShort = 256;
constexpr int kSortLongFrom = 65536;                      // vertices from which the long tile is used
inline int sort_threads(int32_t n) { return n >= kSortLongFrom ? kSortThreadsLong : kSortThreadsShort; }
// Passes over a key of `bits` bits: digits of 8 bits, of up to 9 where allowed.
inline int pct_passes(int bits, bool wide) { return (bits + (wide ? 9 : 8) - 1) / (wide ? 9 : 8); }

inline int hip_status(hipError_t e) { return e == hipSuccess ? CP_OK : CP_ERR_HIP; }

// ---------------------------------------------------------------- keys

struct KeyArgs {
    const void *b;            // ticks [n][P]
    const uint8_t *assign;
    int64_t a_stride_p, a_stride_v;
    void *keys;               // Key [P][n]
    int32_t *status;
    int64_t max_b;
    int32_t n, P, k, bb;
};

// b is vertex-major, the sort wants one contiguous key array per partition: 64 x 64
// tiles through LDS.  The device id is read in whichever phase reads it coalesced.
template <typename Tick, typename Key>
__global__ __launch_bounds__(256) void pct_keys_kernel(KeyArgs a) {
    __shared__ Key tile[64][65];
    const int lane = threadIdx.x & 63, row0 = threadIdx.x >> 6;
    const int64_t v0 = (int64_t)blockIdx.x * 64, q0 = (int64_t)blockIdx.y * 64;
    const Tick *b = (const Tick *)a.b;
    Key *keys = (Key *)a.keys;
    const bool ids_by_partition = a.a_stride_p == 1;      // vertex-major assignments
    bool bad_id = false, bad_b = false;
    for (int r = row0; r < 64; r += 4) {
        const int64_t v = v0 + r, q = q0 + lane;
        if (v < a.n && q < a.P) {
            long long bv = (long long)b[v * a.P + q];
            if (bv < 0 || bv > a.max_b) { bad_b = true; bv = bv < 0 ? 0 : a.max_b; }
            Key key = (Key)(a.max_b - bv);
            if (ids_by_partition) {
                uint32_t dev = a.assign[q * a.a_stride_p + v * a.a_stride_v];
                if (dev >= (uint32_t)a.k) { bad_id = true; dev = (uint32_t)a.k - 1; }
                key |= (Key)dev << a.bb;
            }
            tile[r][lane] = key;
        }
    }
    __syncthreads();
    for (int r = row0; r < 64; r += 4) {
        const int64_t q = q0 + r, v = v0 + lane;
        if (v < a.n && q < a.P) {
            Key key = tile[lane][r];
            if (!ids_by_partition) {
                uint32_t dev = a.assign[q * a.a_stride_p + v * a.a_stride_v];
                if (dev >= (uint32_t)a.k) { bad_id = true; dev = (uint32_t)a.k - 1; }
                key |= (Key)dev << a.bb;
            }
            keys[q * a.n + v] = key;
        }
    }
    if (bad_id) atomicOr(a.status, CP_STATUS_BAD_DEVICE_ID);
    if (bad_b) atomicOr(a.status, CP_STATUS_B_OUT_OF_RANGE);
}

// The same from b laid out [P][n]: no transpose, one key per thread.
template <typename Tick, typename Key>
__global__ __launch_bounds__(256) void pct_keys_rows_kernel(KeyArgs a) {
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= a.n) return;
    bool bad_b = false, bad_id = false;
    for (int64_t q = blockIdx.y; q < a.P; q += gridDim.y) {
        long long bv = (long long)((const Tick *)a.b)[q * a.n + v];
        if (bv < 0 || bv > a.max_b) { bad_b = true; bv = bv < 0 ? 0 : a.max_b; }
        uint32_t dev = a.assign[q * a.a_stride_p + v * a.a_stride_v];
        if (dev >= (uint32_t)a.k) { bad_id = true; dev = (uint32_t)a.k - 1; }
        ((Key *)a.keys)[q * a.n + v] = (Key)(a.max_b - bv) | (Key)dev << a.bb;
    }
    if (bad_id) atomicOr(a.status, CP_STATUS_BAD_DEVICE_ID);
    if (bad_b) atomicOr(a.status, CP_STATUS_B_OUT_OF_RANGE);
}

// ---------------------------------------------------------------- one digit pass

template <int RB, typename Key>
__device__ __forceinline__ uint32_t digit_of(Key key, int shift) {
    return (uint32_t)(key >> shift) & ((1u << RB) - 1);
}

// counts[q][digit][tile] = items of the tile with that digit
template <typename Key, int kSortThreads, int RB>
__global__ __launch_bounds__(kSortThreads) void pct_count_kernel(const Key *__restrict__ keys, int32_t n,
                                                                 int32_t tiles, int shift,
                                                                 uint32_t *__restrict__ counts) {
    constexpr int kSortWaves = kSortThreads / 64, kSortTile = kSortThreads * kSortRounds, kRadix = 1 << RB;
    static_assert(kSortThreads >= kRadix, "one thread per digit writes the counts");
    __shared__ uint32_t h[kSortWaves][kRadix];
    const int tid = threadIdx.x, wave = tid >> 6;
    const int32_t tile = (int32_t)(blockIdx.x % (uint32_t)tiles), q = (int32_t)(blockIdx.x / (uint32_t)tiles);
    for (int i = tid; i < kSortWaves * kRadix; i += kSortThreads) (&h[0][0])[i] = 0;
    __syncthreads();
    const Key *src = keys + (int64_t)q * n;
    const int64_t base = (int64_t)tile * kSortTile;
    Key key[kSortRounds];
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {               // all loads first, then the LDS updates
        const int64_t i = base + r * kSortThreads + tid;
        key[r] = i < n ? src[i] : (Key)0;
    }
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = base + r * kSortThreads + tid;
        const uint32_t d = digit_of<RB>(key[r], shift);
        // a wavefront whose lanes all hold one digit (the usual case for the leading digit)
        // adds once instead of 64 times to one counter
        const uint32_t d0 = __builtin_amdgcn_readfirstlane(d);
        const unsigned long long live = __ballot(i < n);
        if (__ballot(i < n && d != d0) == 0) {
            if ((tid & 63) == 0 && live) h[wave][d0] += (uint32_t)__popcll(live);
        } else if (i < n) {
            atomicAdd(&h[wave][d], 1u);
        }
    }
    __syncthreads();
    if (tid < kRadix) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) c += h[w][tid];
        counts[((int64_t)q * kRadix + tid) * tiles + tile] = c;
    }
}

// In place: counts[q][*] becomes its exclusive prefix sum in (digit, tile) order, i.e.
// where the tile's run of that digit starts in the partition's output.
__global__ __launch_bounds__(1024) void pct_scan_kernel(uint32_t *__restrict__ counts, int32_t entries) {
    __shared__ uint32_t wave_sum[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t *c = counts + (int64_t)blockIdx.x * entries;
    const int32_t per = (entries + 1023) / 1024;
    const int32_t lo = min(tid * per, entries), hi = min(lo + per, entries);
    uint32_t sum = 0;
    for (int32_t i = lo; i < hi; ++i) sum += c[i];
    uint32_t inc = sum;                                   // inclusive scan over the wavefront
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(inc, off);
        if (lane >= off) inc += up;
    }
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    uint32_t run = before + inc - sum;
    for (int32_t i = lo; i < hi; ++i) {
        const uint32_t x = c[i];
        c[i] = run;
        run += x;
    }
}

// Stable scatter of one tile.  Wavefront w owns items [w*1024, (w+1)*1024) of the tile
// and takes them 64 at a time, so item order is (wavefront, round, lane).  Inside a
// round, lanes with equal digits find each other by ballots; the lowest of them
// advances the wavefront's counter for that digit.  The tile is then put in digit order
// in LDS and written out in runs: first the keys, then, through the same LDS buffer,
// the vertex numbers.
template <typename Key, int kSortThreads, int RB, bool FIRST, bool LAST>
__global__ __launch_bounds__(kSortThreads) void pct_scatter_kernel(const Key *__restrict__ keys_in,
                                                                   const int32_t *__restrict__ vals_in,
                                                                   Key *__restrict__ keys_out,
                                                                   int32_t *__restrict__ vals_out, int32_t n,
                                                                   int32_t tiles, int shift,
                                                                   const uint32_t *__restrict__ starts) {
    constexpr int kSortWaves = kSortThreads / 64, kSortTile = kSortThreads * kSortRounds, kRadix = 1 << RB;
    static_assert(kSortThreads >= kRadix, "one thread per digit when the tile's digit starts are computed");
    extern __shared__ __align__(16) uint8_t sort_lds[];      // kSortTile keys, later kSortTile vertex numbers
    __shared__ uint32_t cnt[kSortWaves][kRadix];
    __shared__ uint32_t tile_start[kRadix];
    __shared__ int32_t out_base[kRadix];
    __shared__ uint32_t wave_sum[kRadix / 64];
    Key *skey = (Key *)sort_lds;
    int32_t *sval = (int32_t *)sort_lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t tile = (int32_t)(blockIdx.x % (uint32_t)tiles), q = (int32_t)(blockIdx.x / (uint32_t)tiles);
    const int64_t seg = (int64_t)q * n;
    const int64_t base = (int64_t)tile * kSortTile;
    const int32_t tile_items = (int32_t)min((int64_t)kSortTile, (int64_t)n - base);
    for (int i = tid; i < kSortWaves * kRadix; i += kSortThreads) (&cnt[0][0])[i] = 0;
    __syncthreads();

    Key key[kSortRounds];
    int32_t val[kSortRounds];
    uint32_t loc[kSortRounds];       // rank among equal digits, then position in the sorted tile
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t t = wave * (kSortRounds * 64) + r * 64 + lane;      // index inside the tile
        const bool valid = t < tile_items;
        key[r] = valid ? keys_in[seg + base + t] : (Key)0;
        val[r] = FIRST ? (int32_t)(base + t) : (valid ? vals_in[seg + base + t] : 0);
    }
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t t = wave * (kSortRounds * 64) + r * 64 + lane;
        const bool valid = t < tile_items;
        const uint32_t d = digit_of<RB>(key[r], shift);
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < RB; ++bit) {
            const bool one = (d >> bit) & 1u;
            const unsigned long long bal = __ballot(one);
            same &= one ? bal : ~bal;
        }
        if (!valid) same = 1ull << lane;
        const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32),
                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
        const int leader = __ffsll((long long)same) - 1;
        uint32_t old = 0;
        if (valid && lane == leader) {
            old = cnt[wave][d];
            cnt[wave][d] = old + (uint32_t)__popcll(same);
        }
        old = __shfl(old, leader);
        loc[r] = old + rank;
    }
    __syncthreads();
    uint32_t run = 0, inc = 0;
    if (tid < kRadix) {   // thread d: wavefront bases, then the tile's digit starts
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const uint32_t c = cnt[w][tid];
            cnt[w][tid] = run;
            run += c;
        }
        inc = run;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        if (lane == 63) wave_sum[wave] = inc;
    }
    __syncthreads();
    if (tid < kRadix) {
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wave_sum[w];
        const uint32_t start = before + inc - run;
        tile_start[tid] = start;
        out_base[tid] = (int32_t)starts[((int64_t)q * kRadix + tid) * tiles + tile] - (int32_t)start;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t t = wave * (kSortRounds * 64) + r * 64 + lane;
        if (t < tile_items) {
            const uint32_t d = digit_of<RB>(key[r], shift);
            loc[r] = tile_start[d] + cnt[wave][d] + loc[r];
            skey[loc[r]] = key[r];
        }
    }
    __syncthreads();
    int32_t dst[kSortRounds];        // where item i of the sorted tile goes in the partition's output
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t i = r * kSortThreads + tid;
        dst[r] = 0;
        if (i < tile_items) {
            const Key kk = skey[i];
            dst[r] = out_base[digit_of<RB>(kk, shift)] + i;
            if (!LAST) keys_out[seg + dst[r]] = kk;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t t = wave * (kSortRounds * 64) + r * 64 + lane;
        if (t < tile_items) sval[loc[r]] = val[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t i = r * kSortThreads + tid;
        if (i < tile_items) vals_out[seg + dst[r]] = sval[i];
    }
}

// seg[q][d] = first position of the sorted list whose vertex sits on a device >= d
__global__ void pct_segments_kernel(const int32_t *__restrict__ order, const uint8_t *__restrict__ assign,
                                    int64_t a_stride_p, int64_t a_stride_v, int32_t n, int32_t P, int32_t k,
                                    int32_t *__restrict__ seg) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)P * (k + 1)) return;
    const int32_t q = (int32_t)(i / (k + 1)), d = (int32_t)(i % (k + 1));
    const int32_t *ord = order + (int64_t)q * n;
    int32_t lo = 0, hi = n;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        const int32_t dev = min((int32_t)assign[q * a_stride_p + (int64_t)ord[mid] * a_stride_v], k - 1);
        if (dev < d) lo = mid + 1; else hi = mid;
    }
    seg[i] = lo;
}

// One digit pass of RB bits starting at bit `shift`.
template <typename Key, int THREADS, int RB>
int run_pass(const PctOrderLaunch &s, hipStream_t st, int shift, bool first, bool last, const Key *kin, Key *kout,
             const int32_t *vin, int32_t *vout) {
    constexpr int kTile = THREADS * kSortRounds;
    const int32_t n = s.n, P = s.P;
    const int32_t tiles = (n + kTile - 1) / kTile;
    const dim3 grid((unsigned)((int64_t)tiles * P)), block(THREADS);     // one workgroup per (partition, tile)
    const size_t lds = (size_t)kTile * sizeof(Key);
    hipLaunchKernelGGL((pct_count_kernel<Key, THREADS, RB>), grid, block, 0, st, kin, n, tiles, shift, s.counts);
    hipLaunchKernelGGL(pct_scan_kernel, dim3((unsigned)P), dim3(1024), 0, st, s.counts, (1 << RB) * tiles);
#define CP_SCATTER(F, L)                                                                                   \
    do {                                                                                                   \
        auto kern = pct_scatter_kernel<Key, THREADS, RB, F, L>;                                            \
        /* more than 64 KB of dynamic LDS has to be asked for */                                           \
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                   (int)lds) != hipSuccess)                                \
            return CP_ERR_HIP;                                                                             \
        hipLaunchKernelGGL(kern, grid, block, lds, st, kin, vin, kout, vout, n, tiles, shift, s.counts);   \
    } while (0)
    if (first && last) CP_SCATTER(true, true);
    else if (first) CP_SCATTER(true, false);
    else if (last) CP_SCATTER(false, true);
    else CP_SCATTER(false, false);
#undef CP_SCATTER
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
}

// WIDE: 9-bit digits may be used (long tiles of 32-bit keys: the counters of a 64-bit
// tile's 512 digits would not fit LDS beside the tile).
template <typename Key, int THREADS, bool WIDE>
int run_sort(const PctOrderLaunch &s, hipStream_t st) {
    Key *ka = (Key *)s.keys_a, *kb = (Key *)s.keys_b;
    const int passes = pct_passes(s.key_bits, WIDE);
    // 8 bits per pass; where that leaves bits over, the leading passes take 9
    const int wide_passes = std::max(0, s.key_bits - 8 * passes);
    int shift = 0;
    // vertex lists alternate between the scratch list and the output so that the last
    // pass writes the output
    for (int p = 0; p < passes; ++p) {
        const bool first = p == 0, last = p == passes - 1;
        const Key *kin = (p & 1) ? kb : ka;
        Key *kout = (p & 1) ? ka : kb;
        const bool to_out = ((passes - 1 - p) & 1) == 0;
        int32_t *vout = to_out ? s.order_out : s.vals_tmp;
        const int32_t *vin = to_out ? s.vals_tmp : s.order_out;
        int rc;
        if (WIDE && p < wide_passes) {
            rc = run_pass<Key, THREADS, WIDE ? 9 : 8>(s, st, shift, first, last, kin, kout, vin, vout);
            shift += 9;
        } else {
            rc = run_pass<Key, THREADS, 8>(s, st, shift, first, last, kin, kout, vin, vout);
            shift += 8;
        }
        if (rc) return rc;
    }
    return CP_OK;
}

}  // namespace

int32_t pct_sort_tiles(int32_t n) {
    const int tile = sort_threads(n) * kSortRounds;
    return (n + tile - 1) / tile;
}
size_t pct_counts_bytes(int32_t n, int32_t P) {
    return align_up((size_t)P * kMaxRadix * (size_t)pct_sort_tiles(n) * sizeof(uint32_t));
}

int launch_pct_order(const PctOrderLaunch &s, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    KeyArgs a{};
    a.b = s.b;
    a.assign = s.assign;
    a.a_stride_p = s.a_stride_p;
    a.a_stride_v = s.a_stride_v;
    a.keys = s.keys_a;
    a.status = s.status;
    a.max_b = s.max_b;
    a.n = s.n; a.P = s.P; a.k = s.k; a.bb = s.b_bits;
#define CP_KEYS(KERNEL, GRID)                                                                         \
    do {                                                                                              \
        if (s.key_bytes == 4) {                                                                       \
            if (s.tick_bytes == 4) hipLaunchKernelGGL((KERNEL<int32_t, uint32_t>), GRID, dim3(256), 0, st, a); \
            else hipLaunchKernelGGL((KERNEL<int64_t, uint32_t>), GRID, dim3(256), 0, st, a);          \
        } else {                                                                                      \
            if (s.tick_bytes == 4) hipLaunchKernelGGL((KERNEL<int32_t, uint64_t>), GRID, dim3(256), 0, st, a); \
            else hipLaunchKernelGGL((KERNEL<int64_t, uint64_t>), GRID, dim3(256), 0, st, a);          \
        }                                                                                             \
    } while (0)
    if (s.b_by_partition) {
        const dim3 kgrid((unsigned)((s.n + 255) / 256), (unsigned)std::min(s.P, 65535));
        CP_KEYS(pct_keys_rows_kernel, kgrid);
    } else {
        const dim3 kgrid((unsigned)((s.n + 63) / 64), (unsigned)((s.P + 63) / 64));
        CP_KEYS(pct_keys_kernel, kgrid);
    }
#undef CP_KEYS
    if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
    int rc;
    if (sort_threads(s.n) == kSortThreadsLong)
        rc = s.key_bytes == 4 ? run_sort<uint32_t, kSortThreadsLong, true>(s, st)
                              : run_sort<uint64_t, kSortThreadsLong, false>(s, st);
    else
        rc = s.key_bytes == 4 ? run_sort<uint32_t, kSortThreadsShort, false>(s, st)
                              : run_sort<uint64_t, kSortThreadsShort, false>(s, st);
    if (rc) return rc;
    const int64_t cells = (int64_t)s.P * (s.k + 1);
    hipLaunchKernelGGL(pct_segments_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, st,
                       (const int32_t *)s.order_out, s.assign, s.a_stride_p, s.a_stride_v, s.n, s.P, s.k,
                       s.seg_out);
    return hip_status(hipGetLastError());
}

}  // namespace cpeval
