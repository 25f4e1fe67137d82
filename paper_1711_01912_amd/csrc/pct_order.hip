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
//
// Ranking inside a wavefront is done by ballots (one per key bit): lanes with equal digits
// find each other, every lane reads its digit's counter, the last lane of a group moves it on.
//
// Partitions of at most 20,480 vertices with 32-bit keys are sorted by one workgroup each, entirely
// inside LDS (the bucket kernel below with the whole partition as its bucket).
//
// Long partitions of 32-bit keys take a shorter way where they can: a pass on the LEADING 9
// bits cuts a partition into 512 buckets, and a bucket of at most 4,096 or 8,192 items is then
// sorted on the remaining bits entirely inside LDS by one workgroup (the same ranking, LDS to
// LDS) and leaves as the finished list: an item crosses HBM three times (keys written, the
// leading digit's scatter, the bucket sort) whatever the key length.  Whether every bucket fits
// is only known on the device, after the scan of the leading digit's counts.  So both
// continuations are launched -- the leading digit's scatter and the bucket sort, or the
// ordinary passes from the low digit up -- and a flag the bucket check sets lets the kernels of
// one of them return at once.  With rows of b per partition, one kernel writes the keys and
// counts their leading digit.
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

// the bucket path cuts a partition by its leading kBucketBits bits, in tiles of kLeadThreads x 16
// items: half the long tile, so that two workgroups of the leading scatter share a compute unit
// and one's ranking overlaps the other's loads and stores
constexpr int kBucketBits = 9, kBuckets = 1 << kBucketBits;
constexpr int kLeadThreads = 512;

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

// A kernel launched for one of two continuations returns at once when the device-side flag
// says the other one runs (flag == nullptr: always runs).  Uniform for the whole grid.
struct Gate {
    const uint32_t *flag;
    uint32_t want;
    __device__ __forceinline__ bool closed() const { return flag != nullptr && *flag != want; }
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

// The counting kernels keep several copies of the histogram in LDS, a lane adding to copy
// (lane mod copies): the vertices of a wavefront often share a handful of leading digits, and
// adds to one counter queue up behind each other.  A copy's row is one word longer than the
// radix, so that equal digits in different copies fall into different banks.
template <int kThreads, int kRadix>
struct Histogram {
    static constexpr int kCopies = kThreads >= 1024 ? 8192 / kRadix : 8;      // 16 or 32; 8 for the short tile
    uint32_t h[kCopies][kRadix + 1];
    __device__ __forceinline__ void clear(int tid) {
        for (int i = tid; i < kCopies * (kRadix + 1); i += kThreads) (&h[0][0])[i] = 0;
    }
    __device__ __forceinline__ void add(int tid, uint32_t d) { atomicAdd(&h[tid & (kCopies - 1)][d], 1u); }
    __device__ __forceinline__ uint32_t total(uint32_t d) const {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kCopies; ++w) c += h[w][d];
        return c;
    }
};

// counts[q][digit][tile] = items of the tile with that digit
template <typename Key, int kSortThreads, int RB>
__global__ __launch_bounds__(kSortThreads) void pct_count_kernel(const Key *__restrict__ keys, int32_t n,
                                                                 int32_t tiles, int shift,
                                                                 uint32_t *__restrict__ counts, Gate gate) {
    constexpr int kSortTile = kSortThreads * kSortRounds, kRadix = 1 << RB;
    static_assert(kSortThreads >= kRadix, "one thread per digit writes the counts");
    if (gate.closed()) return;
    __shared__ Histogram<kSortThreads, kRadix> hist;
    const int tid = threadIdx.x;
    const int32_t tile = (int32_t)(blockIdx.x % (uint32_t)tiles), q = (int32_t)(blockIdx.x / (uint32_t)tiles);
    hist.clear(tid);
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
        if (i < n) hist.add(tid, digit_of<RB>(key[r], shift));
    }
    __syncthreads();
    if (tid < kRadix) counts[((int64_t)q * kRadix + tid) * tiles + tile] = hist.total(tid);
}

// Keys from rows of b ([P][n]) and, in the same pass, the counts of their leading digit: what
// pct_keys_rows_kernel and the first pct_count_kernel do, with one read of b.  A thread takes four
// consecutive vertices per round (VEC: as one 16-byte load of b, one 4-byte load of device ids, one
// 16-byte store of keys; needs n % 4 == 0, unit stride between a partition's ids and aligned rows).
struct alignas(16) Keys4 { uint32_t x[4]; };
template <typename Tick> struct alignas(16) Ticks4 { Tick x[4]; };
template <typename Tick, bool VEC>
__global__ __launch_bounds__(kLeadThreads) void pct_keys_count_kernel(KeyArgs a, int32_t tiles, int shift,
                                                                          uint32_t *__restrict__ counts) {
    constexpr int kRadix = 1 << kBucketBits, kTile = kLeadThreads * kSortRounds;
    constexpr int kQuadRounds = kSortRounds / 4;
    __shared__ Histogram<kLeadThreads, kRadix> hist;
    const int tid = threadIdx.x;
    const int32_t tile = (int32_t)(blockIdx.x % (uint32_t)tiles), q = (int32_t)(blockIdx.x / (uint32_t)tiles);
    hist.clear(tid);
    __syncthreads();
    const Tick *b = (const Tick *)a.b + (int64_t)q * a.n;
    const uint8_t *ids = a.assign + q * a.a_stride_p;
    uint32_t *keys = (uint32_t *)a.keys + (int64_t)q * a.n;
    const int32_t base = tile * kTile;
    uint32_t key[kQuadRounds][4];
    bool bad_b = false, bad_id = false;
#pragma unroll
    for (int r = 0; r < kQuadRounds; ++r) {
        const int32_t i0 = base + (r * kLeadThreads + tid) * 4;
        Ticks4<Tick> bv{};
        uint32_t dv = 0;
        if (VEC) {
            if (i0 < a.n) {
                bv = *(const Ticks4<Tick> *)(b + i0);
                dv = *(const uint32_t *)(ids + i0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i0 + j < a.n) {
                    bv.x[j] = b[i0 + j];
                    dv |= (uint32_t)ids[(int64_t)(i0 + j) * a.a_stride_v] << (8 * j);
                }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            long long t = (long long)bv.x[j];
            if (t < 0 || t > a.max_b) { bad_b = true; t = t < 0 ? 0 : a.max_b; }
            uint32_t dev = (dv >> (8 * j)) & 0xffu;
            if (dev >= (uint32_t)a.k) { bad_id = true; dev = (uint32_t)a.k - 1; }
            key[r][j] = (uint32_t)(a.max_b - t) | dev << a.bb;
        }
        if (VEC) {
            if (i0 < a.n) *(Keys4 *)(keys + i0) = Keys4{{key[r][0], key[r][1], key[r][2], key[r][3]}};
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i0 + j < a.n) keys[i0 + j] = key[r][j];
        }
    }
    if (bad_id) atomicOr(a.status, CP_STATUS_BAD_DEVICE_ID);
    if (bad_b) atomicOr(a.status, CP_STATUS_B_OUT_OF_RANGE);
#pragma unroll
    for (int r = 0; r < kQuadRounds; ++r) {
        const int32_t i0 = base + (r * kLeadThreads + tid) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i0 + j < a.n) hist.add(tid, digit_of<kBucketBits>(key[r][j], shift));
    }
    __syncthreads();
    if (tid < kRadix) counts[((int64_t)q * kRadix + tid) * tiles + tile] = hist.total(tid);
}

// In place: counts[q][*] becomes its exclusive prefix sum in (digit, tile) order, i.e.
// where the tile's run of that digit starts in the partition's output.  One workgroup per
// partition walks the entries 4,096 at a time, four neighbours per thread (entries is a
// multiple of the radix, so of four, and every partition's row is 16-byte aligned).
struct alignas(16) Counts4 { uint32_t x[4]; };
__global__ __launch_bounds__(1024) void pct_scan_kernel(uint32_t *__restrict__ counts, int32_t entries, Gate gate) {
    __shared__ uint32_t wave_sum[2][16];                  // (two sets: one barrier per step)
    if (gate.closed()) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t *c = counts + (int64_t)blockIdx.x * entries;
    uint32_t carry = 0;
    int set = 0;
    for (int32_t base = 0; base < entries; base += 4096, set ^= 1) {
        const int32_t i = base + tid * 4;
        Counts4 v{};
        if (i < entries) v = *(const Counts4 *)(c + i);
        const uint32_t sum = v.x[0] + v.x[1] + v.x[2] + v.x[3];
        uint32_t inc = sum;                               // inclusive scan over the wavefront
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        if (lane == 63) wave_sum[set][wave] = inc;
        __syncthreads();
        uint32_t before = carry;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const uint32_t ws = wave_sum[set][w];
            if (w < wave) before += ws;
            carry += ws;
        }
        uint32_t run = before + inc - sum;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t x = v.x[j];
            v.x[j] = run;
            run += x;
        }
        if (i < entries) *(Counts4 *)(c + i) = v;
    }
}

// The lanes of the wavefront whose item is valid and has the same RB-bit digit as this lane's
// (for a lane with a valid item).  One ballot per bit; a lane collects, per half of the
// wavefront, the lanes whose bit differs from its own.
template <int RB>
__device__ __forceinline__ unsigned long long lanes_with_same_digit(uint32_t d, bool valid) {
    uint32_t diff_lo = 0, diff_hi = 0;
#pragma unroll
    for (int bit = 0; bit < RB; ++bit) {
        const uint32_t mine = (uint32_t)((int32_t)(d << (31 - bit)) >> 31);      // all ones where the bit is set
        const unsigned long long bal = __ballot(mine != 0);
        diff_lo |= (uint32_t)bal ^ mine;
        diff_hi |= (uint32_t)(bal >> 32) ^ mine;
    }
    const unsigned long long live = __ballot(valid);
    return live & ~((unsigned long long)diff_hi << 32 | diff_lo);
}

// Rank of a valid lane's item among the wavefront's earlier items with its digit: the digit's
// counter (one row of counters per wavefront) plus the lane's place among the lanes of this
// round that share the digit; the last of them moves the counter on.  LDS reads and writes of
// one wavefront keep their order, so every lane has read before one writes.
template <int RB>
__device__ __forceinline__ uint32_t rank_in_wavefront(uint32_t *counters, uint32_t d, bool valid) {
    const unsigned long long same = lanes_with_same_digit<RB>(d, valid);
    const uint32_t place = __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32),
                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
    const uint32_t together = (uint32_t)__popcll(same);
    uint32_t before = 0;
    if (valid) {
        before = counters[d];
        if (place + 1 == together) counters[d] = before + together;
    }
    return before + place;
}

// Where the scatter kernel keeps what belongs to digit d in its LDS tables: a permutation of
// the digits that moves digits 32, 64, ... apart into different banks (the device id sits in
// the upper bits of the leading digit, so the digits of one wavefront often differ by that).
__device__ __forceinline__ uint32_t cell_of(uint32_t d) { return d ^ (d >> 5); }

// Stable scatter of one tile.  Wavefront w owns items [w*1024, (w+1)*1024) of the tile
// and takes them 64 at a time, so item order is (wavefront, round, lane).  Inside a
// round, lanes with equal digits find each other by ballots; the last of them
// advances the wavefront's counter for that digit.  The tile is then put in digit order
// in LDS and written out in runs: first the keys, then, through the same LDS buffer,
// the vertex numbers.
template <typename Key, int kSortThreads, int RB, bool FIRST, bool LAST>
__global__ __launch_bounds__(kSortThreads) void pct_scatter_kernel(const Key *__restrict__ keys_in,
                                                                   const int32_t *__restrict__ vals_in,
                                                                   Key *__restrict__ keys_out,
                                                                   int32_t *__restrict__ vals_out, int32_t n,
                                                                   int32_t tiles, int shift,
                                                                   const uint32_t *__restrict__ starts, Gate gate) {
    constexpr int kSortWaves = kSortThreads / 64, kSortTile = kSortThreads * kSortRounds, kRadix = 1 << RB;
    static_assert(kSortThreads >= kRadix, "one thread per digit when the tile's digit starts are computed");
    if (gate.closed()) return;
    extern __shared__ __align__(16) uint8_t sort_lds[];      // kSortTile keys, later kSortTile vertex numbers
    __shared__ uint32_t cnt[kSortWaves][kRadix];
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
        loc[r] = rank_in_wavefront<RB>(cnt[wave], cell_of(digit_of<RB>(key[r], shift)), valid);
    }
    __syncthreads();
    uint32_t run = 0, inc = 0;
    if (tid < kRadix) {   // thread d: wavefront bases, then the tile's digit starts
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const uint32_t c = cnt[w][cell_of(tid)];
            cnt[w][cell_of(tid)] = run;
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
        out_base[cell_of(tid)] = (int32_t)starts[((int64_t)q * kRadix + tid) * tiles + tile] - (int32_t)start;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) cnt[w][cell_of(tid)] += start;   // now positions in the sorted tile
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int32_t t = wave * (kSortRounds * 64) + r * 64 + lane;
        if (t < tile_items) {
            const uint32_t d = cell_of(digit_of<RB>(key[r], shift));
            loc[r] = cnt[wave][d] + loc[r];
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
            dst[r] = out_base[cell_of(digit_of<RB>(kk, shift))] + i;
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

// ---------------------------------------------------------------- buckets of the leading digit

// a bucket is sorted by a workgroup of 256 or 512 threads, 16 items per thread at most
constexpr int kBucketCapSmall = 256 * kSortRounds, kBucketCapLarge = 512 * kSortRounds;     // 4,096 / 8,192 items

__global__ void pct_flag_clear_kernel(uint32_t *flag) { *flag = 0; }

// After the scan of the leading digit's counts, bucket d of partition q starts where tile 0's
// run of digit d starts.  flag |= 1 if some bucket holds more than `cap` items.
__global__ __launch_bounds__(kBuckets) void pct_bucket_check_kernel(const uint32_t *__restrict__ starts, int32_t n,
                                                                    int32_t tiles, int32_t cap, uint32_t *flag) {
    const int32_t q = blockIdx.x, d = threadIdx.x;
    const uint32_t lo = starts[((int64_t)q * kBuckets + d) * tiles];
    const uint32_t hi = d + 1 < kBuckets ? starts[((int64_t)q * kBuckets + d + 1) * tiles] : (uint32_t)n;
    // (one atomic per partition at most, none once the flag is up: they queue up on the one word)
    const int any = __syncthreads_or(hi - lo > (uint32_t)cap);
    if (any && threadIdx.x == 0 && *(volatile const uint32_t *)flag == 0) atomicOr(flag, 1u);
}

// WHOLE: the "bucket" is a whole partition (at most kBucketThreads * kRounds vertices), its keys
// in vertex order in keys_in, sorted on all `bits` key bits: short partitions need no pass over
// HBM at all.
// One bucket, sorted on the low `bits` bits inside LDS: stable passes of 8 bits, each ranking
// the items as the scatter kernel does (wavefront w owns items [w*1024, (w+1)*1024) of the
// bucket in (round, lane) order) and moving keys and vertex numbers through one LDS buffer;
// the vertex numbers of the last pass go straight out.
template <int kBucketThreads, int kRounds, bool WHOLE>
__global__ __launch_bounds__(kBucketThreads) void pct_bucket_sort_kernel(const uint32_t *__restrict__ keys_in,
                                                                         const int32_t *__restrict__ vals_in,
                                                                         int32_t *__restrict__ vals_out, int32_t n,
                                                                         int32_t tiles, int bits,
                                                                         const uint32_t *__restrict__ starts, Gate gate) {
    constexpr int kWaves = kBucketThreads / 64, kRadix = 256, kBucketCap = kBucketThreads * kRounds;
    extern __shared__ __align__(16) uint32_t slot[];      // kBucketCap keys, then vertex numbers, in sorted order
    __shared__ uint32_t cnt[kWaves][kRadix];
    __shared__ uint32_t wave_sum[kRadix / 64];
    if (gate.closed()) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t q = WHOLE ? (int32_t)blockIdx.x : (int32_t)(blockIdx.x / kBuckets);
    const int32_t d = WHOLE ? 0 : (int32_t)(blockIdx.x % kBuckets);
    const uint32_t lo = WHOLE ? 0u : starts[((int64_t)q * kBuckets + d) * tiles];
    const uint32_t hi = WHOLE || d + 1 == kBuckets ? (uint32_t)n : starts[((int64_t)q * kBuckets + d + 1) * tiles];
    const int32_t items = (int32_t)(hi - lo);
    if (items <= 0 || items > kBucketCap) return;         // (larger buckets: the other continuation runs)
    const int64_t at = (int64_t)q * n + lo;
    // rounds this bucket needs (the same for every wavefront: wavefront w owns items
    // [w * nr * 64, (w + 1) * nr * 64) of the bucket)
    const int nr = (items + kBucketThreads - 1) / kBucketThreads;

    uint32_t key[kRounds], loc[kRounds];
    int32_t val[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int32_t t = wave * (nr * 64) + r * 64 + lane;
        const bool valid = r < nr && t < items;
        key[r] = valid ? keys_in[at + t] : 0u;
        val[r] = WHOLE ? t : (valid ? vals_in[at + t] : 0);       // WHOLE: the keys come in vertex order
    }
    for (int shift = 0; shift < bits; shift += 8) {
        const bool last = shift + 8 >= bits;
        for (int i = tid; i < kWaves * kRadix; i += kBucketThreads) (&cnt[0][0])[i] = 0;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            if (r >= nr) continue;           // (uniform)
            const int32_t t = wave * (nr * 64) + r * 64 + lane;
            const bool valid = t < items;
            loc[r] = rank_in_wavefront<8>(cnt[wave], digit_of<8>(key[r], shift), valid);
        }
        __syncthreads();
        // thread dg: the digit's items per wavefront, the bucket's digit starts, then every
        // wavefront's first position for the digit
        uint32_t per_wave[kWaves], run = 0, inc = 0;
        if (tid < kRadix) {
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                per_wave[w] = cnt[w][tid];
                run += per_wave[w];
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
            uint32_t first = inc - run;
            for (int w = 0; w < wave; ++w) first += wave_sum[w];
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                cnt[w][tid] = first;
                first += per_wave[w];
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int32_t t = wave * (nr * 64) + r * 64 + lane;
            if (r < nr && t < items) {
                const uint32_t dg = digit_of<8>(key[r], shift);
                loc[r] = cnt[wave][dg] + loc[r];
                if (!last) slot[loc[r]] = key[r];
            }
        }
        if (!last) {          // the keys come back in sorted order, then the vertex numbers the same way
            __syncthreads();
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int32_t t = wave * (nr * 64) + r * 64 + lane;
                if (r < nr && t < items) key[r] = slot[t];
            }
            __syncthreads();
        }
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int32_t t = wave * (nr * 64) + r * 64 + lane;
            if (r < nr && t < items) slot[loc[r]] = (uint32_t)val[r];
        }
        __syncthreads();
        if (last) {
            for (int32_t i = tid; i < items; i += kBucketThreads) vals_out[at + i] = (int32_t)slot[i];
        } else {
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int32_t t = wave * (nr * 64) + r * 64 + lane;
                if (r < nr && t < items) val[r] = (int32_t)slot[t];
            }
            __syncthreads();
        }
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

// The launches of one digit pass of RB bits starting at bit `shift`: counts, scan, scatter.
template <typename Key, int THREADS, int RB>
struct DigitPass {
    static constexpr int kTile = THREADS * kSortRounds;
    const PctOrderLaunch &s;
    hipStream_t st;
    int shift;
    Gate gate;
    int32_t tiles() const { return (s.n + kTile - 1) / kTile; }
    dim3 grid() const { return dim3((unsigned)((int64_t)tiles() * s.P)); }     // one workgroup per (partition, tile)
    void count(const Key *kin) const {
        hipLaunchKernelGGL((pct_count_kernel<Key, THREADS, RB>), grid(), dim3(THREADS), 0, st, kin, s.n, tiles(), shift,
                           s.counts, gate);
    }
    void scan() const {
        hipLaunchKernelGGL(pct_scan_kernel, dim3((unsigned)s.P), dim3(1024), 0, st, s.counts, (1 << RB) * tiles(), gate);
    }
    int scatter(bool first, bool last, const Key *kin, Key *kout, const int32_t *vin, int32_t *vout) const {
        const size_t lds = (size_t)kTile * sizeof(Key);
#define CP_SCATTER(F, L)                                                                                   \
    do {                                                                                                   \
        auto kern = pct_scatter_kernel<Key, THREADS, RB, F, L>;                                            \
        /* more than 64 KB of dynamic LDS has to be asked for */                                           \
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                   (int)lds) != hipSuccess)                                \
            return CP_ERR_HIP;                                                                             \
        hipLaunchKernelGGL(kern, grid(), dim3(THREADS), lds, st, kin, vin, kout, vout, s.n, tiles(), shift, s.counts, \
                           gate);                                                                          \
    } while (0)
        if (first && last) CP_SCATTER(true, true);
        else if (first) CP_SCATTER(true, false);
        else if (last) CP_SCATTER(false, true);
        else CP_SCATTER(false, false);
#undef CP_SCATTER
        return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
    }
};

template <typename Key, int THREADS, int RB>
int run_pass(const PctOrderLaunch &s, hipStream_t st, int shift, bool first, bool last, const Key *kin, Key *kout,
             const int32_t *vin, int32_t *vout, Gate gate) {
    const DigitPass<Key, THREADS, RB> pass{s, st, shift, gate};
    pass.count(kin);
    pass.scan();
    return pass.scatter(first, last, kin, kout, vin, vout);
}

// WIDE: 9-bit digits may be used (long tiles of 32-bit keys: the counters of a 64-bit
// tile's 512 digits would not fit LDS beside the tile).
template <typename Key, int THREADS, bool WIDE>
int run_sort(const PctOrderLaunch &s, hipStream_t st, Gate gate = Gate{nullptr, 0}) {
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
            rc = run_pass<Key, THREADS, WIDE ? 9 : 8>(s, st, shift, first, last, kin, kout, vin, vout, gate);
            shift += 9;
        } else {
            rc = run_pass<Key, THREADS, 8>(s, st, shift, first, last, kin, kout, vin, vout, gate);
            shift += 8;
        }
        if (rc) return rc;
    }
    return CP_OK;
}

// The key kernels, for all four (tick, key) widths.
void launch_keys(const PctOrderLaunch &s, const KeyArgs &a, hipStream_t st) {
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
}

// The leading digit's counts, the bucket check on their scan, and both continuations: the
// leading digit's scatter and the buckets sorted inside LDS (flag 0), or the ordinary passes
// from the untouched keys (flag 1).  With rows of b per partition one kernel writes the keys
// and counts their leading digit.
int run_bucket_sort(const PctOrderLaunch &s, const KeyArgs &a, hipStream_t st) {
    constexpr int kTile = kLeadThreads * kSortRounds;
    const int32_t tiles = (s.n + kTile - 1) / kTile;
    uint32_t *flag = s.counts + (size_t)s.P * kMaxRadix * (size_t)tiles;     // behind the counts
    hipLaunchKernelGGL(pct_flag_clear_kernel, dim3(1), dim3(1), 0, st, flag);
    const int rem = s.key_bits - kBucketBits;
    if (s.b_by_partition) {
        const dim3 grid((unsigned)((int64_t)tiles * s.P)), block(kLeadThreads);
        const bool vec = s.n % 4 == 0 && s.a_stride_v == 1 && s.a_stride_p % 4 == 0 && (uintptr_t)s.assign % 4 == 0 &&
                         (uintptr_t)s.b % 16 == 0 && (uintptr_t)s.keys_a % 16 == 0;
        if (s.tick_bytes == 4) {
            if (vec) hipLaunchKernelGGL((pct_keys_count_kernel<int32_t, true>), grid, block, 0, st, a, tiles, rem, s.counts);
            else hipLaunchKernelGGL((pct_keys_count_kernel<int32_t, false>), grid, block, 0, st, a, tiles, rem, s.counts);
        } else {
            if (vec) hipLaunchKernelGGL((pct_keys_count_kernel<int64_t, true>), grid, block, 0, st, a, tiles, rem, s.counts);
            else hipLaunchKernelGGL((pct_keys_count_kernel<int64_t, false>), grid, block, 0, st, a, tiles, rem, s.counts);
        }
    } else {
        launch_keys(s, a, st);
    }
    const DigitPass<uint32_t, kLeadThreads, kBucketBits> lead{s, st, rem, Gate{nullptr, 0u}};
    if (!s.b_by_partition) lead.count((const uint32_t *)s.keys_a);
    lead.scan();
    // the smaller workgroup (more of them per compute unit) where buckets of twice the average size fit it
    const bool small = 2 * ((int64_t)s.n / kBuckets + 1) <= kBucketCapSmall;
    hipLaunchKernelGGL(pct_bucket_check_kernel, dim3((unsigned)s.P), dim3(kBuckets), 0, st, s.counts, s.n, tiles,
                       small ? kBucketCapSmall : kBucketCapLarge, flag);
    if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
    const DigitPass<uint32_t, kLeadThreads, kBucketBits> lead_if_fit{s, st, rem, Gate{flag, 0u}};
    const int rc = lead_if_fit.scatter(/*first=*/true, /*last=*/false, (const uint32_t *)s.keys_a, (uint32_t *)s.keys_b,
                                       nullptr, s.vals_tmp);
    if (rc) return rc;
    const dim3 bgrid((unsigned)((int64_t)s.P * kBuckets));
    if (small)
        hipLaunchKernelGGL((pct_bucket_sort_kernel<256, kSortRounds, false>), bgrid, dim3(256),
                           (size_t)kBucketCapSmall * 4, st, (const uint32_t *)s.keys_b,
                           (const int32_t *)s.vals_tmp, s.order_out, s.n, tiles, rem, (const uint32_t *)s.counts,
                           Gate{flag, 0u});
    else
        hipLaunchKernelGGL((pct_bucket_sort_kernel<512, kSortRounds, false>), bgrid, dim3(512),
                           (size_t)kBucketCapLarge * 4, st, (const uint32_t *)s.keys_b,
                           (const int32_t *)s.vals_tmp, s.order_out, s.n, tiles, rem, (const uint32_t *)s.counts,
                           Gate{flag, 0u});
    if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
    return run_sort<uint32_t, kSortThreadsLong, true>(s, st, Gate{flag, 1u});
}

// Partitions of at most 20,480 vertices with 32-bit keys: one workgroup sorts a whole partition
// inside LDS.
constexpr int kWholeRoundsMax = 20, kWholeMax = kSortThreadsLong * kWholeRoundsMax;
template <int THREADS, int ROUNDS>
int launch_whole(const PctOrderLaunch &s, hipStream_t st) {
    auto kern = pct_bucket_sort_kernel<THREADS, ROUNDS, true>;
    const size_t lds = (size_t)THREADS * ROUNDS * 4;
    // more than 64 KB of dynamic LDS has to be asked for
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return CP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)s.P), dim3(THREADS), lds, st, (const uint32_t *)s.keys_a,
                       (const int32_t *)nullptr, s.order_out, s.n, 0, s.key_bits, (const uint32_t *)nullptr,
                       Gate{nullptr, 0u});
    return hip_status(hipGetLastError());
}
int run_whole_sort(const PctOrderLaunch &s, hipStream_t st) {
    if (s.n <= 256 * kSortRounds) return launch_whole<256, kSortRounds>(s, st);
    if (s.n <= 512 * kSortRounds) return launch_whole<512, kSortRounds>(s, st);
    if (s.n <= 1024 * kSortRounds) return launch_whole<1024, kSortRounds>(s, st);
    return launch_whole<1024, kWholeRoundsMax>(s, st);
}

}  // namespace

int32_t pct_sort_tiles(int32_t n) {
    // (long partitions: the leading pass of the bucket path has the most tiles)
    const int tile = (n >= kSortLongFrom ? kLeadThreads : kSortThreadsShort) * kSortRounds;
    return (n + tile - 1) / tile;
}
size_t pct_counts_bytes(int32_t n, int32_t P) {
    // (and the flag of the bucket path behind them)
    return align_up((size_t)P * kMaxRadix * (size_t)pct_sort_tiles(n) * sizeof(uint32_t) + 256);
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
    int rc;
    // the bucket path: long partitions of 32-bit keys whose buckets hold a quarter of their
    // capacity on average (so that an uneven spread still fits), at least two passes to save
    const bool buckets = sort_threads(s.n) == kSortThreadsLong && s.key_bytes == 4 && s.key_bits > kBucketBits + 8 &&
                         (int64_t)s.n <= (int64_t)kBuckets * kBucketCapLarge / 4 && (int64_t)s.P * kBuckets < (1ll << 31);
    const bool whole = s.key_bytes == 4 && s.n <= kWholeMax;
    if (!buckets) {
        launch_keys(s, a, st);
        if (hipGetLastError() != hipSuccess) return CP_ERR_HIP;
    }
    if (whole)
        rc = run_whole_sort(s, st);
    else if (buckets)
        rc = run_bucket_sort(s, a, st);
    else if (sort_threads(s.n) == kSortThreadsLong)
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
