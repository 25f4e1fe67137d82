// Streamed resident-window sweep: the resident-window plan without the graph in LDS.
//
// In the resident-window kernel dedicated loader wavefronts copy every tick's packet (slice
// descriptors, vertex records, entries) through an LDS stage, and the compute wavefronts read
// it back: three dependent LDS round trips (descriptor, then record and entries, then the ring)
// before the first relaxation, and a third of the kernel's LDS traffic.  Here compute
// wavefront j owns slice j of every tick and fetches that slice's descriptor, records and
// entries straight from global memory into registers, two ticks ahead; what goes through LDS
// is only what depends on the partition: the ring of recent values, the tick's device ids
// (and, for the mask, its b values), and the cost tables.  The recurrences are those of the
// other plans (b-level: the PCT equation of section 4.1; t-level: the downward rank of
// section 3.2 without the own term; mask: tl + b = CP).
//
// Needs: a packed ring of 32-bit ticks, 4-byte entries, no far reads, at most
// kWindowTickSlices slices per tick (one per compute wavefront).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_math.hpp"
#include "launch.hpp"

namespace cpeval {
namespace {

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

struct StreamArgs {
    const uint8_t *stream;     // tick packets
    const uint4 *slice_tab;    // [ticks][smax][2]: {record chunk, entry chunk, width | rows << 16 | log2(lanes per row) << 24,
                               //                    lowest vertex id of the tick} {ring slot of row 0, 0, 0, 0}
    const uint32_t *tick_tab;  // [ticks+1][4] {first chunk, chunks, lowest vertex id, id span}
    const uint8_t *ids;        // direct: the caller's assignments[P][n]; else [P][ticks*wpad] ids in sweep order
    int64_t ids_row;           // bytes between the rows of two partitions
    int32_t *out;              // ticks of (v, q) at v * out_sv + q * out_sq, or NULL
    int64_t *cp_out;           // [P] or NULL
    const Magic *edge_tab;
    const Magic *vert_tab;
    int32_t *status;
    int64_t out_sq;
    uint32_t out_sv;
    int32_t out32;             // every byte offset inside a partition's outputs fits 32 bits
    int32_t P, L, k, slots, wpad, smax, idpad, direct;   // L counts ticks
    int32_t nc, nlw;           // compute and loader wavefronts
    int32_t per_xcd;           // workgroups per XCD
    uint32_t stage_off, tab_off;   // LDS byte offsets of the stage slots and the cost tables
    // t sweep that also writes the critical-vertex mask (partition-major rows only)
    const int32_t *bvals;      // b [P][n]
    const int64_t *cp_in;      // [P]
    uint32_t *mask32;          // mask rows as 32-bit words, zeroed by the caller
    int64_t mask_row32;        // 32-bit words per mask row
    int64_t n;
    int32_t bpad;              // bytes a stage slot reserves for the tick's b values
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;

// What a compute wavefront holds of one slice: fetched two ticks before it is used.
template <int E>
struct SliceRegs {
    uint2 rc;            // {vertex, c} of this lane's row
    uint32_t e[E];       // entries: ring byte offset | t << 16
    // uniform
    int width, rows, lsh;
    uint32_t lo;
    int rbase;
    uint32_t ent_chunk;
};

// LDS: [ring: (R+1) x {value, 8 * device}][2 stage slots][cost tables]; a stage slot is
// [idpad bytes of device ids][bpad bytes of b values].  Wavefronts 0..nc-1 compute,
// nc..nc+nlw-1 stage the per-partition bytes of tick t+1 while tick t runs.
template <bool TSWEEP, int E, bool MASK, int NL, int DR>
__global__ __launch_bounds__(kWindowMaxWaves * 64) void window_stream_kernel(StreamArgs a) {
    extern __shared__ uint4 lds16[];
    __shared__ long long red[kWindowMaxWaves];
    __shared__ uint32_t mbits[MASK ? 2 : 1][MASK ? kMaskWords : 1];   // critical vertices of two ticks in flight
    uint8_t *lds = (uint8_t *)lds16;
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = a.k, L = a.L, R = a.slots;

    // blocks are dealt round-robin to the 8 XCDs; each XCD gets a run of consecutive partitions
    const int32_t q = (int32_t)(blockIdx.x % 8) * a.per_xcd + (int32_t)(blockIdx.x / 8);
    if (q >= a.P) return;      // whole workgroup: no barrier has been reached yet

    const uint32_t etab_off = a.tab_off, vtab_off = a.tab_off + 8u * (uint32_t)(k * k);
    const int slot_bytes = NL * a.nlw * 1024;
    uint8_t *stage = lds + a.stage_off;
    {
        const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
        uint64_t *t64 = (uint64_t *)(lds + etab_off);
        for (int i = tid; i < k * k; i += nt) t64[i] = e[i];
        for (int i = tid; i < k; i += nt) t64[k * k + i] = v[i];
        if constexpr (MASK)
            for (int i = tid; i < 2 * kMaskWords; i += nt) (&mbits[0][0])[i] = 0;
        if (tid == 0) ((uint2 *)lds)[R] = make_uint2(0, 0);    // the constant-zero slot padding entries point at
    }
    const int id16 = a.idpad / 16;               // 16-byte chunks of a slot that hold device ids
    uint32_t best = 0;

    if (wave >= a.nc) {
        // ------------------------------------------------ loader wavefronts
        constexpr int Lstep = DR;
        const int Lpad = (L + Lstep - 1) / Lstep * Lstep;
        const int lw = wave - a.nc;
        const_u32_ptr tick_tab = (const_u32_ptr)a.tick_tab;
        int cid[NL];
        const uint4 *base[NL];
        bool is_b[NL];
        const uint8_t *row = a.ids + (size_t)q * a.ids_row;
        // direct staging starts at the 16-byte boundary below the tick's lowest id
        const uint32_t row_mis = a.direct ? (uint32_t)((uintptr_t)row & 15) : 0u;
        const uint8_t *brow = MASK ? (const uint8_t *)a.bvals + (size_t)q * (size_t)a.n * 4 : nullptr;
        const uint32_t brow_mis = (uint32_t)((uintptr_t)brow & 15);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            cid[i] = (i * a.nlw + lw) * 64 + lane;
            is_b[i] = MASK && cid[i] >= id16;
            base[i] = is_b[i] ? (const uint4 *)(brow - brow_mis) : (const uint4 *)(row - row_mis);
        }
        u32x4 buf[DR][NL];
        // every lane always loads: chunks past the end of the ids or of the b values re-read the
        // last chunk of that part
#define CP_ISSUE(R_, S_)                                                                        \
    do {                                                                                        \
        const int s_ = min((S_), L - 1);                                                        \
        const u32x4 tt_ = *(const u32x4 __attribute__((address_space(4))) *)(tick_tab + 4 * s_); \
        const uint32_t lo_ = tt_.z, span_ = tt_.w;                                              \
        int id_first_, id_last_;                                                                \
        if (a.direct) {                                                                         \
            id_first_ = (int)((row_mis + lo_) >> 4);                                            \
            id_last_ = (int)((row_mis + lo_ + span_ - 1) >> 4) - id_first_;                     \
        } else {                                                                                \
            id_first_ = s_ * (a.wpad / 16);                                                     \
            id_last_ = a.wpad / 16 - 1;                                                         \
        }                                                                                       \
        int b_first_ = 0, b_last_ = 0;                                                          \
        if (MASK) {                                                                             \
            b_first_ = (int)((brow_mis + 4u * lo_) >> 4);                                       \
            b_last_ = (int)((brow_mis + 4u * (lo_ + span_) - 1) >> 4) - b_first_;               \
        }                                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                     \
            int c_ = min(cid[i_], id_last_) + id_first_;                                        \
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
        lds_barrier();                       // the bytes of tick 0 are staged
        for (int t0 = 0; t0 < Lpad; t0 += DR) {
#pragma unroll
            for (int r = 0; r < DR; ++r) {
                const int t = t0 + r;
                lds_barrier();
                // the compute wavefronts now read slot t&1, which tick t-1 has left (past the
                // last tick the last tick's bytes are staged again: nobody reads them)
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
        __builtin_amdgcn_s_setprio(1);
        const int j = wave;                                  // this wavefront's slice of every tick
        int32_t *out = a.out ? a.out + (size_t)q * (size_t)a.out_sq : nullptr;
        const uint32_t out_sv = a.out_sv;
        const uint32_t k8 = 8u * (uint32_t)k;
        const uint32_t row_mis = a.direct ? (uint32_t)((uintptr_t)(a.ids + (size_t)q * a.ids_row) & 15) : 0u;
        const uint32_t brow_mis = MASK ? (uint32_t)(((uintptr_t)a.bvals + (size_t)q * (size_t)a.n * 4) & 15) : 0u;
        const uint32_t cpq = MASK ? (uint32_t)a.cp_in[q] : 0u;   // tl + b <= CP: no overflow in 32 bits
        uint32_t worst = 0;                                  // largest device id seen
        const int Lpad = (L + DR - 1) / DR * DR;             // barriers the loaders take (DR is even)
        static_assert(DR % 2 == 0, "the compute loop takes two ticks per trip");

        // the descriptor of slice j of tick s: every lane loads the same 32 bytes (the table
        // goes on past the last tick with empty slices, so the loop below needs no end test:
        // a fixed number of loads and stores per trip lets the waits on the fetches count them)
        auto desc_load = [&](int s, uint4 &d0, uint4 &d1) {
            const uint4 *p = a.slice_tab + ((size_t)s * (size_t)a.smax + (size_t)j) * 2;
            d0 = p[0];
            d1 = p[1];
        };
        // the records and entries the descriptor names
        auto slice_load = [&](SliceRegs<E> &s, const uint4 &d0, const uint4 &d1) {
            const uint32_t rec_chunk = (uint32_t)__builtin_amdgcn_readfirstlane((int)d0.x);
            s.ent_chunk = (uint32_t)__builtin_amdgcn_readfirstlane((int)d0.y);
            const uint32_t meta = (uint32_t)__builtin_amdgcn_readfirstlane((int)d0.z);
            s.lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)d0.w);
            s.rbase = __builtin_amdgcn_readfirstlane((int)d1.x);
            s.width = (int)(meta & 0xffffu);
            s.rows = (int)((meta >> 16) & 0xffu);
            s.lsh = (int)(meta >> 24);
            s.rc = *((const uint2 *)(a.stream + 16 * (size_t)rec_chunk) + (lane >> s.lsh));
            const uint32_t *ent = (const uint32_t *)(a.stream + 16 * (size_t)s.ent_chunk) + lane;
            // always E loads: past the slice's width they read what follows in the stream
#pragma unroll
            for (int i = 0; i < E; ++i) s.e[i] = ent[i * 64];
        };

        // One slice out of registers: relaxes its rows and publishes its vertices, then fetches the
        // slice two ticks on into the same registers (and the descriptor four ticks on).  The
        // fetches come last: issuing them costs the wavefront a few hundred cycles, which are
        // better spent after the ring has its values (measured: 1.71 against 1.85 ms per b sweep
        // of the large sparse workload with the fetches before the publication).
        auto run_slice = [&](SliceRegs<E> &s, int t, uint4 &d0, uint4 &d1) {
            const int width = s.width, lsh = s.lsh, rows = s.rows, rbase = s.rbase;
            const uint8_t *st = stage + (size_t)(t & 1) * slot_bytes;
            const uint32_t lo = s.lo;
            const uint2 rc = s.rc;
            const int p = j * 64 + (lane >> lsh);
            uint32_t pv = 0, bv = 0, acc = 0, erow = 0;
            Magic mv{0, 0};
            if (rows != 0) {
            // the vertex's own device id: byte (v - lo) of the staged id range (padding rows
            // carry v = lo, so every lane reads a staged byte), or position p of the gathered row
            pv = st[a.direct ? rc.x - lo + ((row_mis + lo) & 15u) : (uint32_t)p];
            if (MASK) bv = *(const uint32_t *)(st + a.idpad + 4u * (rc.x - lo) + ((brow_mis + 4u * lo) & 15u));
            // N relaxations as one straight-line block: N ring reads beside the own id, N
            // cost-table reads beside the own table entry, then the arithmetic
#define CP_HEAD(N)                                                                              \
    do {                                                                                        \
        uint2 rg_[N + 1];                                                                       \
        Magic mg_[N + 1];                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) rg_[i_] = *(const uint2 *)(lds + (s.e[i_] & 0xffffu)); \
        worst = max(worst, pv);                                                                 \
        pv = min(pv, (uint32_t)(k - 1));                                                        \
        erow = etab_off + __umul24(pv, k8);                                                     \
        mv = *(const Magic *)(lds + vtab_off + 8u * pv);                                        \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) mg_[i_] = *(const Magic *)(lds + erow + rg_[i_].y); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_)                                        \
            acc = max(acc, rg_[i_].x + magic_div(s.e[i_] >> 16, mg_[i_]));                      \
    } while (0)
#define CP_MORE(FROM, N)                                                                        \
    do {                                                                                        \
        uint2 rg_[N];                                                                           \
        Magic mg_[N];                                                                           \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) rg_[i_] = *(const uint2 *)(lds + (s.e[FROM + i_] & 0xffffu)); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) mg_[i_] = *(const Magic *)(lds + erow + rg_[i_].y); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_)                                        \
            acc = max(acc, rg_[i_].x + magic_div(s.e[FROM + i_] >> 16, mg_[i_]));               \
    } while (0)
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
            if constexpr (E > 8) {
                switch (min(width, 16) - 8) {
                    case 1: CP_MORE(8, 1); break;
                    case 2: CP_MORE(8, 2); break;
                    case 3: CP_MORE(8, 3); break;
                    case 4: CP_MORE(8, 4); break;
                    case 5: CP_MORE(8, 5); break;
                    case 6: CP_MORE(8, 6); break;
                    case 7: CP_MORE(8, 7); break;
                    case 8: CP_MORE(8, 8); break;
                    default: break;
                }
            }
#undef CP_HEAD
#undef CP_MORE
            // rows wider than the registers hold: the rest of their entries straight from memory
            if (width > E) {
                const uint32_t *ent = (const uint32_t *)(a.stream + 16 * (size_t)s.ent_chunk) + lane;
                for (int jj = E; jj < width; ++jj) {
                    const uint32_t en = ent[jj * 64];
                    const uint2 rg = *(const uint2 *)(lds + (en & 0xffffu));
                    const Magic mg = *(const Magic *)(lds + erow + rg.y);
                    acc = max(acc, rg.x + magic_div(en >> 16, mg));
                }
            }
            // fold the lanes of a row; afterwards the row's first lane holds the row's maximum
            if (lsh >= 1) acc = max(acc, (uint32_t)__shfl_xor((int)acc, 1));
            if (lsh >= 2) acc = max(acc, (uint32_t)__shfl_xor((int)acc, 2));
            if (lsh >= 3) acc = max(acc, (uint32_t)__shfl_xor((int)acc, 4));
            if (lsh >= 4) acc = max(acc, (uint32_t)__shfl_xor((int)acc, 8));
            if (lsh >= 5) acc = max(acc, (uint32_t)__shfl_xor((int)acc, 16));
            if (lsh >= 6) acc = max(acc, (uint32_t)__shfl_xor((int)acc, 32));
            // the row's first lane publishes the vertex: ring, output, running maximum, mask bit
            const int row = lane >> lsh;
            const bool first = lsh == 0 || (lane & ((1 << lsh) - 1)) == 0;
            if (row < rows && first) {
                const uint32_t fin = acc + magic_div(rc.y, mv);      // b(v), or tl(v) + w(v)
                int rs = rbase + row;
                if (rs >= R) rs -= R;
                ((uint2 *)lds)[rs] = make_uint2(fin, 8u * pv);
                if (out) {
                    const int32_t o = (int32_t)(TSWEEP ? acc : fin);
                    if (a.out32) *(int32_t *)((char *)out + (__umul24(rc.x, out_sv) << 2)) = o;
                    else out[(size_t)rc.x * out_sv] = o;
                }
                best = max(best, fin);
                if constexpr (MASK) {        // tl(v) + b(v) = CP marks a critical vertex
                    if (acc + bv == cpq) {
                        const uint32_t rel = rc.x - (lo & ~31u);
                        atomicOr(&mbits[t & 1][rel >> 5], 1u << (rel & 31u));
                    }
                }
            }
            }
            slice_load(s, d0, d1);
            desc_load(t + 4, d0, d1);
        };

        // Two ticks lie between every fetch and its use (descriptors four ticks ahead, records and
        // entries two), so that a wait on a fetch leaves the other parity's fetches, and with
        // them the stores issued since, in flight.
        SliceRegs<E> s0, s1;
        uint4 da0, da1, db0, db1;
        // (the start-up issues its fetches in the loop's order: the waits inside the loop are
        // counted along both ways into it)
        desc_load(0, da0, da1);
        slice_load(s0, da0, da1);
        desc_load(1, db0, db1);
        desc_load(2, da0, da1);
        slice_load(s1, db0, db1);
        desc_load(3, db0, db1);
        lds_barrier();                       // the bytes of tick 0 are staged
        for (int t = 0; t < Lpad; t += 2) {
            lds_barrier();
            run_slice(s0, t, da0, da1);          // and fetches tick t + 2
            lds_barrier();
            run_slice(s1, t + 1, db0, db1);      // ... tick t + 3
        }
        if (worst >= (uint32_t)k) *a.status = CP_STATUS_BAD_DEVICE_ID;
        if (MASK) lds_barrier();             // pairs with the loaders' barrier before the last flush
    }

    if (a.cp_out) {   // the partition's maximum
        long long b64 = (long long)best;
        for (int off = 32; off > 0; off >>= 1) b64 = max(b64, __shfl_xor(b64, off));
        if (lane == 0) red[wave] = b64;
        lds_barrier();
        if (wave == 0 && lane == 0) {
            for (int w2 = 1; w2 < a.nc; ++w2) b64 = max(b64, red[w2]);
            a.cp_out[q] = b64;
        }
    }
}

inline int hip_ok(hipError_t e) { return e == hipSuccess ? CP_OK : CP_ERR_HIP; }

template <bool TSWEEP, int E, bool MASK, int NL, int DR>
int launch_stream_k(const SweepLaunch &s, const StreamCfg &cfg, hipStream_t st) {
    const WindowDir &dir = *s.win;
    StreamArgs a{};
    a.stream = s.blob + dir.stream_off;
    a.slice_tab = (const uint4 *)(s.blob + dir.stab_off);
    a.tick_tab = (const uint32_t *)(s.blob + dir.tick_off);
    a.direct = s.direct_ids ? 1 : 0;
    a.ids = s.direct_ids ? s.assign : s.pperm;
    a.ids_row = s.direct_ids ? s.a_stride_p : (int64_t)dir.ticks * dir.wpad;
    a.out = (int32_t *)s.val;
    a.cp_out = s.cp_out;
    a.edge_tab = (const Magic *)s.edge_tab;
    a.vert_tab = (const Magic *)s.vert_tab;
    a.status = s.status;
    a.out_sq = s.out_sq;
    a.out_sv = (uint32_t)s.out_sv;
    a.out32 = s.n < (1 << 24) && s.out_sv < (1 << 24) && (uint64_t)s.n * (uint64_t)s.out_sv * 4 < (1ull << 32);
    a.P = s.P; a.L = dir.ticks; a.k = s.k; a.slots = dir.slots; a.wpad = dir.wpad; a.smax = dir.smax;
    a.idpad = dir.idpad;
    a.nc = cfg.nc; a.nlw = cfg.nlw;
    a.per_xcd = (s.P + 7) / 8;
    a.stage_off = (uint32_t)cfg.stage_off;
    a.tab_off = (uint32_t)cfg.tab_off;
    if (MASK) {
        a.bvals = (const int32_t *)s.mask_b;
        a.cp_in = s.mask_cp;
        a.mask32 = (uint32_t *)s.mask_out;
        a.mask_row32 = 2 * (((int64_t)s.n + 63) / 64);
        a.n = s.n;
        a.bpad = window_mask_bpad(dir);
    }
    auto kern = window_stream_kernel<TSWEEP, E, MASK, NL, DR>;
    if (cfg.lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)cfg.lds_bytes);
        if (e != hipSuccess) return CP_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * a.per_xcd)), dim3((cfg.nc + cfg.nlw) * 64), cfg.lds_bytes, st, a);
    return hip_ok(hipGetLastError());
}

template <bool TSWEEP, bool MASK>
int launch_stream_e(const SweepLaunch &s, const StreamCfg &cfg, hipStream_t st) {
    // one 16-byte load per loader lane and tick for the device ids alone, two with the b values
    if (cfg.wide) return MASK ? launch_stream_k<TSWEEP, 16, MASK, 2, 8>(s, cfg, st)
                              : launch_stream_k<TSWEEP, 16, MASK, 1, 8>(s, cfg, st);
    return MASK ? launch_stream_k<TSWEEP, 8, MASK, 2, 8>(s, cfg, st)
                : launch_stream_k<TSWEEP, 8, MASK, 1, 8>(s, cfg, st);
}

}  // namespace

bool stream_config(const WindowDir &d, int32_t k, size_t lds_limit, bool with_mask, StreamCfg &out) {
    if (!d.packed || !d.ent4 || d.far_cap > 0 || d.stab_off == 0 || d.smax > kWindowTickSlices) return false;
    if (with_mask && (!d.direct_ok || (d.idpad + 62) / 32 > kMaskWords)) return false;
    const size_t ring = align_up(((size_t)d.slots + 1) * 8, 16);
    const size_t tab = align_up(sizeof(Magic) * ((size_t)k * k + k), 16);
    const int64_t need = d.idpad / 16 + (with_mask ? window_mask_bpad(d) / 16 : 0);
    const int nl = with_mask ? 2 : 1;
    const int64_t nlw = (need + 64 * nl - 1) / (64 * nl);
    if (nlw > kWindowMaxWaves - d.smax) return false;
    StreamCfg c;
    c.wide = d.max_width > 8;
    c.nl = nl;
    c.nlw = (int)nlw;
    c.nc = d.smax;
    c.stage_off = ring;
    c.tab_off = ring + (size_t)2 * nl * nlw * 1024;
    c.lds_bytes = c.tab_off + tab;
    if (c.lds_bytes > lds_limit) return false;
    out = c;
    return true;
}

int launch_window_stream(const SweepLaunch &s, const StreamCfg &cfg, void *stream) {
    if (s.tick_bytes != 4) return CP_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (s.mask_out) {
        if (!s.tsweep || !s.direct_ids) return CP_ERR_ARG;
        return launch_stream_e<true, true>(s, cfg, st);
    }
    return s.tsweep ? launch_stream_e<true, false>(s, cfg, st) : launch_stream_e<false, false>(s, cfg, st);
}

}  // namespace cpeval
