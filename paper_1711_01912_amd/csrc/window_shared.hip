// Shared-window sweep: the resident-window plan for large batches.
//
// The resident-window kernel gives every partition a workgroup of its own, and every one of
// them loads, stages and reads the same tick packets.  Here one workgroup owns G consecutive
// partitions (G = 2 or 4) and walks the sweep once for all of them: one loader set and one
// pair of stage slots serve the group, a compute lane reads a packet entry once and relaxes
// the edge for all G partitions out of one wide ring read.  The recurrences are the same
// (b-level: the PCT equation of section 4.1; t-level: the downward rank of section 3.2 without
// the own term).
//
// LDS: [device ids of the ring, (R+1) x G bytes][values of the ring, (R+1) x G ticks]
//      [2 stage slots][cost tables].  A stage slot is [G x idpad bytes of device ids][packet].
// With far reads (neighbours computed too long ago to be kept in the ring: see the resident-window
// kernel) both ring regions go on behind slot R with two sets of far_cap slots, one per tick
// parity, which far wavefronts fill from the output rows: an entry's field / 8 is a slot number
// either way.
// The packets are the resident-window plan's (WindowDir with a packed ring: an entry's ring
// field is 8 x slot), read unchanged.
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

struct SharedArgs {
    const uint4 *stream;       // tick packets
    const uint32_t *tick_tab;  // [ticks+1][4] {first chunk, chunks, lowest vertex id, id span}
    const uint8_t *ids;        // direct: the caller's assignments[P][n]; else [P][ticks*wpad] ids in sweep order
    int64_t ids_row;           // bytes between the rows of two partitions
    int32_t *out;              // ticks of (v, q) at v * out_sv + q * out_sq, or NULL
    int64_t *cp_out;           // [P] or NULL
    const Magic *edge_tab;
    const Magic *vert_tab;
    const uint32_t *edge_tab4; // TAB4: the same tables as 4-byte entries
    const uint32_t *vert_tab4;
    int32_t tab_rs;            // TAB4: every transfer entry sits 2^tab_rs times in LDS
    int32_t *status;
    int64_t out_sq;
    uint32_t out_sv;
    int32_t P, L, k, slots, wpad, smax, idpad, direct;   // L counts ticks
    int32_t nc, nlw;           // compute and loader wavefronts
    int32_t wgs, per_xcd;      // workgroups with partitions; workgroups per XCD
    uint32_t vals_off, stage_off, tab_off;   // LDS byte offsets
    int32_t out32;             // every output index fits 32 bits
    // t sweep that also writes the critical-vertex mask (rows per partition): b with the strides of
    // `out`, CP per partition, the zeroed mask rows as 32-bit words; all null otherwise
    const int32_t *mask_b;
    const int64_t *mask_cp;
    uint32_t *mask32;
    int64_t mask_row32;        // 32-bit words per mask row
    // far reads: {vertex, c} per tick and read; the caller's assignments, device of (v, q) at
    // v * far_a_sv + q * far_a_sp; reads per tick (a multiple of 64); far wavefronts (after the
    // loaders); output stores a compute wavefront issues per tick
    const uint2 *far_list;
    const uint8_t *far_assign;
    int64_t far_a_sp, far_a_sv;
    int32_t far_cap, nfw, stores_per_tick;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;

template <int G> struct GroupVals;
template <> struct GroupVals<2> { typedef uint2 type; };
template <> struct GroupVals<4> { typedef uint4 type; };

template <int G>
__device__ __forceinline__ uint32_t val_of(const typename GroupVals<G>::type &v, int g) {
    if constexpr (G == 2) return g == 0 ? v.x : v.y;
    else return g == 0 ? v.x : (g == 1 ? v.y : (g == 2 ? v.z : v.w));
}

// Wavefronts 0..nc-1 compute, nc..nc+nlw-1 load.  Tick t: after the barrier the compute
// wavefronts relax the tick out of stage slot t&1 while the loaders copy packet t+1
// (requested DR ticks earlier, held in registers) into the other slot and request packet
// t+1+DR.
//
// TAB4: the cost tables are 4-byte entries and every transfer entry sits 2^tab_rs times in LDS,
// copy r in bank (r mod 32); lane l reads copy l mod 2^tab_rs: fewer lanes meet in a bank.
template <bool TSWEEP, int G, bool ENT4, int NL, int DR, bool TAB4, bool FAR>
__global__ __launch_bounds__(kWindowMaxWaves * 64) void window_shared_kernel(SharedArgs a) {
    typedef typename std::conditional<TAB4, uint32_t, Magic>::type Tab;
    extern __shared__ uint4 lds16[];
    __shared__ long long red[G][kWindowMaxWaves];
    uint8_t *lds = (uint8_t *)lds16;
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = a.k, L = a.L, R = a.slots;
    // ring: slot s holds G device bytes at s*G and G ticks at vals_off + s*4G; an entry's
    // field is 8*s
    constexpr int kDevShift = G == 4 ? 1 : 2;    // field >> kDevShift = s*G
    constexpr int kValShift = G == 4 ? 1 : 0;    // field << kValShift = s*4G
    typedef typename GroupVals<G>::type Vals;
    typedef typename std::conditional<G == 4, uint32_t, uint16_t>::type Devs;

    // blocks are dealt round-robin to the 8 XCDs; each XCD gets a run of consecutive groups
    const int32_t wg = (int32_t)(blockIdx.x % 8) * a.per_xcd + (int32_t)(blockIdx.x / 8);
    if (wg >= a.wgs) return;   // whole workgroup: no barrier has been reached yet
    // a last group that is not full repeats its last partition (same values to the same places)
    int32_t q[G];
#pragma unroll
    for (int g = 0; g < G; ++g) q[g] = min(wg * G + g, a.P - 1);

    const int dev_sh = TAB4 ? 2 + a.tab_rs : 3;          // bytes between the entries of two devices, as a shift
    const uint32_t etab_off = a.tab_off, vtab_off = a.tab_off + ((uint32_t)(k * k) << dev_sh);
    const int slot_bytes = NL * a.nlw * 1024;
    uint8_t *stage = lds + a.stage_off;
    {
        if constexpr (TAB4) {
            uint32_t *t32 = (uint32_t *)(lds + etab_off);
            const int copies = k * k << a.tab_rs;
            for (int i = tid; i < copies; i += nt) t32[i] = a.edge_tab4[i >> a.tab_rs];
            for (int i = tid; i < k; i += nt) t32[copies + i] = a.vert_tab4[i];
        } else {
            const uint64_t *e = (const uint64_t *)a.edge_tab, *v = (const uint64_t *)a.vert_tab;
            uint64_t *t64 = (uint64_t *)(lds + etab_off);
            for (int i = tid; i < k * k; i += nt) t64[i] = e[i];
            for (int i = tid; i < k; i += nt) t64[k * k + i] = v[i];
        }
        if (tid < G) {                           // the constant-zero slot padding entries point at
            lds[(size_t)R * G + tid] = 0;
            ((uint32_t *)(lds + a.vals_off))[(size_t)R * G + tid] = 0;
        }
    }
    // ticks rounded up so that the loaders' and the far wavefronts' unrolled loops end together
    constexpr int kStep = !FAR ? DR : (DR % kWindowFarLead == 0 ? DR : DR * kWindowFarLead / (DR % 2 == 0 ? 2 : 1));
    static_assert(kStep % DR == 0 && (!FAR || kStep % kWindowFarLead == 0), "tick padding");
    const int Lpad = (L + kStep - 1) / kStep * kStep;
    // first far slot: behind the ring as the packer laid it out (pairs of 8 bytes, 16-byte aligned)
    const uint32_t far0 = (uint32_t)((((size_t)R + 1) * 8 + 15) / 16 * 2);
    const int id16 = a.idpad / 16;               // 16-byte chunks of device ids per partition and slot
    const int head = G * a.idpad;                // bytes of a slot before the packet
    uint32_t best[G];
#pragma unroll
    for (int g = 0; g < G; ++g) best[g] = 0;

    if (FAR && wave >= a.nc + a.nlw) {
        // ------------------------------------------------ far wavefronts
        // Lane f of far wavefront fw owns far read number fw*64 + f of every tick, for all G
        // partitions.  For tick tau its {vertex, c} is loaded 2*X + 1 steps ahead, the values and
        // devices of that vertex X + 1 steps ahead (from the output rows: the vertex was published
        // at least kWindowFarTicks ticks before tau, and the compute wavefronts wait for their
        // older stores before each barrier), and the slot is written one step ahead.
        constexpr int X = kWindowFarLead;
        const int f = (wave - a.nc - a.nlw) * 64 + lane;
        const int32_t *outq[G];
        const uint8_t *arow[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            outq[g] = a.out + (size_t)q[g] * (size_t)a.out_sq;
            arow[g] = a.far_assign + (size_t)q[g] * (size_t)a.far_a_sp;
        }
        const Tab *vtab = (const Tab *)(lds + vtab_off);
        bool bad = false;
        struct Got { uint32_t val[G], devs; };
        auto list_load = [&](int tau) -> uint2 {
            return a.far_list[(size_t)min(tau, L - 1) * (size_t)a.far_cap + f];
        };
        auto fetch = [&](uint2 e) -> Got {
            Got r;
            r.devs = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                // the value left this compute unit through its write-through cache: read it from L2
                uint32_t val = (uint32_t)__hip_atomic_load(outq[g] + (size_t)e.x * a.out_sv, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
                uint32_t dev = arow[g][(size_t)e.x * (size_t)a.far_a_sv];
                if (dev >= (uint32_t)k) { bad = true; dev = (uint32_t)k - 1; }
                if (TSWEEP) val += magic_div(e.y, vtab[dev]);       // the ring holds tl + w
                r.val[g] = val;
                r.devs |= dev << (8 * g);
            }
            return r;
        };
        uint2 lst[X];
        Got got[X];
#pragma unroll
        for (int j = 1; j <= X; ++j) {
            lst[j % X] = list_load(j + X);
            got[j % X].devs = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) got[j % X].val[g] = 0;
        }
        lds_barrier();                       // pairs with "packet 0 is staged"
        for (int t0 = 0; t0 < Lpad; t0 += X) {
#pragma unroll
            for (int r = 0; r < X; ++r) {
                const int t = t0 + r;
                lds_barrier();
                const int sl = (r + 1) % X;
                const uint32_t slot = far0 + (uint32_t)((t + 1) & 1) * (uint32_t)a.far_cap + (uint32_t)f;
                *(Devs *)(lds + (size_t)slot * G) = (Devs)got[sl].devs;
                Vals fv;
                if constexpr (G == 2) fv = make_uint2(got[sl].val[0], got[sl].val[1]);
                else fv = make_uint4(got[sl].val[0], got[sl].val[1], got[sl].val[2], got[sl].val[3]);
                *(Vals *)(lds + a.vals_off + (size_t)slot * (4 * G)) = fv;
                got[sl] = fetch(lst[sl]);                 // for tick t + 1 + X
                lst[sl] = list_load(t + 1 + 2 * X);
            }
        }
        if (bad) *a.status = CP_STATUS_BAD_DEVICE_ID;
    } else if (wave >= a.nc) {
        // ------------------------------------------------ loader wavefronts
        const int lw = wave - a.nc;
        const_u32_ptr tick_tab = (const_u32_ptr)a.tick_tab;
        int cid[NL], cidl[NL];
        const uint4 *base[NL];
        bool is_id[NL];
        uint32_t mis[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            cid[i] = (i * a.nlw + lw) * 64 + lane;
            is_id[i] = cid[i] < G * id16;
            const int g = is_id[i] ? cid[i] / id16 : 0;
            cidl[i] = cid[i] - g * id16;
            int32_t qg = q[0];
#pragma unroll
            for (int gg = 1; gg < G; ++gg) qg = g == gg ? q[gg] : qg;
            const uint8_t *row = a.ids + (size_t)qg * a.ids_row;
            // direct staging starts at the 16-byte boundary below the tick's lowest id
            mis[i] = a.direct ? (uint32_t)((uintptr_t)row & 15) : 0u;
            base[i] = is_id[i] ? (const uint4 *)(row - mis[i]) : a.stream;
        }
        u32x4 buf[DR][NL];
        // every lane always loads: chunks past the end of the ids or of the packet re-read
        // the last chunk of that part
#define CP_ISSUE(R_, S_)                                                                        \
    do {                                                                                        \
        const int s_ = min((S_), L - 1);                                                        \
        const u32x4 tt_ = *(const u32x4 __attribute__((address_space(4))) *)(tick_tab + 4 * s_); \
        const uint32_t o0_ = tt_.x, oc_ = tt_.y, lo_ = tt_.z, span_ = tt_.w;                    \
        const int pk_last_ = G * id16 + (int)oc_ - 1, off_pk_ = (int)o0_ - G * id16;            \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                     \
            int c_;                                                                             \
            if (is_id[i_]) {                                                                    \
                int first_, last_;                                                              \
                if (a.direct) {                                                                 \
                    first_ = (int)((mis[i_] + lo_) >> 4);                                       \
                    last_ = (int)((mis[i_] + lo_ + span_ - 1) >> 4) - first_;                   \
                } else {                                                                        \
                    first_ = s_ * (a.wpad / 16);                                                \
                    last_ = a.wpad / 16 - 1;                                                    \
                }                                                                               \
                c_ = min(cidl[i_], last_) + first_;                                             \
            } else {                                                                            \
                c_ = min(cid[i_], pk_last_) + off_pk_;                                          \
            }                                                                                   \
            buf[R_][i_] = *(const u32x4 *)(base[i_] + c_);                                      \
        }                                                                                       \
    } while (0)
#define CP_STORE(R_, SLOT_)                                                                     \
    do {                                                                                        \
        u32x4 *dst_ = (u32x4 *)(stage + (size_t)(SLOT_) * slot_bytes);                          \
        _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) dst_[cid[i_]] = buf[R_][i_];          \
    } while (0)
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
            }
        }
#undef CP_ISSUE
#undef CP_STORE
    } else {
        // ------------------------------------------------ compute wavefronts
        __builtin_amdgcn_s_setprio(1);
        typedef typename std::conditional<ENT4, uint32_t, uint2>::type Ent;
        const uint32_t out_sv = a.out_sv;
        const uint32_t k8 = (uint32_t)k << dev_sh;        // bytes of one table row
        const uint32_t copy_off = TAB4 ? 4u * ((uint32_t)lane & ((1u << a.tab_rs) - 1u)) : 0u;   // this lane's copy
        const uint32_t rec_off = (uint32_t)head + 16u * (uint32_t)a.smax;   // records, from the slot base
        const uint32_t vals_off = a.vals_off;
        int32_t *outq[G];
        uint32_t row_mis[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            outq[g] = a.out ? a.out + (size_t)q[g] * (size_t)a.out_sq : nullptr;
            row_mis[g] = a.direct ? (uint32_t)((uintptr_t)(a.ids + (size_t)q[g] * a.ids_row) & 15) : 0u;
        }
        uint32_t worst = 0;                  // largest device id seen
        // Mask (t sweep): tl(v) + b(v) = CP marks a critical vertex.  b(v) comes from the b array in
        // global memory: the lane that publishes v asks for it right after, and compares two ticks
        // later, at the start of its slice; even and odd ticks keep their requests apart, so that
        // the wait for one tick's values leaves the next tick's in flight.
        const bool with_mask = TSWEEP && a.mask32 != nullptr;
        struct Pending {
            bool on = false;                 // this lane published v
            uint32_t v = 0, tl[G], b[G];
        } pend_even, pend_odd;
        uint32_t cpq[G];
        const int32_t *bq[G];
        uint32_t *mq[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            pend_even.tl[g] = pend_even.b[g] = pend_odd.tl[g] = pend_odd.b[g] = 0;
            cpq[g] = with_mask ? (uint32_t)a.mask_cp[q[g]] : 0u;      // tl + b <= CP: no overflow in 32 bits
            bq[g] = with_mask ? a.mask_b + (size_t)q[g] * (size_t)a.out_sq : nullptr;
            mq[g] = with_mask ? a.mask32 + (size_t)q[g] * (size_t)a.mask_row32 : nullptr;
        }
        auto flush_pending = [&](const Pending &pd) {
            uint32_t hits = 0;               // critical vertices are rare: one branch for all G
#pragma unroll
            for (int g = 0; g < G; ++g) hits |= (uint32_t)(pd.tl[g] + pd.b[g] == cpq[g]) << g;
            if (pd.on && hits) {
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if ((hits >> g) & 1u) atomicOr(mq[g] + (pd.v >> 5), 1u << (pd.v & 31u));
            }
        };

        auto ent_field = [](Ent e) -> uint32_t {
            if constexpr (ENT4) return e & 0xffffu; else return e.x;
        };
        auto ent_t = [](Ent e) -> uint32_t {
            if constexpr (ENT4) return e >> 16; else return e.y;
        };
        // one slice of the current tick out of its stage slot, for all G partitions
        auto slice = [&](const uint8_t *st, int j, Pending &pd) {
            const uint4 d = ((const uint4 *)(st + head))[j];
            const uint32_t ent_off = d.x;
            const int width = __builtin_amdgcn_readfirstlane((int)(d.y & 0xffffu));
            const int lsh = __builtin_amdgcn_readfirstlane((int)(d.y >> 24));
            const int rows = (int)((d.y >> 16) & 0xffu);
            const uint32_t lo = d.z;
            const int rbase = (int)d.w;
            if (width == 0 && lsh == 0 && __builtin_amdgcn_readfirstlane(rows) == 0) return;   // (what is pending stays so)
            // the vertex of this lane's slice two ticks ago.  At the slice's start: the wait for its
            // b values is a wait for everything older, and must come before this slice's own
            // stores.  (The cost of the mask is instructions, not latency: comparing after one tick
            // instead of two costs 2 % more, comparing just before the publication 17 % more,
            // asking for b at the start of the slice 23 % more; 64-bit address arithmetic per
            // access instead of one 32-bit offset beside uniform row addresses 7 % more.)
            if constexpr (TSWEEP) {
                if (with_mask) flush_pending(pd);
            }
            const int p = j * 64 + (lane >> lsh);
            const uint2 rc = *((const uint2 *)(st + rec_off) + p);
            const Ent *ent = (const Ent *)(st + head + ent_off) + lane;
            uint32_t pv[G], erow[G], acc[G];
            Tab mv[G];
            // N relaxations for all G partitions as one straight-line block: N entry reads,
            // N reads of the G device ids and N of the G values, N*G cost-table reads, then
            // the arithmetic
#define CP_BLOCK(N)                                                                             \
    do {                                                                                        \
        Ent en_[N];                                                                             \
        Vals vu_[N];                                                                            \
        uint32_t du_[N];                                                                        \
        Tab mg_[N][G];                                                                          \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) en_[i_] = ent[(jj + i_) * 64];         \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_) {                                      \
            const uint32_t f_ = ent_field(en_[i_]);                                             \
            du_[i_] = *(const Devs *)(lds + (f_ >> kDevShift));                                 \
            vu_[i_] = *(const Vals *)(lds + vals_off + (f_ << kValShift));                      \
        }                                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_)                                        \
            _Pragma("unroll") for (int g_ = 0; g_ < G; ++g_)                                    \
                mg_[i_][g_] = *(const Tab *)(lds + erow[g_] + (((du_[i_] >> (8 * g_)) & 0xffu) << dev_sh)); \
        _Pragma("unroll") for (int i_ = 0; i_ < N; ++i_)                                        \
            _Pragma("unroll") for (int g_ = 0; g_ < G; ++g_)                                    \
                acc[g_] = max(acc[g_], val_of<G>(vu_[i_], g_) + magic_div(ent_t(en_[i_]), mg_[i_][g_])); \
    } while (0)
            // the vertex's own device ids: position p of the gathered rows, or byte (v - lo) of
            // the staged id ranges (padding rows carry v = lo, so every lane reads a staged byte)
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const uint32_t at = a.direct ? rc.x - lo + ((row_mis[g] + lo) & 15u) : (uint32_t)p;
                pv[g] = st[(uint32_t)g * (uint32_t)a.idpad + at];
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                worst = max(worst, pv[g]);
                pv[g] = min(pv[g], (uint32_t)(k - 1));
                erow[g] = etab_off + __umul24(pv[g], k8) + copy_off;
                mv[g] = *(const Tab *)(lds + vtab_off + (uint32_t)sizeof(Tab) * pv[g]);
                acc[g] = 0;
            }
            int jj = 0;
            for (; jj + 4 <= width; jj += 4) CP_BLOCK(4);
            switch (width - jj) {
                case 1: CP_BLOCK(1); break;
                case 2: CP_BLOCK(2); break;
                case 3: CP_BLOCK(3); break;
                default: break;
            }
#undef CP_BLOCK
            // fold the lanes of a row; afterwards the row's first lane holds the row's maxima
            if (lsh > 0) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    uint32_t x = acc[g];
                    if (lsh >= 1) x = max(x, (uint32_t)__shfl_xor((int)x, 1));
                    if (lsh >= 2) x = max(x, (uint32_t)__shfl_xor((int)x, 2));
                    if (lsh >= 3) x = max(x, (uint32_t)__shfl_xor((int)x, 4));
                    if (lsh >= 4) x = max(x, (uint32_t)__shfl_xor((int)x, 8));
                    if (lsh >= 5) x = max(x, (uint32_t)__shfl_xor((int)x, 16));
                    if (lsh >= 6) x = max(x, (uint32_t)__shfl_xor((int)x, 32));
                    acc[g] = x;
                }
            }
            const int row = lane >> lsh;
            const bool first = lsh == 0 || (lane & ((1 << lsh) - 1)) == 0;
            // (the requests for b go out before this slice's stores: the wait for them, two ticks on,
            // then leaves the stores issued since in flight, whatever their number)
            if constexpr (TSWEEP) {
                if (with_mask) {
                    pd.on = row < rows && first;
                    pd.v = rc.x;                 // padding rows carry a vertex of the tick: a valid index
#pragma unroll
                    for (int g = 0; g < G; ++g) pd.tl[g] = acc[g];
                    const uint32_t off = __umul24(rc.x, out_sv) << 2;      // (the launcher checked that it fits)
#pragma unroll
                    for (int g = 0; g < G; ++g) pd.b[g] = (uint32_t) * (const int32_t *)((const char *)bq[g] + off);
                }
            }
            // the row's first lane publishes the vertex: ring, output, running maxima
            if (row < rows && first) {
                int rs = rbase + row;
                if (rs >= R) rs -= R;
                uint32_t fin[G], devs = 0;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    fin[g] = acc[g] + magic_div(rc.y, mv[g]);      // b(v), or tl(v) + w(v)
                    devs |= pv[g] << (8 * g);
                    best[g] = max(best[g], fin[g]);
                }
                *(Devs *)(lds + (size_t)rs * G) = (Devs)devs;
                Vals fv;
                if constexpr (G == 2) fv = make_uint2(fin[0], fin[1]);
                else fv = make_uint4(fin[0], fin[1], fin[2], fin[3]);
                *(Vals *)(lds + vals_off + (size_t)rs * (4 * G)) = fv;
                if (a.out) {
                    if (a.out32) {               // one 32-bit byte offset beside G uniform row addresses
                        const uint32_t off = __umul24(rc.x, out_sv) << 2;
#pragma unroll
                        for (int g = 0; g < G; ++g)
                            *(int32_t *)((char *)outq[g] + off) = (int32_t)(TSWEEP ? acc[g] : fin[g]);
                    } else {
#pragma unroll
                        for (int g = 0; g < G; ++g) outq[g][(size_t)rc.x * out_sv] = (int32_t)(TSWEEP ? acc[g] : fin[g]);
                    }
                }
            }
        };
        // far reads take values from the output rows kWindowFarTicks ticks later: keep at most
        // two ticks' worth of stores in flight
        auto far_wait = [&]() {
            if constexpr (FAR) {
                const int pending = 2 * G * a.stores_per_tick;
                if (pending == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                else if (pending == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
                else if (pending == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        };
        lds_barrier();                       // packet 0 is staged
        for (int t = 0; t < Lpad; t += 2) {
            far_wait();
            lds_barrier();
            if (t < L) {
                const uint8_t *st = stage + (size_t)(t & 1) * slot_bytes;
                for (int j = wave; j < a.smax; j += a.nc) slice(st, j, pend_even);
            }
            if (t + 1 < Lpad) {
                far_wait();
                lds_barrier();
                if (t + 1 < L) {
                    const uint8_t *st = stage + (size_t)((t + 1) & 1) * slot_bytes;
                    for (int j = wave; j < a.smax; j += a.nc) slice(st, j, pend_odd);
                }
            }
        }
        if constexpr (TSWEEP) {              // the last two ticks' vertices
            if (with_mask) {
                flush_pending(pend_even);
                flush_pending(pend_odd);
            }
        }
        if (worst >= (uint32_t)k) *a.status = CP_STATUS_BAD_DEVICE_ID;
    }

    if (a.cp_out) {   // the partitions' maxima
#pragma unroll
        for (int g = 0; g < G; ++g) {
            long long b64 = (long long)best[g];
            for (int off = 32; off > 0; off >>= 1) b64 = max(b64, __shfl_xor(b64, off));
            if (lane == 0) red[g][wave] = b64;
        }
        lds_barrier();
        if (wave == 0 && lane < G) {
            long long b64 = 0;
            for (int w2 = 0; w2 < a.nc; ++w2) b64 = max(b64, red[lane][w2]);
            a.cp_out[min(wg * G + lane, a.P - 1)] = b64;
        }
    }
}

inline int hip_ok(hipError_t e) { return e == hipSuccess ? CP_OK : CP_ERR_HIP; }

template <bool TSWEEP, int G, bool ENT4, int NL, int DR, bool TAB4, bool FAR>
int launch_shared_k(const SweepLaunch &s, const SharedCfg &cfg, hipStream_t st) {
    const WindowDir &dir = *s.win;
    SharedArgs a{};
    a.stream = (const uint4 *)(s.blob + dir.stream_off);
    a.tick_tab = (const uint32_t *)(s.blob + dir.tick_off);
    a.direct = s.direct_ids ? 1 : 0;
    a.ids = s.direct_ids ? s.assign : s.pperm;
    a.ids_row = s.direct_ids ? s.a_stride_p : (int64_t)dir.ticks * dir.wpad;
    a.out = (int32_t *)s.val;
    a.cp_out = s.cp_out;
    a.edge_tab = (const Magic *)s.edge_tab;
    a.vert_tab = (const Magic *)s.vert_tab;
    a.edge_tab4 = s.edge_tab4;
    a.vert_tab4 = s.vert_tab4;
    a.tab_rs = cfg.tab_rs;
    if (TAB4 && (cfg.tab_rs < 0 || cfg.tab_rs > 5 || !s.edge_tab4 || !s.vert_tab4)) return CP_ERR_ARG;
    a.status = s.status;
    a.out_sq = s.out_sq;
    a.out_sv = (uint32_t)s.out_sv;
    a.P = s.P; a.L = dir.ticks; a.k = s.k; a.slots = dir.slots; a.wpad = dir.wpad; a.smax = dir.smax;
    a.idpad = dir.idpad;
    a.nc = cfg.nc; a.nlw = cfg.nlw;
    a.wgs = (s.P + G - 1) / G;
    a.per_xcd = (a.wgs + 7) / 8;
    a.vals_off = (uint32_t)cfg.vals_off;
    a.stage_off = (uint32_t)cfg.stage_off;
    a.tab_off = (uint32_t)cfg.tab_off;
    // every byte offset of a vertex inside a partition's row of outputs fits 32 bits (and both factors 24)
    a.out32 = s.n < (1 << 24) && s.out_sv < (1 << 24) && (uint64_t)s.n * (uint64_t)s.out_sv * 4 < (1ull << 32);
    if (s.mask_out) {
        if (!TSWEEP || !s.mask_b || !s.mask_cp || !s.val || cfg.nc < dir.smax || !a.out32) return CP_ERR_ARG;
        a.mask_b = (const int32_t *)s.mask_b;
        a.mask_cp = s.mask_cp;
        a.mask32 = (uint32_t *)s.mask_out;
        a.mask_row32 = 2 * (((int64_t)s.n + 63) / 64);
    }
    if (FAR != (dir.far_cap > 0) || cfg.nfw != dir.far_cap / kWave) return CP_ERR_ARG;
    if (FAR) {
        if (!s.val || s.mask_out) return CP_ERR_ARG;     // far reads come out of the output rows
        a.far_list = (const uint2 *)(s.blob + dir.far_off);
        a.far_assign = s.assign;
        a.far_a_sp = s.a_stride_p;
        a.far_a_sv = s.a_stride_v;
        a.far_cap = dir.far_cap;
        a.nfw = cfg.nfw;
        a.stores_per_tick = (dir.smax + cfg.nc - 1) / cfg.nc;
    }
    auto kern = window_shared_kernel<TSWEEP, G, ENT4, NL, DR, TAB4, FAR>;
    if (cfg.lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)cfg.lds_bytes);
        if (e != hipSuccess) return CP_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * a.per_xcd)), dim3((cfg.nc + cfg.nlw + cfg.nfw) * 64), cfg.lds_bytes, st, a);
    return hip_ok(hipGetLastError());
}

template <bool TSWEEP, int G, bool ENT4, bool TAB4, bool FAR>
int launch_shared_t(const SweepLaunch &s, const SharedCfg &cfg, hipStream_t st) {
    switch (cfg.nl) {   // loads per loader lane per tick x ticks in flight: 64 registers at most
        case 1: return launch_shared_k<TSWEEP, G, ENT4, 1, 8, TAB4, FAR>(s, cfg, st);
        case 2: return launch_shared_k<TSWEEP, G, ENT4, 2, 8, TAB4, FAR>(s, cfg, st);
        case 3: return launch_shared_k<TSWEEP, G, ENT4, 3, 5, TAB4, FAR>(s, cfg, st);
        case 4: return launch_shared_k<TSWEEP, G, ENT4, 4, 4, TAB4, FAR>(s, cfg, st);
        default: return CP_ERR_ARG;
    }
}

template <bool TSWEEP, int G, bool ENT4>
int launch_shared_e(const SweepLaunch &s, const SharedCfg &cfg, hipStream_t st) {
    if (s.win->far_cap > 0)                  // (far reads go with the 8-byte tables only)
        return cfg.tab_rs >= 0 ? CP_ERR_ARG : launch_shared_t<TSWEEP, G, ENT4, false, true>(s, cfg, st);
    return cfg.tab_rs >= 0 ? launch_shared_t<TSWEEP, G, ENT4, true, false>(s, cfg, st)
                           : launch_shared_t<TSWEEP, G, ENT4, false, false>(s, cfg, st);
}

template <bool TSWEEP>
int launch_shared_g(const SweepLaunch &s, const SharedCfg &cfg, hipStream_t st) {
    if (cfg.groups == 4)
        return s.win->ent4 ? launch_shared_e<TSWEEP, 4, true>(s, cfg, st) : launch_shared_e<TSWEEP, 4, false>(s, cfg, st);
    if (cfg.groups == 2)
        return s.win->ent4 ? launch_shared_e<TSWEEP, 2, true>(s, cfg, st) : launch_shared_e<TSWEEP, 2, false>(s, cfg, st);
    return CP_ERR_ARG;
}

}  // namespace

bool shared_config(const WindowDir &d, int32_t k, int groups, size_t lds_limit, SharedCfg &out, bool tab4) {
    if (!d.packed || (groups != 2 && groups != 4)) return false;
    const size_t G = (size_t)groups;
    // slots of either ring region: the ring and its constant-zero slot, then, with far reads, from
    // the 16-byte boundary behind them two sets of far_cap slots
    const int nfw = d.far_cap / kWave;
    const size_t nslots = d.far_cap > 0 ? (((size_t)d.slots + 1) * 8 + 15) / 16 * 2 + 2 * (size_t)d.far_cap
                                        : (size_t)d.slots + 1;
    const size_t devs = align_up(nslots * G, 16);
    const size_t vals = align_up(nslots * 4 * G, 16);
    const size_t tab = align_up(sizeof(Magic) * ((size_t)k * k + k), 16);
    // the entries' ring fields are read as LDS byte offsets of the device bytes and, doubled
    // at most, of the values: both regions lie below 2^32 trivially, the fields below 8 * (slots + 1)
    const int64_t need = (int64_t)G * (d.idpad / 16) + (int64_t)d.max_chunks;    // 16-byte chunks per stage slot
    static const int kNl[4] = {1, 2, 3, 4};
    for (int nl : kNl) {
        const int64_t nlw = (need + 64 * nl - 1) / (64 * nl);
        if (nlw > 8 || nlw + nfw > kWindowMaxWaves - 1) continue;
        SharedCfg c;
        c.groups = groups;
        c.nl = nl;
        c.nlw = (int)nlw;
        c.nfw = nfw;
        c.nc = std::max(1, std::min(d.smax, kWindowMaxWaves - (int)nlw - nfw));
        c.vals_off = devs;
        c.stage_off = devs + vals;
        c.tab_off = c.stage_off + (size_t)2 * nl * nlw * 1024;
        c.lds_bytes = c.tab_off + tab;
        if (c.lds_bytes > lds_limit) continue;
        // 4-byte cost tables with as many copies of every transfer entry as fit (up to one per
        // LDS bank): wide ticks only, as for the resident-window kernel
        for (int rs = 5; tab4 && d.far_cap == 0 && d.smax >= 4 && rs >= 2; --rs) {
            if (c.tab_off + tab4_lds_bytes(k, rs) <= lds_limit) {
                c.tab_rs = rs;
                c.lds_bytes = c.tab_off + tab4_lds_bytes(k, rs);
                break;
            }
        }
        out = c;
        return true;
    }
    return false;
}

int launch_window_shared(const SweepLaunch &s, const SharedCfg &cfg, void *stream) {
    if (s.tick_bytes != 4 || (s.mask_out && !s.tsweep)) return CP_ERR_ARG;
    return s.tsweep ? launch_shared_g<true>(s, cfg, (hipStream_t)stream)
                    : launch_shared_g<false>(s, cfg, (hipStream_t)stream);
}

}  // namespace cpeval
