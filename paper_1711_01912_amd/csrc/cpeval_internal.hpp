// Internal declarations shared by the host-side graph packer, the cost-table
// builder and the kernel launchers.  Nothing here is part of the C ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/cpeval.h"

namespace cpeval {

constexpr int kWave = 64;              // wavefront width on gfx950
constexpr int kHubDegree = 256;        // wave-column plan: rows this long get a whole workgroup
constexpr int kHubWaves = 16;          // ... of this many wavefronts
constexpr int kMagicMaxK = 64;         // multiply-shift tables are staged in LDS up to this many devices
constexpr size_t kAlign = 256;
constexpr size_t kLdsBudget = 160 * 1024;   // LDS per workgroup on gfx950
constexpr int kWindowMaxWaves = 16;      // wavefronts per workgroup (compute + loader)
constexpr int kWindowTickSlices = 8;     // slices (compute wavefronts) per tick
constexpr int kStreamSlackChunks = 256;  // 16-byte chunks behind the packet stream that a fixed-count entry fetch may touch
constexpr int kStreamTailTicks = 16;     // empty ticks behind the last one in the slice table (the streaming loop runs on
                                         // to a multiple of 8 ticks and fetches four ticks ahead)
constexpr uint64_t kWindowTickBytes = 15 * 1024;   // packet bytes per tick, unless one slice alone is larger
constexpr int kWindowFarTicks = 12;      // a neighbour this many ticks back (or more) is read from the output array
constexpr int kWindowFarLead = 4;        // ticks a far wavefront runs ahead (twice: read list, then gather)
constexpr int kWindowMaxFarWaves = 4;    // 64 far reads per tick each
constexpr int kWindowMaxGroups = 8;     // partitions one workgroup may hold
constexpr int kMaskWords = 72;           // 32-bit mask words one tick's id range may touch (fused mask)

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// One sweep direction of the wave-column plan: a CSR over original vertex ids.
struct ColumnDir {
    size_t ptr_off = 0;     // int32 [n+1]
    size_t idx_off = 0;     // int32 [m]     neighbour vertex (head for the b sweep, tail for the t sweep)
    size_t wt_off = 0;      // uint32 or int64 [m]  t(e) in this CSR's order
    size_t order_off = 0;   // int32 [n]     vertices in sweep order, long rows first inside a level
    size_t rows_off = 0;    // int32 [n][4]  {vertex, first edge, end of its edges, 0} in sweep order: what a
                            //               wavefront of the wave-column plan needs to start, in one load
    size_t lvl_off = 0;     // int32 [L][4]  {first position, hub rows, rows, 0} per level in sweep order
    // per level, in sweep order
    std::vector<int32_t> lvl_begin, lvl_hubs, lvl_count;
};

// One sweep direction of the resident-window plan.  Vertices are renumbered by
// position in sweep order.  A level is cut into ticks (runs of at most
// kWindowTickSlices slices and about kWindowTickBytes of packet), and everything
// a tick needs is one contiguous "packet" of 16-byte chunks, so that loader
// wavefronts can stream it into LDS ahead of the compute wavefronts.  A slice is
// 64 rows (vertices), one per compute wavefront; a slice of at most 32 rows gives
// each row 2..64 lanes that share its edges and fold their maxima at the end.
//   descriptors  smax x {byte offset of the slice's entries in the packet,
//                        width | rows << 16 | log2(lanes per row) << 24,
//                        lowest vertex id of the tick, ring slot of row 0}
//                (rows = 0 for slices this tick does not have)
//   records      per slice 64 x {original vertex id, c}; rows past `rows` are padding
//                and carry the tick's lowest vertex id
//   entries      per slice width x 64 x {ring field of the neighbour, t(e)}: entry j
//                of lane l of a slice sits at base + j*64 + l.  The ring field is the
//                neighbour's slot (times 8 when the ring holds {value, device}
//                pairs: a byte offset); padding entries point at slot `slots`,
//                which holds the constant 0, with t = 0.  When the ring cannot hold
//                every neighbour (far_cap > 0), a neighbour computed far_ticks or more
//                ticks earlier is a far read: its entry points at a pair behind the ring
//                (byte offset ring bytes + (tick & 1) * 8 * far_cap + 8 * index) that a far
//                wavefront fills from the output array before the tick starts.  An entry is two uint32, or
//                one uint32 (field | t << 16) when both fit 16 bits (ent4).
struct WindowDir {
    size_t stream_off = 0;   // uint4 [total_chunks]
    size_t tick_off = 0;     // uint32 [ticks+1][4] {first chunk, chunks, lowest id, id span}
    size_t gmap_off = 0;     // int32 [ticks*wpad] original id per padded position, -1 = padding
    size_t far_off = 0;      // uint32 [ticks][far_cap][2] {vertex, c} of the tick's far reads (padding: vertex 0)
    size_t stab_off = 0;     // uint32 [ticks][smax][8] per slice {record chunk, entry chunk, width | rows << 16 | log2 lanes
                             // per row << 24, lowest id of the tick, ring slot of row 0, 0, 0, 0}: where a compute wavefront
                             // that streams its own slices finds them (chunks of 16 bytes from the start of the stream;
                             // slices a tick does not have point at its packet with rows = 0).  0 = not built (only
                             // for 4-byte entries, a packed ring and no far reads)
    int32_t max_width = 0;   // entries per lane of the widest slice
    int32_t far_cap = 0;     // far reads per tick, a multiple of 64; 0 = every neighbour is in the ring
    int64_t total_chunks = 0;
    int32_t ticks = 0;
    int32_t max_chunks = 0;  // largest packet
    int32_t wpad = 0;        // tick width rounded up to whole slices of 64
    int32_t smax = 0;        // slices of the widest tick
    int32_t slots = 0;       // ring capacity R: slot of position i is i mod R
    int32_t idpad = 0;       // bytes a stage slot reserves for device ids
    bool direct_ok = false;  // every tick's vertices lie in a short id range
    bool packed = false;     // ring of {value, device} pairs (32-bit ticks only)
    bool ent4 = false;       // 4-byte entries
};

struct Packed {
    int32_t n = 0, L = 0;
    int64_t m = 0;
    bool narrow = false;        // every c and t < 2^32: weights stored as uint32
    cp_graph_info info{};
    ColumnDir col_b, col_t;
    size_t c_off = 0;           // uint32 or int64 [n], original ids
    size_t sources_off = 0;     // int32 [num_sources]
    bool have_window = false;
    WindowDir win_b, win_t;
    int32_t max_width = 0;
    std::vector<uint8_t> blob;  // host image of the device blob
};

// Validate and pack.  Returns CP_OK or an error code.
int pack_graph(int32_t n, int64_t m, int32_t L,
               const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *succ_t,
               const int32_t *pred_ptr, const int32_t *pred_idx, const int32_t *pred_eid,
               const int64_t *c, const int32_t *level_ptr, const int32_t *level_vtx,
               Packed &out);

// ---- cost tables -----------------------------------------------------------

// Multiply-shift form of ceil(a/d) for a 32-bit dividend:
//   ceil(a/d) = ((a + dm1) * mul + (a + dm1)) >> 32     with dm1 = d-1, mul = ceil(2^32/d) - 1.
// A free transfer (same device) is the pair {0, 0}, which yields 0 for every a < 2^32.
struct alignas(8) Magic { uint32_t mul, dm1; };

struct CostTables {
    int32_t k = 0;
    bool magic_ok = false;              // every divisor admits the exact 32-bit form for this graph's weights
    std::vector<Magic> magic;           // [k*k edge (row = own device, col = neighbour), b sweep]
                                        // [k*k the same transposed, t sweep] [k vertex]
    std::vector<int64_t> divisor;       // same layout, plain divisors; 0 = free transfer
    // The compact form: every divisor <= 256 and exact as (d - 1) | (upper 24 bits of the multiplier) << 8
    // for this graph's weights, which must be below 2^24.  A 4-byte entry can sit in LDS once per
    // bank, which takes the bank conflicts out of the kernels' table reads.
    bool tab4_ok = false;
    std::vector<uint32_t> tab4;         // same layout; 0 = free transfer
};

// Returns CP_OK, CP_ERR_SPEED or CP_ERR_BANDWIDTH.
int build_cost_tables(int32_t k, const int64_t *speeds, const int64_t *bandwidth,
                      bool narrow, int64_t max_c, int64_t max_t, CostTables &out);

inline size_t table_entries(int32_t k) { return (size_t)2 * k * k + k; }
// 64-bit words of one call's tables in device memory: the 8-byte entries, then the 4-byte ones
inline size_t table_words(int32_t k) { return table_entries(k) + (table_entries(k) + 1) / 2; }

}  // namespace cpeval

struct cp_graph {
    cpeval::Packed packed;
    void *device_blob = nullptr;
};
