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
constexpr int kWindowMaxThreads = 1024;

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// One sweep direction of the wave-column plan: a CSR over original vertex ids.
struct ColumnDir {
    size_t ptr_off = 0;     // int32 [n+1]
    size_t idx_off = 0;     // int32 [m]     neighbour vertex (head for the b sweep, tail for the t sweep)
    size_t wt_off = 0;      // uint32 or int64 [m]  t(e) in this CSR's order
    size_t order_off = 0;   // int32 [n]     vertices in sweep order, long rows first inside a level
    // per level, in sweep order
    std::vector<int32_t> lvl_begin, lvl_hubs, lvl_count;
};

// One sweep direction of the resident-window plan.  Vertices are renumbered by
// position in sweep order; rows are packed in slices of 64 positions (one per
// wavefront), entry j of lane l of a slice at slice_off + j*64 + l.
struct WindowDir {
    size_t vtx_off = 0;     // int32 [n]        original id at each position
    size_t c_off = 0;       // uint32 [n]       c at each position
    size_t deg_off = 0;     // int32 [n]        row length at each position
    size_t lvl_off = 0;     // int32 [L+1][2]   per level in sweep order: {first position, first slice}
    size_t slice_off = 0;   // uint32 [slices+1] entry offset of each slice
    size_t ent_off = 0;     // uint2 [entries]  {LDS slot of the neighbour, t(e)}
    int64_t entries = 0;
    int32_t slices = 0;
    int32_t slots = 0;      // ring capacity R: slot of position i is i mod R
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
struct Magic { uint32_t mul, dm1; };

struct CostTables {
    int32_t k = 0;
    bool magic_ok = false;              // every divisor admits the exact 32-bit form for this graph's weights
    std::vector<Magic> magic;           // [k*k edge (row = own device, col = neighbour), b sweep]
                                        // [k*k the same transposed, t sweep] [k vertex]
    std::vector<int64_t> divisor;       // same layout, plain divisors; 0 = free transfer
};

// Returns CP_OK, CP_ERR_SPEED or CP_ERR_BANDWIDTH.
int build_cost_tables(int32_t k, const int64_t *speeds, const int64_t *bandwidth,
                      bool narrow, int64_t max_c, int64_t max_t, CostTables &out);

inline size_t table_entries(int32_t k) { return (size_t)2 * k * k + k; }

}  // namespace cpeval

struct cp_graph {
    cpeval::Packed packed;
    void *device_blob = nullptr;
};
