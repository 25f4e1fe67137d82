// Host-callable launchers implemented in kernels.hip.
#pragma once

#include <algorithm>

#include "cpeval_internal.hpp"

namespace cpeval {

struct SweepLaunch {
    const uint8_t *blob = nullptr;      // device blob base
    const ColumnDir *dir = nullptr;     // wave-column plan
    const WindowDir *win = nullptr;     // resident-window plan
    size_t c_off = 0;
    bool tsweep = false;
    bool magic = false;                 // multiply-shift tables (else plain divisors)
    bool narrow = false;                // 32-bit weights in the blob
    int tick_bytes = 4;
    int32_t n = 0, P = 0, k = 0, L = 0, max_width = 0;
    const uint8_t *pT = nullptr;        // [n][P] device ids (wave-column)
    const uint8_t *assign = nullptr;    // caller's assignments (resident-window: input of the gather)
    const uint8_t *pperm = nullptr;     // [P][ticks*wpad] device ids in sweep order (resident-window)
    bool direct_ids = false;            // resident-window: stage ids straight from `assign`
    int64_t a_stride_p = 0, a_stride_v = 0;
    void *val = nullptr;                // ticks of (v, q) at v * out_sv + q * out_sq (resident-window sweep,
                                        // critical-path walk); the wave-column sweep writes [n][P]
    int64_t out_sv = 0, out_sq = 1;
    int64_t *cp_out = nullptr;          // resident-window b sweep only
    const void *edge_tab = nullptr;
    const void *vert_tab = nullptr;
    const uint32_t *edge_tab4 = nullptr;   // the same tables as 4-byte entries, or null
    const uint32_t *vert_tab4 = nullptr;
    int32_t *status = nullptr;
    // resident-window t sweep that also writes the mask rows (partition-major): b, CP and the
    // zeroed mask; all null otherwise
    const void *mask_b = nullptr;
    const int64_t *mask_cp = nullptr;
    uint64_t *mask_out = nullptr;
};

// Launch shape of the resident-window kernel for one sweep direction.
struct WindowCfg {
    int nl = 0;        // 16-byte loads per loader lane per level
    int nlw = 0;       // loader wavefronts
    int nc = 0;        // compute wavefronts
    int nfw = 0;       // far wavefronts
    int dr = 0;        // levels a loader runs ahead in registers
    bool packed = false;   // ring holds {value, device} pairs (one LDS read per relaxation)
    int groups = 1;        // partitions per workgroup (they share the cost tables)
    size_t sub_bytes = 0;  // LDS of one partition: ring, far pairs, two stage slots
    size_t lds_bytes = 0;  // of the workgroup: groups * sub_bytes + tables
};

// Launch shape of the shared-window kernel (several partitions per workgroup behind one
// loader set and one pair of stage slots) for one sweep direction.
struct SharedCfg {
    int groups = 0;    // partitions per workgroup: 2 or 4
    int nl = 0;        // 16-byte loads per loader lane per tick
    int nlw = 0;       // loader wavefronts
    int nc = 0;        // compute wavefronts
    int nfw = 0;       // far wavefronts
    size_t vals_off = 0, stage_off = 0, tab_off = 0;   // LDS byte offsets: ring values, stage slots, cost tables
    size_t lds_bytes = 0;
    int tab_rs = -1;   // >= 0: 4-byte cost-table entries, each 2^tab_rs times in LDS
};
// False if the direction cannot run that way under `lds_limit` bytes of dynamic LDS.
// tab4: the call's cost tables exist as 4-byte entries.
bool shared_config(const WindowDir &d, int32_t k, int groups, size_t lds_limit, SharedCfg &out, bool tab4 = false);
// Bytes of the cost tables in LDS as 4-byte entries, every transfer entry 2^rs times.
inline size_t tab4_lds_bytes(int32_t k, int rs) {
    return ((((size_t)k * k * 4) << rs) + (size_t)k * 4 + 15) & ~(size_t)15;
}
int launch_window_shared(const SweepLaunch &s, const SharedCfg &cfg, void *stream);

// Launch shape of the streamed resident-window kernel (compute wavefronts fetch their own
// slices; only the per-partition bytes are staged) for one sweep direction.
struct StreamCfg {
    bool wide = false; // some slice has more than 8 entries per lane: 16 entry registers instead of 8
    int nl = 0;        // 16-byte loads per loader lane per tick
    int nlw = 0;       // loader wavefronts
    int nc = 0;        // compute wavefronts = slices of the widest tick
    size_t stage_off = 0, tab_off = 0;   // LDS byte offsets of the stage slots and the cost tables
    size_t lds_bytes = 0;
};
// False if the direction cannot run that way under `lds_limit` bytes of dynamic LDS.
// with_mask: the t sweep also stages the tick's b values and writes the mask.
bool stream_config(const WindowDir &d, int32_t k, size_t lds_limit, bool with_mask, StreamCfg &out);
int launch_window_stream(const SweepLaunch &s, const StreamCfg &cfg, void *stream);

// False if the direction cannot run under `lds_limit` bytes of LDS.
// with_mask: the t sweep also stages the tick's b values and writes the mask.
bool window_config(const WindowDir &d, int32_t k, size_t tick_bytes, size_t lds_limit, WindowCfg &out,
                   bool with_mask = false);
// The two sweeps side by side in one launch (window_pair_kernel): shapes for both, or false
// where that form does not apply.
bool window_pair_config(const WindowDir &db, const WindowDir &dt, int32_t k, size_t lds_limit, WindowCfg &out_b,
                        WindowCfg &out_t);
int launch_window_pair(const SweepLaunch &sb, const SweepLaunch &st, const WindowCfg &cfg_b, const WindowCfg &cfg_t,
                       void *stream);
int32_t window_mask_bpad(const WindowDir &d);
int launch_gather_assign(const SweepLaunch &s, uint8_t *out, void *stream);

int launch_clear(int64_t *cp_out, int32_t batch, int32_t *status, void *stream);
int launch_transpose(const uint8_t *in, uint8_t *out, int32_t n, int32_t P, void *stream);
int launch_column_sweep(const SweepLaunch &s, void *stream, int32_t *launches);
int launch_window_sweep(const SweepLaunch &s, const WindowCfg &cfg, void *stream, int32_t *launches);
int launch_column_slice(const SweepLaunch &s, void *stream);   // CP_ERR_ARG without 32-bit multiply-shift tables
int launch_cp_sources(const int32_t *sources, int32_t nsrc, const void *b, int32_t P,
                      int tick_bytes, int64_t *cp_out, void *stream);
// One segmented radix sort per call: the PCT priority lists of section 4.1.
struct PctOrderLaunch {
    int32_t n = 0, P = 0, k = 0;
    const void *b = nullptr;          // ticks [n][P], or [P][n] with b_by_partition
    bool b_by_partition = false;
    int tick_bytes = 4;
    const uint8_t *assign = nullptr;
    int64_t a_stride_p = 0, a_stride_v = 0;
    int64_t max_b = 0;                // every b lies in [0, max_b]
    int b_bits = 1, key_bits = 1, key_bytes = 4;
    void *keys_a = nullptr, *keys_b = nullptr;   // key [P][n] each
    int32_t *vals_tmp = nullptr;      // [P][n]
    uint32_t *counts = nullptr;       // pct_counts_bytes
    int32_t *order_out = nullptr, *seg_out = nullptr, *status = nullptr;
};
size_t pct_counts_bytes(int32_t n, int32_t P);
int32_t pct_sort_tiles(int32_t n);
int launch_pct_order(const PctOrderLaunch &s, void *stream);

// List-scheduling simulation (sections 4, 4.1, 5.1), one wavefront per partition.
struct SimulateLaunch {
    const uint8_t *blob = nullptr;
    const ColumnDir *succ = nullptr;    // successor CSR
    const ColumnDir *pred = nullptr;    // predecessor CSR (row bounds only)
    size_t c_off = 0;
    bool magic = false, narrow = false, pct = false;
    int32_t n = 0, P = 0, k = 0;
    uint32_t window = 0;                // shortest execution time + shortest transfer time - 1
    int32_t groups = 1;                 // partitions per wavefront (at most 64 / k)
    const uint8_t *assign = nullptr;
    int64_t a_stride_p = 0, a_stride_v = 0;
    const void *b = nullptr;
    int64_t b_sv = 0, b_sq = 0;
    int b_bytes = 4;
    const int32_t *tie = nullptr;
    int32_t *tie_inv = nullptr;         // [n] scratch when tie is given
    const void *edge_tab = nullptr, *vert_tab = nullptr;
    int32_t *ready = nullptr, *need = nullptr, *inbox = nullptr;   // [P][n] each
    uint64_t *pending = nullptr, *available = nullptr;             // [P][n] each (available: PCT only)
    int64_t *makespan = nullptr;
    int32_t *start = nullptr;
    int32_t *status = nullptr;
};
int launch_simulate(const SimulateLaunch &s, void *stream);

int launch_validate(const uint8_t *assign, int64_t a_stride_p, int64_t a_stride_v, int32_t n, int32_t P, int32_t k,
                    int64_t num_pairs, const int32_t *pairs, int64_t num_pins, const int32_t *pins,
                    uint8_t *valid, int32_t *violations, int32_t *status, void *stream);
int launch_zero_bytes(uint8_t *dst, int64_t bytes, void *stream);
int launch_zero_words(uint64_t *dst, int64_t words, void *stream);
int launch_ranks(const void *b, const void *tl, const void *c, bool narrow, int tick_bytes, int32_t n,
                 int64_t *up, int64_t *down, int64_t *total, void *stream);
int launch_critical_path(const SweepLaunch &s, const int32_t *sources, int32_t nsrc, const int64_t *cp,
                         int32_t max_len, int32_t *path, int32_t *len, void *stream);
int launch_mask(const void *b, const void *tl, const int64_t *cp, int32_t n, int32_t P,
                int tick_bytes, bool by_partition, uint64_t *mask, void *stream);
int launch_transpose_ticks(const void *in, void *out, int32_t rows, int32_t cols, int tick_bytes, void *stream);

}  // namespace cpeval
