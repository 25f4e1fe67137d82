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
    int32_t P = 0, k = 0, L = 0, max_width = 0;
    const uint8_t *pT = nullptr;        // [n][P] device ids (wave-column)
    const uint8_t *assign = nullptr;    // caller's assignments (resident-window)
    int64_t a_stride_p = 0, a_stride_v = 0;
    void *val = nullptr;                // [n][P] ticks
    int64_t *cp_out = nullptr;          // resident-window b sweep only
    const void *edge_tab = nullptr;
    const void *vert_tab = nullptr;
    int32_t *status = nullptr;
};

size_t window_lds_bytes(int32_t k, int32_t slots, size_t tick_bytes);

int launch_clear(int64_t *cp_out, int32_t batch, int32_t *status, void *stream);
int launch_transpose(const uint8_t *in, uint8_t *out, int32_t n, int32_t P, void *stream);
int launch_column_sweep(const SweepLaunch &s, void *stream, int32_t *launches);
int launch_window_sweep(const SweepLaunch &s, void *stream, int32_t *launches);
int launch_cp_sources(const int32_t *sources, int32_t nsrc, const void *b, int32_t P,
                      int tick_bytes, int64_t *cp_out, void *stream);
int launch_mask(const void *b, const void *tl, const int64_t *cp, int32_t n, int32_t P,
                int tick_bytes, uint64_t *mask, void *stream);

}  // namespace cpeval
