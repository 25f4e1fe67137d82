// Host side of cp_graph_create: validation of the caller's arrays and packing
// into the device image used by the two kernel families.  No GPU call here.
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>

#include "cpeval_internal.hpp"

namespace cpeval {
namespace {

struct BlobWriter {
    std::vector<uint8_t> &buf;
    explicit BlobWriter(std::vector<uint8_t> &b) : buf(b) {}
    size_t reserve(size_t bytes) {
        size_t off = align_up(buf.size());
        buf.resize(off + bytes, 0);
        return off;
    }
    template <typename T> T *at(size_t off) { return reinterpret_cast<T *>(buf.data() + off); }
};

struct Csr {
    const int32_t *ptr;
    const int32_t *idx;
    std::vector<int64_t> wt;  // t(e) in this CSR's order
};

int check_csr(int32_t n, int64_t m, const int32_t *ptr, const int32_t *idx) {
    if (ptr[0] != 0 || (int64_t)ptr[n] != m) return CP_ERR_CSR;
    for (int32_t v = 0; v < n; ++v)
        if (ptr[v + 1] < ptr[v]) return CP_ERR_CSR;
    for (int64_t e = 0; e < m; ++e)
        if (idx[e] < 0 || idx[e] >= n) return CP_ERR_CSR;
    return CP_OK;
}

// Vertices in sweep order: levels first-to-last (forward) or last-to-first, and
// inside a level the longest rows first, so that hubs lead and rows of similar
// length share a wavefront.
void sweep_order(int32_t n, int32_t L, const int32_t *level_ptr, const int32_t *level_vtx,
                 const int32_t *ptr, bool forward, std::vector<int32_t> &order, ColumnDir &dir) {
    order.resize(n);
    dir.lvl_begin.assign(L, 0);
    dir.lvl_hubs.assign(L, 0);
    dir.lvl_count.assign(L, 0);
    int32_t pos = 0;
    for (int32_t s = 0; s < L; ++s) {
        int32_t l = forward ? s : L - 1 - s;
        int32_t a = level_ptr[l], b = level_ptr[l + 1];
        std::copy(level_vtx + a, level_vtx + b, order.begin() + pos);
        std::stable_sort(order.begin() + pos, order.begin() + pos + (b - a),
                         [&](int32_t x, int32_t y) {
                             return ptr[x + 1] - ptr[x] > ptr[y + 1] - ptr[y];
                         });
        int32_t hubs = 0;
        while (hubs < b - a) {
            int32_t v = order[pos + hubs];
            if (ptr[v + 1] - ptr[v] < kHubDegree) break;
            ++hubs;
        }
        dir.lvl_begin[s] = pos;
        dir.lvl_hubs[s] = hubs;
        dir.lvl_count[s] = b - a;
        pos += b - a;
    }
}

void pack_column_dir(BlobWriter &w, int32_t n, int64_t m, bool narrow, const Csr &csr,
                     const std::vector<int32_t> &order, ColumnDir &dir) {
    dir.ptr_off = w.reserve(sizeof(int32_t) * ((size_t)n + 1));
    std::memcpy(w.at<int32_t>(dir.ptr_off), csr.ptr, sizeof(int32_t) * ((size_t)n + 1));
    dir.idx_off = w.reserve(sizeof(int32_t) * (size_t)std::max<int64_t>(m, 1));
    if (m) std::memcpy(w.at<int32_t>(dir.idx_off), csr.idx, sizeof(int32_t) * (size_t)m);
    if (narrow) {
        dir.wt_off = w.reserve(sizeof(uint32_t) * (size_t)std::max<int64_t>(m, 1));
        uint32_t *p = w.at<uint32_t>(dir.wt_off);
        for (int64_t e = 0; e < m; ++e) p[e] = (uint32_t)csr.wt[e];
    } else {
        dir.wt_off = w.reserve(sizeof(int64_t) * (size_t)std::max<int64_t>(m, 1));
        if (m) std::memcpy(w.at<int64_t>(dir.wt_off), csr.wt.data(), sizeof(int64_t) * (size_t)m);
    }
    dir.order_off = w.reserve(sizeof(int32_t) * (size_t)n);
    std::memcpy(w.at<int32_t>(dir.order_off), order.data(), sizeof(int32_t) * (size_t)n);
    dir.rows_off = w.reserve(sizeof(int32_t) * 4 * (size_t)n);
    int32_t *rows = w.at<int32_t>(dir.rows_off);
    for (int32_t i = 0; i < n; ++i) {
        const int32_t v = order[i];
        rows[4 * (size_t)i] = v;
        rows[4 * (size_t)i + 1] = csr.ptr[v];
        rows[4 * (size_t)i + 2] = csr.ptr[v + 1];
        rows[4 * (size_t)i + 3] = 0;
    }
    const size_t L = dir.lvl_begin.size();
    dir.lvl_off = w.reserve(sizeof(int32_t) * 4 * std::max<size_t>(L, 1));
    int32_t *lvl = w.at<int32_t>(dir.lvl_off);
    for (size_t l = 0; l < L; ++l) {
        lvl[4 * l] = dir.lvl_begin[l];
        lvl[4 * l + 1] = dir.lvl_hubs[l];
        lvl[4 * l + 2] = dir.lvl_count[l];
        lvl[4 * l + 3] = 0;
    }
}

// A slice with few rows spreads each row over several lanes: log2 of the lanes
// per row for a slice of `rows` vertices.
int lanes_per_row_log2(int rows) {
    int sh = 0;
    while ((rows << (sh + 1)) <= kWave) ++sh;
    return sh;
}

// Resident-window packing for one direction (layout: see WindowDir).  Returns
// false if the graph does not suit that plan.
bool pack_window_dir(BlobWriter &w, int32_t n, int32_t L, const int64_t *c, int64_t max_t,
                     bool ticks32, const Csr &csr, const std::vector<int32_t> &level_order,
                     const ColumnDir &col, WindowDir &dir) {
    // A slice is 64 consecutive positions of a level in the order the wave-column plan uses
    // (long rows first).  Inside a slice the order is free: by vertex number, so that the
    // lanes of an output store (and of the mask's reads of b) walk memory in one direction
    // and neighbouring lanes share cache lines.
    std::vector<int32_t> order(level_order);
    std::vector<int32_t> slice_deg((size_t)n, 0);       // longest row of the slice that starts at this position
    for (size_t s = 0; s < col.lvl_begin.size(); ++s) {
        const int32_t a = col.lvl_begin[s], b = a + col.lvl_count[s];
        for (int32_t p0 = a; p0 < b; p0 += kWave) {
            const int32_t e = std::min(b, p0 + kWave);
            int32_t deg = 0;
            for (int32_t i = p0; i < e; ++i) deg = std::max(deg, csr.ptr[order[i] + 1] - csr.ptr[order[i]]);
            slice_deg[p0] = deg;
            std::sort(order.begin() + p0, order.begin() + e);
        }
    }
    std::vector<int32_t> pos(n);
    for (int32_t i = 0; i < n; ++i) pos[order[i]] = i;

    auto slice_entries = [&](int32_t p0, int32_t rows) -> uint64_t {
        int64_t deg0 = slice_deg[p0];
        int sh = lanes_per_row_log2(rows);
        return (uint64_t)((deg0 + (1 << sh) - 1) >> sh) * kWave;
    };
    // Far edges: a neighbour computed kWindowFarTicks or more ticks earlier is not kept in
    // the ring; its value is read back from the output array by a far wavefront (32-bit
    // ticks only: the far values are staged as {value, device} pairs like the ring's).
    // Before the ticks are known the level distance stands in for the tick distance (a
    // level is at least one tick), which can only overestimate the ring.
    std::vector<int32_t> lvl_of((size_t)n);
    for (int32_t s = 0; s < L; ++s)
        for (int32_t i = col.lvl_begin[s]; i < col.lvl_begin[s] + col.lvl_count[s]; ++i) lvl_of[i] = s;
    // An upper bound of the ring capacity (exact value below, once the ticks are known)
    // fixes the entry format: the ring holds {value, device} pairs if that leaves room
    // for two stage slots and small cost tables, else separate arrays.
    auto ring_bound = [&](bool skip_far) {
        int64_t bound = 1;
        for (int32_t i = 0; i < n; ++i) {
            int32_t v = order[i];
            int32_t end = col.lvl_begin[lvl_of[i]] + col.lvl_count[lvl_of[i]];
            for (int32_t e = csr.ptr[v]; e < csr.ptr[v + 1]; ++e) {
                int32_t pn = pos[csr.idx[e]];
                if (skip_far && lvl_of[i] - lvl_of[pn] >= kWindowFarTicks) continue;
                bound = std::max<int64_t>(bound, (int64_t)end - pn);
            }
        }
        return bound;
    };
    auto pairs_fit = [&](int64_t slots, uint64_t far_bytes) {
        return 8 * ((uint64_t)slots + 1) + far_bytes + 2 * (kWindowTickBytes + 1024) + 4096 <= kLdsBudget - 512;
    };
    // far reads only where a ring of pairs for every neighbour does not fit
    int64_t need_ub = ring_bound(false);
    const bool far_allowed = ticks32 && !pairs_fit(need_ub, 0);
    if (far_allowed) need_ub = ring_bound(true);
    const uint64_t far_bytes_ub = far_allowed ? 2 * 8 * (uint64_t)kWave * kWindowMaxFarWaves : 0;
    dir.packed = ticks32 && pairs_fit(need_ub, far_bytes_ub);
    const uint64_t field_max = dir.packed ? 8 * (uint64_t)need_ub + 32 + far_bytes_ub : (uint64_t)need_ub;
    dir.ent4 = field_max < 65536 && max_t < 65536;
    const uint64_t esz = dir.ent4 ? 4 : 8;

    // Ticks: a level is cut into runs of at most kWindowTickSlices slices and about
    // kWindowTickBytes of packet, so that one typical packet size fits every tick
    // (vertices of one level do not depend on each other, so any cut is valid).
    std::vector<int32_t> tick_a, tick_b;
    for (int32_t s = 0; s < L; ++s) {
        int32_t a = col.lvl_begin[s], b = a + col.lvl_count[s];
        if (a == b) continue;
        int32_t start = a, nsl = 0;
        uint64_t bytes = 0;
        for (int32_t p0 = a; p0 < b; p0 += kWave) {
            int32_t rows = std::min(kWave, b - p0);
            uint64_t add = 8 * (uint64_t)kWave + esz * slice_entries(p0, rows);
            if (nsl > 0 && (nsl == kWindowTickSlices || bytes + add > kWindowTickBytes)) {
                tick_a.push_back(start);
                tick_b.push_back(p0);
                start = p0;
                nsl = 0;
                bytes = 0;
            }
            ++nsl;
            bytes += add;
        }
        tick_a.push_back(start);
        tick_b.push_back(b);
    }
    const int32_t T = (int32_t)tick_a.size();
    dir.ticks = T;

    std::vector<int32_t> tick_of((size_t)n);
    for (int32_t s = 0; s < T; ++s)
        for (int32_t i = tick_a[s]; i < tick_b[s]; ++i) tick_of[i] = s;
    // A neighbour far_ticks or more ticks back is a far read.  The smallest distance is the
    // one the far wavefronts' timing needs; it is doubled until the far reads of every tick
    // fit the far wavefronts (a longer ring for fewer far reads).
    const bool far_on = far_allowed && dir.packed;
    int32_t far_ticks = kWindowFarTicks;
    auto is_far = [&](int32_t s, int32_t pn) { return far_on && s - tick_of[pn] >= far_ticks; };
    int64_t need = 1, far_max = 0;
    for (;;) {
        need = 1;
        far_max = 0;
        for (int32_t s = 0; s < T; ++s) {
            int32_t a = tick_a[s], b = tick_b[s];
            int64_t far_here = 0;
            // a tick's vertices take consecutive slots with at most one wrap, whether or not
            // anything reads them: the ring is at least as long as the widest tick
            need = std::max<int64_t>(need, (int64_t)b - a);
            for (int32_t i = a; i < b; ++i) {
                int32_t v = order[i];
                for (int32_t e = csr.ptr[v]; e < csr.ptr[v + 1]; ++e) {
                    int32_t pn = pos[csr.idx[e]];
                    if (is_far(s, pn)) ++far_here;
                    else need = std::max<int64_t>(need, (int64_t)b - pn);
                }
            }
            far_max = std::max(far_max, far_here);
        }
        if (!far_on || far_max <= (int64_t)kWave * kWindowMaxFarWaves || far_ticks > T) break;
        far_ticks *= 2;
    }
    if (far_on && !pairs_fit(need, 2 * 8 * (uint64_t)((far_max + kWave - 1) / kWave * kWave))) return false;
    if (dir.ent4 && dir.packed && 8 * ((uint64_t)need + 1) + 32 + far_bytes_ub >= 65536) return false;

    int32_t wmax = 1;
    int64_t idspan = 1;
    std::vector<uint32_t> tick_tab(4 * ((size_t)T + 1), 0);   // {first chunk, chunks, lowest id, id span}
    uint64_t total = 0;
    uint32_t max_chunks = 1;
    for (int32_t s = 0; s < T; ++s) {
        int32_t a = tick_a[s], b = tick_b[s];
        wmax = std::max(wmax, b - a);
        int32_t lo = order[a], hi = order[a];
        for (int32_t i = a; i < b; ++i) { lo = std::min(lo, order[i]); hi = std::max(hi, order[i]); }
        idspan = std::max<int64_t>(idspan, (int64_t)hi - lo + 1);
        tick_tab[4 * s + 2] = (uint32_t)lo;
        tick_tab[4 * s + 3] = (uint32_t)(hi - lo + 1);
    }
    dir.slots = (int32_t)need;
    dir.far_cap = (int32_t)((far_max + kWave - 1) / kWave * kWave);
    if (dir.far_cap > kWave * kWindowMaxFarWaves) return false;    // too many far reads per tick
    dir.smax = (wmax + kWave - 1) / kWave;
    dir.wpad = dir.smax * kWave;
    if (dir.smax > kWindowMaxWaves - 1) return false;   // only when one slice alone exceeds every limit
    // the device ids of a tick can be staged straight from the caller's row when its
    // vertices occupy a short id range
    dir.direct_ok = idspan + 15 <= 4 * (int64_t)dir.wpad;
    dir.idpad = dir.direct_ok ? std::max<int32_t>(dir.wpad, (int32_t)((idspan + 15 + 15) / 16 * 16)) : dir.wpad;

    for (int32_t s = 0; s < T; ++s) {
        int32_t a = tick_a[s], b = tick_b[s];
        uint64_t nsl = (uint64_t)(b - a + kWave - 1) / kWave, entries = 0;
        for (int32_t p0 = a; p0 < b; p0 += kWave) entries += slice_entries(p0, std::min(kWave, b - p0));
        uint64_t bytes = 16 * (uint64_t)dir.smax + 8 * kWave * nsl + esz * entries;
        uint64_t chunks = (bytes + 15) / 16;
        if (chunks > (1u << 16)) return false;      // a 1 MB tick never fits LDS
        tick_tab[4 * s] = (uint32_t)total;
        tick_tab[4 * s + 1] = (uint32_t)chunks;
        total += chunks;
        if (total >= (1ull << 31)) return false;
        max_chunks = std::max<uint32_t>(max_chunks, (uint32_t)chunks);
    }
    tick_tab[4 * (size_t)T] = (uint32_t)total;
    dir.total_chunks = (int64_t)total;
    dir.max_chunks = (int32_t)max_chunks;

    // the stream is followed by slack: a wavefront that streams its own slices always fetches a
    // fixed number of entry rows, whatever the slice's width
    dir.stream_off = w.reserve(16 * ((size_t)std::max<uint64_t>(total, 1) + kStreamSlackChunks));
    const bool with_stab = dir.ent4 && dir.packed && dir.far_cap == 0;
    // ... and runs kStreamTailTicks ticks past the end with empty slices
    dir.stab_off = with_stab ? w.reserve(32 * ((size_t)T + kStreamTailTicks) * (size_t)dir.smax) : 0;
    dir.tick_off = w.reserve(sizeof(uint32_t) * tick_tab.size());
    std::memcpy(w.at<uint32_t>(dir.tick_off), tick_tab.data(), sizeof(uint32_t) * tick_tab.size());
    dir.gmap_off = w.reserve(sizeof(int32_t) * (size_t)std::max(T, 1) * dir.wpad);
    dir.far_off = w.reserve(8 * (size_t)std::max(dir.far_cap, 1) * (size_t)std::max(T, 1));
    // every reservation is made: the blob does not move any more
    int32_t *gmap = w.at<int32_t>(dir.gmap_off);
    uint32_t *far_list = w.at<uint32_t>(dir.far_off);
    uint32_t *stab = with_stab ? w.at<uint32_t>(dir.stab_off) : nullptr;
    dir.max_width = 0;
    std::fill(gmap, gmap + (size_t)std::max(T, 1) * dir.wpad, -1);

    // far reads of a tick: {vertex, c} per read, padded with vertex 0; the pairs they are
    // turned into sit behind the ring, one region per tick parity
    const uint32_t ring_bytes = (uint32_t)((8 * ((uint64_t)dir.slots + 1) + 15) & ~(uint64_t)15);
    if (dir.far_cap > 0 && dir.ent4 && ring_bytes + 2 * 8 * (uint64_t)dir.far_cap >= 65536) return false;

    const uint32_t pad_field = (uint32_t)(dir.packed ? 8 * (uint64_t)dir.slots : (uint64_t)dir.slots);
    for (int32_t s = 0; s < T; ++s) {
        int32_t a = tick_a[s], b = tick_b[s];
        uint32_t nsl = (uint32_t)(b - a + kWave - 1) / kWave;
        uint32_t far_next = 0;
        const uint32_t far_base = ring_bytes + (uint32_t)(s & 1) * 8u * (uint32_t)dir.far_cap;
        uint8_t *pk = w.at<uint8_t>(dir.stream_off + 16 * (size_t)tick_tab[4 * s]);
        uint32_t *desc = (uint32_t *)pk;
        uint32_t *rec = (uint32_t *)(pk + 16 * (size_t)dir.smax);         // nsl*64 x {v, c}
        const uint32_t ent_start = 16 * (uint32_t)dir.smax + 8 * kWave * nsl;
        uint32_t *ent = (uint32_t *)(pk + ent_start);
        uint32_t ebase = 0;                                               // in entries
        for (uint32_t j = 0; j < nsl; ++j) {
            int32_t p0 = a + (int32_t)j * kWave;
            int32_t rows = std::min(kWave, b - p0);
            int sh = lanes_per_row_log2(rows);
            int32_t lpr = 1 << sh;
            uint64_t width = (uint64_t)((slice_deg[p0] + lpr - 1) >> sh);
            if (width >= 65536) return false;
            desc[4 * j] = ent_start + (uint32_t)esz * ebase;
            desc[4 * j + 1] = (uint32_t)width | ((uint32_t)rows << 16) | ((uint32_t)sh << 24);
            desc[4 * j + 2] = tick_tab[4 * s + 2];
            desc[4 * j + 3] = (uint32_t)(p0 % dir.slots);
            dir.max_width = std::max(dir.max_width, (int32_t)width);
            if (stab) {
                uint32_t *e = stab + 8 * ((size_t)s * dir.smax + j);
                e[0] = tick_tab[4 * s] + (uint32_t)dir.smax + 32u * j;                  // 64 records of 8 bytes per slice
                e[1] = tick_tab[4 * s] + (ent_start + (uint32_t)esz * ebase) / 16;      // whole chunks: 64 entries a row
                e[2] = desc[4 * j + 1];
                e[3] = desc[4 * j + 2];
                e[4] = desc[4 * j + 3];
            }
            for (int32_t r = 0; r < kWave; ++r) {       // records: one per row
                uint32_t *rc = rec + 2 * ((size_t)j * kWave + r);
                if (r < rows) {
                    int32_t v = order[p0 + r];
                    rc[0] = (uint32_t)v;
                    rc[1] = (uint32_t)c[v];
                    gmap[(size_t)s * dir.wpad + (size_t)j * kWave + r] = v;
                } else {                                // padding row: never published
                    rc[0] = tick_tab[4 * s + 2];
                    rc[1] = 0;
                }
            }
            for (int32_t l = 0; l < kWave; ++l) {       // entries: lane l serves row l >> sh
                int32_t r = l >> sh, sub = l & (lpr - 1);
                int32_t v = r < rows ? order[p0 + r] : -1;
                int32_t d = v >= 0 ? csr.ptr[v + 1] - csr.ptr[v] : 0;
                for (uint32_t jj = 0; jj < (uint32_t)width; ++jj) {
                    const size_t at = (size_t)ebase + (size_t)jj * kWave + l;
                    int64_t ei = (int64_t)jj * lpr + sub;
                    uint32_t field = pad_field, te = 0;    // padding: the constant-zero slot
                    if (ei < d) {
                        int64_t e = (int64_t)csr.ptr[v] + ei;
                        int32_t pn = pos[csr.idx[e]];
                        if (is_far(s, pn)) {
                            uint32_t *fl = far_list + 2 * ((size_t)s * dir.far_cap + far_next);
                            fl[0] = (uint32_t)csr.idx[e];
                            fl[1] = (uint32_t)c[csr.idx[e]];
                            field = far_base + 8 * far_next;
                            ++far_next;
                        } else {
                            uint32_t slot = (uint32_t)(pn % dir.slots);
                            field = dir.packed ? 8 * slot : slot;
                        }
                        te = (uint32_t)csr.wt[e];
                    }
                    if (dir.ent4) {
                        ent[at] = field | (te << 16);
                    } else {
                        ent[2 * at] = field;
                        ent[2 * at + 1] = te;
                    }
                }
            }
            ebase += (uint32_t)width * kWave;
        }
        for (uint32_t j = nsl; stab && j < (uint32_t)dir.smax; ++j) {   // slices this tick does not have
            uint32_t *e = stab + 8 * ((size_t)s * dir.smax + j);
            e[0] = e[1] = tick_tab[4 * s];
            e[3] = tick_tab[4 * s + 2];
        }
    }
    return true;
}

}  // namespace

int pack_graph(int32_t n, int64_t m, int32_t L,
               const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *succ_t,
               const int32_t *pred_ptr, const int32_t *pred_idx, const int32_t *pred_eid,
               const int64_t *c, const int32_t *level_ptr, const int32_t *level_vtx,
               Packed &out) {
    if (n < 1 || m < 0 || L < 1 || m >= (int64_t)0x7fffffff) return CP_ERR_SIZE;
    if (!succ_ptr || !pred_ptr || !c || !level_ptr || !level_vtx) return CP_ERR_NULL;
    if (m > 0 && (!succ_idx || !succ_t || !pred_idx || !pred_eid)) return CP_ERR_NULL;

    int rc = check_csr(n, m, succ_ptr, succ_idx);
    if (rc) return rc;
    rc = check_csr(n, m, pred_ptr, pred_idx);
    if (rc) return rc;

    // both CSRs must describe the same multiset of edges
    std::vector<int32_t> edge_src((size_t)m);
    for (int32_t v = 0; v < n; ++v)
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) edge_src[e] = v;
    {
        std::vector<uint8_t> seen((size_t)m, 0);
        for (int32_t v = 0; v < n; ++v)
            for (int32_t j = pred_ptr[v]; j < pred_ptr[v + 1]; ++j) {
                int32_t e = pred_eid[j];
                if (e < 0 || e >= m || seen[e]) return CP_ERR_CSR;
                seen[e] = 1;
                if (succ_idx[e] != v || edge_src[e] != pred_idx[j]) return CP_ERR_CSR;
            }
    }

    // level index: a partition of V in which every edge climbs
    if (level_ptr[0] != 0 || level_ptr[L] != n) return CP_ERR_LEVELS;
    std::vector<int32_t> level((size_t)n, -1);
    for (int32_t l = 0; l < L; ++l) {
        if (level_ptr[l + 1] < level_ptr[l]) return CP_ERR_LEVELS;
        for (int32_t i = level_ptr[l]; i < level_ptr[l + 1]; ++i) {
            int32_t v = level_vtx[i];
            if (v < 0 || v >= n || level[v] >= 0) return CP_ERR_LEVELS;
            level[v] = l;
        }
    }
    for (int64_t e = 0; e < m; ++e)
        if (level[edge_src[e]] >= level[succ_idx[e]]) return CP_ERR_LEVELS;

    int64_t max_c = 0, max_t = 0;
    for (int32_t v = 0; v < n; ++v) {
        if (c[v] < 0) return CP_ERR_NEGATIVE;
        max_c = std::max(max_c, c[v]);
    }
    for (int64_t e = 0; e < m; ++e) {
        if (succ_t[e] < 0) return CP_ERR_NEGATIVE;
        max_t = std::max(max_t, succ_t[e]);
    }

    // U0: longest path with w = c and x = t bounds every tick value for every s, B >= 1
    const uint64_t kLimit = 1ull << 62;
    uint64_t u0 = 0;
    {
        std::vector<uint64_t> b0((size_t)n, 0);
        for (int32_t l = L - 1; l >= 0; --l)
            for (int32_t i = level_ptr[l]; i < level_ptr[l + 1]; ++i) {
                int32_t v = level_vtx[i];
                uint64_t best = 0;
                for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) {
                    uint64_t cand = (uint64_t)succ_t[e] + b0[succ_idx[e]];  // each term < 2^63
                    best = std::max(best, cand);
                }
                if (best >= kLimit || (uint64_t)c[v] >= kLimit) return CP_ERR_OVERFLOW;
                uint64_t val = best + (uint64_t)c[v];
                if (val >= kLimit) return CP_ERR_OVERFLOW;
                b0[v] = val;
                u0 = std::max(u0, val);
            }
    }

    Packed &P = out;
    P.n = n; P.m = m; P.L = L;
    P.narrow = (uint64_t)max_c < (1ull << 32) && (uint64_t)max_t < (1ull << 32);

    cp_graph_info &info = P.info;
    info = cp_graph_info{};
    info.n = n; info.L = L; info.m = m;
    info.max_c = max_c; info.max_t = max_t;
    info.raw_path_bound = (int64_t)u0;
    info.min_tick_bytes = u0 < (1ull << 31) ? 4 : 8;
    std::vector<int32_t> sources;
    for (int32_t v = 0; v < n; ++v) {
        int32_t od = succ_ptr[v + 1] - succ_ptr[v], id = pred_ptr[v + 1] - pred_ptr[v];
        info.max_out_degree = std::max(info.max_out_degree, od);
        info.max_in_degree = std::max(info.max_in_degree, id);
        if (od == 0) info.num_sinks++;
        if (id == 0) sources.push_back(v);
    }
    info.num_sources = (int32_t)sources.size();
    for (int32_t l = 0; l < L; ++l)
        info.max_level_width = std::max(info.max_level_width, level_ptr[l + 1] - level_ptr[l]);
    P.max_width = info.max_level_width;

    Csr succ{succ_ptr, succ_idx, {}}, pred{pred_ptr, pred_idx, {}};
    succ.wt.assign(succ_t, succ_t + m);
    pred.wt.resize((size_t)m);
    for (int64_t j = 0; j < m; ++j) pred.wt[j] = succ_t[pred_eid[j]];

    std::vector<int32_t> order_b, order_t;
    sweep_order(n, L, level_ptr, level_vtx, succ_ptr, /*forward=*/false, order_b, P.col_b);
    sweep_order(n, L, level_ptr, level_vtx, pred_ptr, /*forward=*/true, order_t, P.col_t);

    try {
        P.blob.clear();
        BlobWriter w(P.blob);
        pack_column_dir(w, n, m, P.narrow, succ, order_b, P.col_b);
        pack_column_dir(w, n, m, P.narrow, pred, order_t, P.col_t);
        if (P.narrow) {
            P.c_off = w.reserve(sizeof(uint32_t) * (size_t)n);
            uint32_t *cp = w.at<uint32_t>(P.c_off);
            for (int32_t v = 0; v < n; ++v) cp[v] = (uint32_t)c[v];
        } else {
            P.c_off = w.reserve(sizeof(int64_t) * (size_t)n);
            std::memcpy(w.at<int64_t>(P.c_off), c, sizeof(int64_t) * (size_t)n);
        }
        P.sources_off = w.reserve(sizeof(int32_t) * sources.size());
        std::memcpy(w.at<int32_t>(P.sources_off), sources.data(), sizeof(int32_t) * sources.size());

        P.have_window = false;
        if (P.narrow) {
            size_t mark = P.blob.size();
            bool ok = pack_window_dir(w, n, L, c, max_t, info.min_tick_bytes == 4, succ, order_b, P.col_b, P.win_b) &&
                      pack_window_dir(w, n, L, c, max_t, info.min_tick_bytes == 4, pred, order_t, P.col_t, P.win_t);
            if (ok) P.have_window = true;
            else P.blob.resize(mark);
        }
        P.blob.resize(align_up(P.blob.size()));
    } catch (const std::bad_alloc &) {
        return CP_ERR_ALLOC;
    }

    info.window_slots_b = P.have_window ? P.win_b.slots : 0;
    info.window_slots_t = P.have_window ? P.win_t.slots : 0;
    info.window_packet_bytes_b = P.have_window ? 16 * P.win_b.max_chunks : 0;
    info.window_packet_bytes_t = P.have_window ? 16 * P.win_t.max_chunks : 0;
    info.window_ticks_b = P.have_window ? P.win_b.ticks : 0;
    info.window_ticks_t = P.have_window ? P.win_t.ticks : 0;
    info.window_slices_b = P.have_window ? P.win_b.smax : 0;
    info.window_slices_t = P.have_window ? P.win_t.smax : 0;
    info.window_far_b = P.have_window ? P.win_b.far_cap : 0;
    info.window_far_t = P.have_window ? P.win_t.far_cap : 0;
    info.blob_bytes = P.blob.size();
    return CP_OK;
}

}  // namespace cpeval
