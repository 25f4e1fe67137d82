/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Plain CPU evaluation of the weighted critical path of a data-flow DAG under
 * candidate device partitions.  It is the definition written out: one partition
 * at a time, one vertex at a time, int64 throughout, partition-major arrays.
 * It shares no code, header, table or constant with the GPU library; only the
 * tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What is computed (paper, section 2 for the model; section 4.1 and its
 * equation for PCT; section 3.2 and its two rank equations; section 2's
 * remark on the artificial final sink):
 *
 *   w(v)  = ceil( c(v) / s[p(v)] )                     execution time of v on its device
 *   x(e)  = 0                      if p(u) == p(v)      transfer time along e = (u -> v)
 *         = ceil( t(e) / B[p(u)][p(v)] )  otherwise
 *   b(v)  = w(v) + max over out-edges e=(v->u) of ( x(e) + b(u) ),  empty max = 0
 *           -- the paper's PCT: a sink's value is its own execution time
 *   tl(v) = max over in-edges e=(u->v) of ( tl(u) + w(u) + x(e) ),  empty max = 0
 *           -- the downward rank without the vertex's own term
 *   CP    = max_v b(v)   (= start time of the zero-cost final sink joined to all sinks)
 *   mask(v) = [ tl(v) + b(v) == CP ]
 *
 * Integer ticks: each term is rounded up on its own, ceil(a/d) = (a + d - 1) div d
 * for a >= 0, d >= 1.
 *
 * The vertex order comes from Kahn's algorithm on the successor lists; the
 * level index used by the GPU path is never consulted.  tl is pushed along
 * out-edges, so the predecessor arrays are not consulted either.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int64_t cp_oracle_ceil_div(int64_t a, int64_t d) { return (a + d - 1) / d; }

/* section 2: execution time = complexity / speed of the device */
int64_t cp_oracle_vertex_cost(int64_t c, int64_t s) { return cp_oracle_ceil_div(c, s); }

/* section 4.1: transfer time is 0 on one device, else volume / rate between the two;
 * bandwidth is k x k, row = device of the edge's source vertex */
int64_t cp_oracle_edge_cost(int64_t t, int pu, int pv, const int64_t *bandwidth, int k)
{
    if (pu == pv) return 0;
    return cp_oracle_ceil_div(t, bandwidth[(size_t)pu * k + pv]);
}

/* Kahn's algorithm on successor lists.  order[n] receives the vertices, sources
 * first.  Returns 0, or -1 if the graph has a cycle. */
int cp_oracle_topo_order(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx, int32_t *order)
{
    int32_t *indeg = (int32_t *)calloc((size_t)n + 1, sizeof(int32_t));
    if (!indeg) return -2;
    for (int32_t v = 0; v < n; ++v)
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) indeg[succ_idx[e]]++;
    int32_t head = 0, tail = 0;
    for (int32_t v = 0; v < n; ++v)
        if (indeg[v] == 0) order[tail++] = v;
    while (head < tail) {
        int32_t v = order[head++];
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) {
            int32_t u = succ_idx[e];
            if (--indeg[u] == 0) order[tail++] = u;
        }
    }
    free(indeg);
    return tail == n ? 0 : -1;
}

/* One partition.  p[n] device of each vertex; outputs b[n], tl[n], mask[n] (any may
 * be NULL except that b and tl are needed internally, so scratch is used). */
static int64_t eval_one(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx,
                        const int64_t *succ_t, const int64_t *c, int k, const int64_t *speeds,
                        const int64_t *bandwidth, const int32_t *order, const uint8_t *p,
                        int64_t *w, int64_t *b, int64_t *tl, uint8_t *mask)
{
    for (int32_t v = 0; v < n; ++v) w[v] = cp_oracle_vertex_cost(c[v], speeds[p[v]]);

    /* b-level: sinks first */
    for (int32_t i = n - 1; i >= 0; --i) {
        int32_t v = order[i];
        int64_t best = 0;
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) {
            int32_t u = succ_idx[e];
            int64_t cand = cp_oracle_edge_cost(succ_t[e], p[v], p[u], bandwidth, k) + b[u];
            if (cand > best) best = cand;
        }
        b[v] = w[v] + best;
    }

    /* t-level: sources first, pushed along out-edges */
    for (int32_t v = 0; v < n; ++v) tl[v] = 0;
    for (int32_t i = 0; i < n; ++i) {
        int32_t v = order[i];
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) {
            int32_t u = succ_idx[e];
            int64_t cand = tl[v] + w[v] + cp_oracle_edge_cost(succ_t[e], p[v], p[u], bandwidth, k);
            if (cand > tl[u]) tl[u] = cand;
        }
    }

    int64_t cp = 0;
    for (int32_t v = 0; v < n; ++v)
        if (b[v] > cp) cp = b[v];
    if (mask)
        for (int32_t v = 0; v < n; ++v) mask[v] = (uint8_t)(tl[v] + b[v] == cp);
    return cp;
}

/*
 * All partitions.  assignments is [P][n]; cp_out [P]; b_out, tl_out [P][n] int64;
 * mask_out [P][n] bytes (0/1).  b_out, tl_out, mask_out may be NULL.
 * threads <= 0 means one thread.  Returns 0; -1 cycle; -2 out of memory;
 * -3 bad argument (device id >= k, speed < 1, off-diagonal bandwidth < 1, negative weight).
 * *threads_used (may be NULL) receives the number of threads that ran.
 */
int cp_oracle_eval(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx,
                   const int64_t *succ_t, const int64_t *c, int k, const int64_t *speeds,
                   const int64_t *bandwidth, int32_t P, const uint8_t *assignments,
                   int64_t *cp_out, int64_t *b_out, int64_t *tl_out, uint8_t *mask_out,
                   int threads, int *threads_used)
{
    if (n < 0 || P < 0 || k < 1 || k > 256) return -3;
    for (int i = 0; i < k; ++i) {
        if (speeds[i] < 1) return -3;
        for (int j = 0; j < k; ++j)
            if (i != j && bandwidth[(size_t)i * k + j] < 1) return -3;
    }
    int64_t m = n ? succ_ptr[n] : 0;
    for (int32_t v = 0; v < n; ++v) if (c[v] < 0) return -3;
    for (int64_t e = 0; e < m; ++e) if (succ_t[e] < 0) return -3;
    for (int64_t i = 0; i < (int64_t)P * n; ++i) if (assignments[i] >= k) return -3;

    int32_t *order = (int32_t *)malloc(((size_t)n + 1) * sizeof(int32_t));
    if (!order) return -2;
    int rc = cp_oracle_topo_order(n, succ_ptr, succ_idx, order);
    if (rc) { free(order); return rc; }

    if (threads < 1) threads = 1;
    int used = 1, failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
#endif
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        int64_t *w = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
        int64_t *bs = b_out ? NULL : (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
        int64_t *ts = tl_out ? NULL : (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
        if (!w || (!b_out && !bs) || (!tl_out && !ts)) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int32_t j = 0; j < P; ++j) {
            if (failed) continue;
            int64_t *b = b_out ? b_out + (size_t)j * n : bs;
            int64_t *tl = tl_out ? tl_out + (size_t)j * n : ts;
            uint8_t *mk = mask_out ? mask_out + (size_t)j * n : NULL;
            cp_out[j] = eval_one(n, succ_ptr, succ_idx, succ_t, c, k, speeds, bandwidth, order,
                                 assignments + (size_t)j * n, w, b, tl, mk);
        }
        free(w); free(bs); free(ts);
    }
    free(order);
    if (threads_used) *threads_used = used;
    return failed ? -2 : 0;
}


/*
 * One critical path per partition (paper, section 3.2.2: "compute the critical
 * path"; the paper walks back from the best sink and leaves ties open).  Reading
 * taken here: among all source-to-sink paths whose cost equals CP, the one whose
 * vertex sequence is lexicographically smallest.  It starts at the lowest-numbered
 * vertex without predecessors whose b equals CP and always moves to the
 * lowest-numbered successor u of v with b(v) = w(v) + x(v->u) + b(u); such a
 * successor exists for every vertex that has successors, so the walk ends at a sink.
 *
 * path_out is [P][max_len] (unused tail = -1), len_out [P].  Returns 0; -1 cycle;
 * -2 out of memory; -3 bad argument; -4 a path longer than max_len.
 */
int cp_oracle_critical_path(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx,
                            const int64_t *succ_t, const int64_t *c, int k, const int64_t *speeds,
                            const int64_t *bandwidth, int32_t P, const uint8_t *assignments,
                            int32_t max_len, int32_t *path_out, int32_t *len_out)
{
    int64_t *cp = (int64_t *)malloc(((size_t)P + 1) * sizeof(int64_t));
    int64_t *b = (int64_t *)malloc(((size_t)P * n + 1) * sizeof(int64_t));
    uint8_t *has_pred = (uint8_t *)calloc((size_t)n + 1, 1);
    if (!cp || !b || !has_pred) { free(cp); free(b); free(has_pred); return -2; }
    int rc = cp_oracle_eval(n, succ_ptr, succ_idx, succ_t, c, k, speeds, bandwidth, P, assignments,
                            cp, b, NULL, NULL, 1, NULL);
    if (rc) { free(cp); free(b); free(has_pred); return rc; }
    for (int32_t v = 0; v < n; ++v)
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) has_pred[succ_idx[e]] = 1;
    for (int32_t j = 0; j < P && rc == 0; ++j) {
        const uint8_t *p = assignments + (size_t)j * n;
        const int64_t *bj = b + (size_t)j * n;
        int32_t *path = path_out + (size_t)j * max_len;
        for (int32_t i = 0; i < max_len; ++i) path[i] = -1;
        int32_t v = -1;
        for (int32_t u = 0; u < n; ++u)
            if (!has_pred[u] && bj[u] == cp[j]) { v = u; break; }
        int32_t len = 0;
        while (v >= 0) {
            if (len >= max_len) { rc = -4; break; }
            path[len++] = v;
            int64_t rest = bj[v] - cp_oracle_vertex_cost(c[v], speeds[p[v]]);
            int32_t next = -1;
            for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) {
                int32_t u = succ_idx[e];
                if (cp_oracle_edge_cost(succ_t[e], p[v], p[u], bandwidth, k) + bj[u] == rest &&
                    (next < 0 || u < next))
                    next = u;
            }
            v = next;
        }
        len_out[j] = len;
    }
    free(cp); free(b); free(has_pred);
    return rc;
}

/*
 * Device-free ranks of section 3.2 (upward rank, downward rank and their sum, the
 * total rank of section 3.2.1), written out from the two rank equations:
 *   upRank(v)   = c(v) + max over successors u of upRank(u)      (c(v) alone for a sink)
 *   downRank(v) = c(v) + max over predecessors u of downRank(u)  (c(v) alone for a source)
 *   totalRank(v) = upRank(v) + downRank(v)
 * Both equations add the vertex's own c, so the total counts c(v) twice.
 * up, down, total are [n].  Returns 0; -1 cycle; -2 out of memory.
 */
int cp_oracle_ranks(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *c,
                    int64_t *up, int64_t *down, int64_t *total)
{
    int32_t *order = (int32_t *)malloc(((size_t)n + 1) * sizeof(int32_t));
    if (!order) return -2;
    int rc = cp_oracle_topo_order(n, succ_ptr, succ_idx, order);
    if (rc) { free(order); return rc; }
    for (int32_t i = n - 1; i >= 0; --i) {
        int32_t v = order[i];
        int64_t best = 0;
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e)
            if (up[succ_idx[e]] > best) best = up[succ_idx[e]];
        up[v] = best + c[v];
    }
    for (int32_t v = 0; v < n; ++v) down[v] = 0;
    for (int32_t i = 0; i < n; ++i) {          /* down[v] holds the best predecessor rank so far */
        int32_t v = order[i];
        down[v] += c[v];
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e)
            if (down[v] > down[succ_idx[e]]) down[succ_idx[e]] = down[v];
    }
    for (int32_t v = 0; v < n; ++v) total[v] = up[v] + down[v];
    free(order);
    return 0;
}

/*
 * PCT priority order (section 4.1: a device always runs the executable vertex with the
 * highest PCT; PCT is computed once after partitioning and the schedule reused).  Per
 * partition, the static priority list of every device: its vertices by descending
 * PCT = b, equal values by ascending vertex number.  order_out[j] lists the vertices
 * of device 0, then device 1, ...; seg_out[j][d] .. seg_out[j][d+1] is device d's range.
 * Written as the definition: a comparison sort under the key (device, -b, vertex).
 * assignments and b are [P][n], order_out [P][n], seg_out [P][k+1].
 * Returns 0; -2 out of memory; -3 a device id >= k.
 */
typedef struct { int64_t b; int32_t v; int32_t dev; } pct_item;

static int pct_before(const void *x, const void *y)
{
    const pct_item *a = (const pct_item *)x, *c = (const pct_item *)y;
    if (a->dev != c->dev) return a->dev < c->dev ? -1 : 1;
    if (a->b != c->b) return a->b > c->b ? -1 : 1;       /* higher PCT first */
    if (a->v != c->v) return a->v < c->v ? -1 : 1;
    return 0;
}

int cp_oracle_pct_order(int32_t n, int k, int32_t P, const uint8_t *assignments, const int64_t *b,
                        int32_t *order_out, int32_t *seg_out, int threads)
{
    int rc = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t j = 0; j < P; ++j) {
        pct_item *it = (pct_item *)malloc(((size_t)n + 1) * sizeof(pct_item));
        if (!it) {
#pragma omp atomic write
            rc = -2;
            continue;
        }
        int32_t *seg = seg_out + (size_t)j * (k + 1);
        for (int d = 0; d <= k; ++d) seg[d] = 0;
        int bad = 0;
        for (int32_t v = 0; v < n; ++v) {
            int dev = assignments[(size_t)j * n + v];
            if (dev >= k) { bad = 1; break; }
            it[v].b = b[(size_t)j * n + v];
            it[v].v = v;
            it[v].dev = dev;
            seg[dev + 1] += 1;
        }
        if (bad) {
#pragma omp atomic write
            rc = -3;
            free(it);
            continue;
        }
        qsort(it, (size_t)n, sizeof(pct_item), pct_before);
        for (int32_t i = 0; i < n; ++i) order_out[(size_t)j * n + i] = it[i].v;
        for (int d = 0; d < k; ++d) seg[d + 1] += seg[d];
        free(it);
    }
    return rc;
}

/*
 * Validity of partitions under the two placement constraints of section 2: every
 * collocation pair (v_i, v_j) must share a device, and every device constraint
 * (v_i, d_j) must have p(v_i) = d_j.  One pair at a time, one partition at a time.
 * pairs is [num_pairs][2] vertices, pins is [num_pins][2] = {vertex, device};
 * valid_out[j] = 1 if partition j meets all of them, violations_out[j] (may be NULL)
 * counts the constraints it breaks.  Returns 0; -3 an index out of range.
 */
int cp_oracle_validate(int32_t n, int k, int32_t P, const uint8_t *assignments,
                       int64_t num_pairs, const int32_t *pairs, int64_t num_pins, const int32_t *pins,
                       uint8_t *valid_out, int32_t *violations_out)
{
    for (int64_t i = 0; i < num_pairs; ++i)
        if (pairs[2 * i] < 0 || pairs[2 * i] >= n || pairs[2 * i + 1] < 0 || pairs[2 * i + 1] >= n) return -3;
    for (int64_t i = 0; i < num_pins; ++i)
        if (pins[2 * i] < 0 || pins[2 * i] >= n || pins[2 * i + 1] < 0 || pins[2 * i + 1] >= k) return -3;
    for (int32_t j = 0; j < P; ++j) {
        const uint8_t *p = assignments + (size_t)j * n;
        int32_t broken = 0;
        for (int64_t i = 0; i < num_pairs; ++i)
            if (p[pairs[2 * i]] != p[pairs[2 * i + 1]]) ++broken;
        for (int64_t i = 0; i < num_pins; ++i)
            if (p[pins[2 * i]] != pins[2 * i + 1]) ++broken;
        valid_out[j] = broken == 0;
        if (violations_out) violations_out[j] = broken;
    }
    return 0;
}

/*
 * Critical-path move search.  The paper's path-based strategies (section 3.2) rest on
 * one idea: the critical path decides the running time, so its vertices deserve the
 * best placement.  This is that idea as a local search over partitions, one vertex
 * move at a time (the paper itself stops at a constructive heuristic):
 *
 *   neighbourhood of p = all partitions that differ from p in exactly one vertex of
 *   p's critical path (the lexicographically smallest one), that vertex placed on any
 *   other device.  Candidate number j = i * (k-1) + r moves path vertex number i to
 *   the r-th device other than its own (devices in increasing order).
 *
 *   step: evaluate CP of every candidate that meets the placement constraints, take
 *   the smallest (lowest candidate number on ties); if it is smaller than CP(p), move
 *   there and repeat, else stop.
 */
int cp_oracle_neighbours(int32_t n, int k, const uint8_t *base, int32_t len, const int32_t *path,
                         uint8_t *out)
{
    if (k < 2) return 0;
    for (int32_t i = 0; i < len; ++i) {
        int32_t v = path[i];
        if (v < 0 || v >= n) return -3;
        for (int r = 0; r < k - 1; ++r) {
            uint8_t *row = out + ((size_t)i * (k - 1) + r) * n;
            memcpy(row, base, (size_t)n);
            row[v] = (uint8_t)(r < base[v] ? r : r + 1);
        }
    }
    return 0;
}

/* Lowest index with the smallest cp among the entries with valid != 0 (all, if valid is
 * NULL).  index_out = -1 and value_out untouched when there is none. */
void cp_oracle_argmin(int32_t P, const int64_t *cp, const uint8_t *valid, int32_t *index_out,
                      int64_t *value_out)
{
    *index_out = -1;
    for (int32_t j = 0; j < P; ++j) {
        if (valid && !valid[j]) continue;
        if (*index_out < 0 || cp[j] < *value_out) { *index_out = j; *value_out = cp[j]; }
    }
}

/*
 * The whole search from `assignment` (in: start, out: result).  cp_trace[0] is the
 * start's CP, cp_trace[i] the CP after move i; moves_out[i] = {vertex, new device}.
 * Returns the number of moves made (<= max_moves) or a negative error.
 */
int cp_oracle_search(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *succ_t,
                     const int64_t *c, int k, const int64_t *speeds, const int64_t *bandwidth,
                     uint8_t *assignment, int64_t num_pairs, const int32_t *pairs, int64_t num_pins,
                     const int32_t *pins, int32_t max_moves, int32_t max_len, int64_t *cp_trace,
                     int32_t *moves_out, int threads)
{
    int32_t *path = (int32_t *)malloc(((size_t)max_len + 1) * sizeof(int32_t));
    size_t max_cand = (size_t)max_len * (size_t)(k > 1 ? k - 1 : 1);
    uint8_t *cand = (uint8_t *)malloc(max_cand * (size_t)n + 1);
    int64_t *cp = (int64_t *)malloc((max_cand + 1) * sizeof(int64_t));
    uint8_t *valid = (uint8_t *)malloc(max_cand + 1);
    int moves = 0, rc = 0;
    if (!path || !cand || !cp || !valid) { rc = -2; goto done; }
    for (;;) {
        int64_t cp_base;
        int32_t len;
        rc = cp_oracle_eval(n, succ_ptr, succ_idx, succ_t, c, k, speeds, bandwidth, 1, assignment, &cp_base,
                            NULL, NULL, NULL, 1, NULL);
        if (rc) goto done;
        cp_trace[moves] = cp_base;
        if (moves >= max_moves || k < 2) break;
        rc = cp_oracle_critical_path(n, succ_ptr, succ_idx, succ_t, c, k, speeds, bandwidth, 1, assignment,
                                     max_len, path, &len);
        if (rc) goto done;
        rc = cp_oracle_neighbours(n, k, assignment, len, path, cand);
        if (rc) goto done;
        int32_t ncand = len * (k - 1);
        rc = cp_oracle_eval(n, succ_ptr, succ_idx, succ_t, c, k, speeds, bandwidth, ncand, cand, cp, NULL,
                            NULL, NULL, threads, NULL);
        if (rc) goto done;
        rc = cp_oracle_validate(n, k, ncand, cand, num_pairs, pairs, num_pins, pins, valid, NULL);
        if (rc) goto done;
        int32_t best;
        int64_t best_cp = 0;
        cp_oracle_argmin(ncand, cp, valid, &best, &best_cp);
        if (best < 0 || best_cp >= cp_base) break;
        int32_t v = path[best / (k - 1)];
        uint8_t d = cand[(size_t)best * n + v];
        assignment[v] = d;
        moves_out[2 * moves] = v;
        moves_out[2 * moves + 1] = d;
        ++moves;
    }
    rc = moves;
done:
    free(path); free(cand); free(cp); free(valid);
    return rc;
}

/*
 * The paper's Critical Path partitioning strategy (section 3.2.2), as a start
 * partition for the search:
 *   1. the critical path is computed from the ranks, which know no devices: vertex cost
 *      c(v), no transfer cost (the rank equations of section 3.2 add c only);
 *   2. it goes to the fastest device (largest s, lowest number on ties) as a whole
 *      (memory capacities are not modelled, so it always fits);
 *   3. every other vertex, in increasing vertex number, goes to the device d with the
 *      smallest  load(d) + w(v, d)  (lowest number on ties), where load(d) is the sum of the
 *      execution times w(u, d) = ceil(c(u) / s[d]) of the vertices already on d, the
 *      critical path included (the strategy's load equation, in integer ticks).
 * assign_out is [n].  Returns 0 or a negative error of the functions it calls.
 */
int cp_oracle_seed(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *c,
                   int k, const int64_t *speeds, int32_t max_len, uint8_t *assign_out)
{
    int64_t m = n ? succ_ptr[n] : 0;
    int64_t *zero_t = (int64_t *)calloc((size_t)m + 1, sizeof(int64_t));
    uint8_t *one_dev = (uint8_t *)calloc((size_t)n + 1, 1);
    int32_t *path = (int32_t *)malloc(((size_t)max_len + 1) * sizeof(int32_t));
    uint8_t *on_path = (uint8_t *)calloc((size_t)n + 1, 1);
    int64_t *load = (int64_t *)calloc((size_t)k + 1, sizeof(int64_t));
    int rc = -2;
    if (zero_t && one_dev && path && on_path && load) {
        const int64_t unit = 1;
        int32_t len = 0;
        rc = cp_oracle_critical_path(n, succ_ptr, succ_idx, zero_t, c, 1, &unit, &unit, 1, one_dev, max_len,
                                     path, &len);
        if (rc == 0) {
            int fastest = 0;
            for (int d = 1; d < k; ++d)
                if (speeds[d] > speeds[fastest]) fastest = d;
            for (int32_t i = 0; i < len; ++i) {
                on_path[path[i]] = 1;
                assign_out[path[i]] = (uint8_t)fastest;
                load[fastest] += cp_oracle_vertex_cost(c[path[i]], speeds[fastest]);
            }
            for (int32_t v = 0; v < n; ++v) {
                if (on_path[v]) continue;
                int best = 0;
                int64_t best_val = load[0] + cp_oracle_vertex_cost(c[v], speeds[0]);
                for (int d = 1; d < k; ++d) {
                    int64_t val = load[d] + cp_oracle_vertex_cost(c[v], speeds[d]);
                    if (val < best_val) { best = d; best_val = val; }
                }
                assign_out[v] = (uint8_t)best;
                load[best] = best_val;
            }
        }
    }
    free(zero_t); free(one_dev); free(path); free(on_path); free(load);
    return rc;
}


/*
 * List-scheduling simulation of one iteration (paper, section 4: the scheduling
 * criteria (1)-(6); section 4.1: PCT scheduling; section 5.1: the FIFO baseline;
 * section 5: an event-based simulation gives the execution time of one iteration).
 *
 * The reading taken here, in integer ticks:
 *   - every device runs its own vertices one at a time, without interruption; v keeps its
 *     device busy for w(v) ticks from start(v) to finish(v) = start(v) + w(v);
 *   - the tensor of an edge e = (u -> v) is at v's device at finish(u) + x(e); transfers
 *     do not occupy devices and do not compete with each other (the model of section 2
 *     has a transfer rate per device pair and nothing else);
 *   - v is executable from ready(v) = max over in-edges of those arrival times, 0 for a
 *     vertex without predecessors;
 *   - a device that is free at time T and owns an executable, unstarted vertex starts one
 *     at T; otherwise it stays idle until the first of its vertices becomes executable
 *     (criterion (6): idle only when nothing is executable);
 *   - the choice among the executable vertices at T:
 *       FIFO (policy 0): the one that became executable first, smallest ready(v); among
 *                        equals the paper draws at random -- here the caller passes the
 *                        draw as tie[v] and the smaller tie wins (tie = NULL: the vertex
 *                        number), equal ties fall back to the smaller vertex number;
 *       PCT  (policy 1): the largest b(v) (section 4.1's path computation time), among
 *                        equals the smaller vertex number;
 *   - makespan = the largest finish time = the start time of the final sink.
 * Every vertex must cost at least one tick (c(v) >= 1): then a vertex started at T can
 * influence another device only after T, so the order in which devices that decide at the
 * same time are served does not matter.  c(v) = 0 is refused.
 *
 * How it runs: per device a plain list of the vertices whose predecessors have all
 * started (so their ready time is final) and that have not started themselves.  Step:
 * for every device d, T_d = max(free(d), smallest ready time in d's list); the device
 * with the smallest T_d (lowest number on ties) decides at T_d by a scan of its list.
 *
 * b is [P][n] (PCT only), tie [n] (FIFO only, may be NULL), makespan_out [P],
 * start_out [P][n] (may be NULL).  Returns 0; -1 cycle (a vertex never started);
 * -2 out of memory; -3 bad argument.
 */
static int64_t simulate_one(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx,
                            const int64_t *succ_t, const int64_t *c, int k, const int64_t *speeds,
                            const int64_t *bandwidth, const int32_t *indeg0, const uint8_t *p,
                            int policy, const int64_t *b, const int32_t *tie,
                            int64_t *start, int64_t *ready, int32_t *indeg,
                            int32_t *list, int32_t *list_at, int32_t *list_len,
                            int64_t *free_at, int64_t *T, uint8_t *stale)
{
    const int64_t NEVER = INT64_MAX;
    /* list of device d occupies list[list_at[d] .. list_at[d] + list_len[d]) */
    for (int d = 0; d <= k; ++d) list_at[d] = 0;
    for (int32_t v = 0; v < n; ++v) list_at[p[v] + 1]++;
    for (int d = 0; d < k; ++d) list_at[d + 1] += list_at[d];
    for (int d = 0; d < k; ++d) { list_len[d] = 0; free_at[d] = 0; stale[d] = 1; }
    for (int32_t v = 0; v < n; ++v) {
        indeg[v] = indeg0[v];
        ready[v] = 0;
        start[v] = -1;
        if (indeg[v] == 0) list[list_at[p[v]] + list_len[p[v]]++] = v;
    }
    int32_t started = 0;
    for (;;) {
        int who = -1;
        for (int d = 0; d < k; ++d) {
            if (stale[d]) {
                int64_t first = NEVER;
                for (int32_t i = 0; i < list_len[d]; ++i) {
                    int64_t r = ready[list[list_at[d] + i]];
                    if (r < first) first = r;
                }
                T[d] = first == NEVER ? NEVER : (first > free_at[d] ? first : free_at[d]);
                stale[d] = 0;
            }
            if (T[d] != NEVER && (who < 0 || T[d] < T[who])) who = d;
        }
        if (who < 0) break;
        const int64_t now = T[who];
        int32_t *mine = list + list_at[who];
        int32_t pick = -1;
        for (int32_t i = 0; i < list_len[who]; ++i) {
            const int32_t v = mine[i];
            if (ready[v] > now) continue;                 /* not executable yet */
            if (pick < 0) { pick = i; continue; }
            const int32_t u = mine[pick];
            int better;
            if (policy == 1) {
                better = b[v] > b[u] || (b[v] == b[u] && v < u);
            } else {
                const int64_t tv = tie ? tie[v] : v, tu = tie ? tie[u] : u;
                better = ready[v] < ready[u] ||
                         (ready[v] == ready[u] && (tv < tu || (tv == tu && v < u)));
            }
            if (better) pick = i;
        }
        const int32_t v = mine[pick];
        mine[pick] = mine[--list_len[who]];
        start[v] = now;
        ++started;
        const int64_t done = now + cp_oracle_vertex_cost(c[v], speeds[who]);
        free_at[who] = done;
        stale[who] = 1;
        for (int32_t e = succ_ptr[v]; e < succ_ptr[v + 1]; ++e) {
            const int32_t u = succ_idx[e];
            const int64_t here = done + cp_oracle_edge_cost(succ_t[e], who, p[u], bandwidth, k);
            if (here > ready[u]) ready[u] = here;
            if (--indeg[u] == 0) {
                list[list_at[p[u]] + list_len[p[u]]++] = u;
                stale[p[u]] = 1;
            }
        }
    }
    if (started != n) return -1;
    int64_t makespan = 0;
    for (int d = 0; d < k; ++d)
        if (free_at[d] > makespan) makespan = free_at[d];
    return makespan;
}

int cp_oracle_simulate(int32_t n, const int32_t *succ_ptr, const int32_t *succ_idx,
                       const int64_t *succ_t, const int64_t *c, int k, const int64_t *speeds,
                       const int64_t *bandwidth, int32_t P, const uint8_t *assignments,
                       int policy, const int64_t *b, const int32_t *tie,
                       int64_t *makespan_out, int64_t *start_out, int threads, int *threads_used)
{
    if (n < 0 || P < 0 || k < 1 || k > 256 || (policy != 0 && policy != 1)) return -3;
    if (policy == 1 && !b) return -3;
    for (int i = 0; i < k; ++i) {
        if (speeds[i] < 1) return -3;
        for (int j = 0; j < k; ++j)
            if (i != j && bandwidth[(size_t)i * k + j] < 1) return -3;
    }
    int64_t m = n ? succ_ptr[n] : 0;
    for (int32_t v = 0; v < n; ++v) if (c[v] < 1) return -3;
    for (int64_t e = 0; e < m; ++e) if (succ_t[e] < 0) return -3;
    for (int64_t i = 0; i < (int64_t)P * n; ++i) if (assignments[i] >= k) return -3;

    int32_t *indeg0 = (int32_t *)calloc((size_t)n + 1, sizeof(int32_t));
    if (!indeg0) return -2;
    for (int64_t e = 0; e < m; ++e) indeg0[succ_idx[e]]++;

    if (threads < 1) threads = 1;
    int used = 1, failed = 0, cyclic = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
#endif
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        int64_t *st = start_out ? NULL : (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
        int64_t *ready = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
        int32_t *indeg = (int32_t *)malloc(((size_t)n + 1) * sizeof(int32_t));
        int32_t *list = (int32_t *)malloc(((size_t)n + 1) * sizeof(int32_t));
        int32_t *list_at = (int32_t *)malloc(((size_t)k + 2) * sizeof(int32_t));
        int32_t *list_len = (int32_t *)malloc(((size_t)k + 1) * sizeof(int32_t));
        int64_t *free_at = (int64_t *)malloc(((size_t)k + 1) * sizeof(int64_t));
        int64_t *T = (int64_t *)malloc(((size_t)k + 1) * sizeof(int64_t));
        uint8_t *stale = (uint8_t *)malloc((size_t)k + 1);
        if ((!start_out && !st) || !ready || !indeg || !list || !list_at || !list_len || !free_at || !T ||
            !stale) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int32_t j = 0; j < P; ++j) {
            if (failed) continue;
            int64_t *s = start_out ? start_out + (size_t)j * n : st;
            int64_t r = simulate_one(n, succ_ptr, succ_idx, succ_t, c, k, speeds, bandwidth, indeg0,
                                     assignments + (size_t)j * n, policy,
                                     b ? b + (size_t)j * n : NULL, tie, s, ready, indeg, list, list_at,
                                     list_len, free_at, T, stale);
            if (r < 0) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
                cyclic = 1;
            }
            makespan_out[j] = r;
        }
        free(st); free(ready); free(indeg); free(list); free(list_at); free(list_len);
        free(free_at); free(T); free(stale);
    }
    free(indeg0);
    if (threads_used) *threads_used = used;
    if (failed) return -2;
    return cyclic ? -1 : 0;
}
