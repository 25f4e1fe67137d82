/*
 * cpeval -- batched evaluation of the weighted critical path of a data-flow DAG
 * under many candidate device partitions, on one AMD MI355X (gfx950).
 *
 * Model (paper, section 2): a DAG G=(V,E) with n vertices and m edges, vertex
 * complexity c(v) >= 0, edge volume t(e) >= 0, k devices of speed s[i] >= 1 and a
 * k x k bandwidth matrix B (row = device of the edge's source vertex, column =
 * device of its target; the diagonal is never read).  A partition p: V -> D is
 * one row of `assignments`.  Costs are integer ticks, each term rounded up on
 * its own:
 *
 *   w(v)  = ceil(c(v) / s[p(v)])                             (section 2: time = complexity / speed)
 *   x(e)  = 0 if p(u) == p(v), else ceil(t(e) / B[p(u)][p(v)])   for e = (u -> v)   (section 4.1)
 *   b(v)  = w(v) + max over out-edges (x(e) + b(head)), empty max = 0
 *           (section 4.1, the PCT equation; a sink's value is its own execution time)
 *   tl(v) = max over in-edges (tl(tail) + w(tail) + x(e)), empty max = 0
 *           (section 3.2, the downward rank without the vertex's own term)
 *   CP    = max_v b(v)     (section 2: the start time of a zero-cost final sink
 *                           joined to every sink by zero-cost edges)
 *   mask(v) = [tl(v) + b(v) == CP]    (the union of all critical paths, section 3.2.2)
 *
 * Multi-edges are allowed (the costlier one decides), c = 0 and t = 0 are allowed,
 * m = 0 is allowed.  B need not be symmetric.
 *
 * Calling convention: plain C, no exceptions, no aborts.  Every function returns
 * CP_OK (0) or a negative CP_ERR_* code.  "host" pointers are ordinary memory that
 * is only read during the call; "device" pointers are HIP device memory owned by
 * the caller.  The library never allocates or frees device memory.  `stream` is
 * a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef CPEVAL_H
#define CPEVAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- error codes (return values) ---- */
#define CP_OK              0
#define CP_ERR_NULL       (-1)   /* a required pointer is NULL */
#define CP_ERR_SIZE       (-2)   /* n < 1, m < 0, L < 1, batch < 1, k < 1 or k > 255 */
#define CP_ERR_CSR        (-3)   /* non-monotone ptr, index out of range, succ/pred mismatch */
#define CP_ERR_LEVELS     (-4)   /* level index is not a partition of V, or an edge does not go to a higher level */
#define CP_ERR_NEGATIVE   (-5)   /* c(v) < 0 or t(e) < 0 */
#define CP_ERR_SPEED      (-6)   /* s[i] < 1 */
#define CP_ERR_BANDWIDTH  (-7)   /* off-diagonal B[i][j] < 1 */
#define CP_ERR_OVERFLOW   (-8)   /* longest raw path >= 2^62, or 32-bit ticks asked for but not provably safe */
#define CP_ERR_WORKSPACE  (-9)   /* workspace or blob too small or misaligned */
#define CP_ERR_HIP        (-10)  /* a HIP runtime call failed */
#define CP_ERR_STATE      (-11)  /* graph not uploaded yet, or profile slot out of range */
#define CP_ERR_ARG        (-12)  /* unknown enum value, or an output requested without the outputs it depends on */
#define CP_ERR_ALLOC      (-13)  /* host allocation failed */

/* ---- value written to *status_out by the device ---- */
#define CP_STATUS_OK             0
#define CP_STATUS_BAD_DEVICE_ID  1   /* some assignments entry is >= k: the call's outputs are meaningless
                                        (the entry was replaced by a valid device so that no access leaves its table) */
#define CP_STATUS_BAD_CONSTRAINT  4   /* cp_validate: a constraint names a vertex >= n or a device >= k; it was skipped */
#define CP_STATUS_B_OUT_OF_RANGE 2   /* cp_pct_order: some b lies outside [0, max_b]: the order is meaningless;
                                        status values are bit flags and may be or-ed */
#define CP_STATUS_BAD_TIE        8   /* cp_simulate: tie is not a permutation of 0 .. n-1: nothing was simulated */
#define CP_STATUS_INCOMPLETE     16  /* cp_simulate: a partition ended with vertices that never started (cannot
                                        happen on a graph that cp_graph_create accepted) */

/* ---- enums ---- */
#define CP_TICK_I32  4   /* b-level / t-level stored as int32 (only if the graph's bound allows) */
#define CP_TICK_I64  8   /* stored as int64 */

#define CP_ASSIGN_PARTITION_MAJOR 0   /* assignments[batch][n] */
#define CP_ASSIGN_VERTEX_MAJOR    1   /* assignments[n][batch] */

/* Layout of the per-vertex outputs.  Vertex-major suits consumers that look at one
 * vertex across partitions (and is what the wave-column plan produces natively);
 * partition-major gives every partition one contiguous row (what the resident-window
 * plan, the priority lists and the critical-path walk work on natively).  Every plan
 * honours either choice. */
#define CP_OUT_VERTEX_MAJOR       0   /* b, tl [n][batch]; mask [n][ceil(batch/64)], bit = partition */
#define CP_OUT_PARTITION_MAJOR    1   /* b, tl [batch][n]; mask [batch][ceil(n/64)], bit = vertex */

#define CP_PLAN_AUTO             0
#define CP_PLAN_WAVE_COLUMN      1   /* one wavefront = one vertex x 64 partitions; one launch per level */
#define CP_PLAN_RESIDENT_WINDOW  2   /* one workgroup = one partition; recent levels kept in LDS; one launch per sweep, or
                                        one for both sweeps where a workgroup of each fits a compute unit side by side
                                        or all workgroups of both sweeps find room on the chip at once */
#define CP_PLAN_SHARED_WINDOW_2  3   /* as 2, but one workgroup = 2 partitions behind one graph stream */
#define CP_PLAN_SHARED_WINDOW_4  4   /* ... 4 partitions */
#define CP_PLAN_STREAMED_WINDOW  6   /* as 2, but the compute wavefronts fetch the graph themselves, two ticks ahead, into
                                        registers; LDS holds only what depends on the partition */
#define CP_PLAN_COLUMN_SLICE     5   /* the wave-column layout, but one persistent workgroup owns 64 partitions and
                                        walks all levels in one launch per sweep (never chosen by CP_PLAN_AUTO) */

/* stages of one cp_eval call, in the order they run; also the index into cp_profile_read's output */
#define CP_STAGE_PREP    0   /* clear outputs, cost tables, assignment transpose */
#define CP_STAGE_BLEVEL  1   /* b-level sweep, last level to first */
#define CP_STAGE_CP      2   /* critical-path length per partition */
#define CP_STAGE_TLEVEL  3   /* t-level sweep, first level to last */
#define CP_STAGE_MASK    4   /* critical-vertex mask */
#define CP_NUM_STAGES    5

typedef struct cp_graph cp_graph;
typedef struct cp_profile cp_profile;

typedef struct cp_graph_info {
    int32_t n, L;
    int64_t m;
    int32_t max_out_degree, max_in_degree, max_level_width;
    int32_t num_sources, num_sinks;
    int64_t max_c, max_t;
    int64_t raw_path_bound;      /* U0: longest path with w = c and x = t; every tick value is <= U0 */
    int32_t min_tick_bytes;      /* 4 if U0 < 2^31, else 8 */
    int32_t window_ok;           /* 1 if the resident-window plan can run this graph */
    int32_t window_slots_b;      /* LDS slots the b-level sweep needs under that plan */
    int32_t window_slots_t;      /* ... and the t-level sweep */
    int32_t window_packet_bytes_b;   /* largest per-level packet of that plan, b-level sweep */
    int32_t window_packet_bytes_t;   /* ... and t-level sweep */
    int32_t window_far_b;        /* far reads per tick of that plan's b-level sweep (neighbours too far back for the
                                    LDS ring are read from the output array); 0 = none */
    int32_t window_far_t;        /* ... and t-level sweep */
    int32_t window_ticks_b;      /* barriers of that plan's b-level sweep: a level is cut into ticks of at most 8 slices
                                    of 64 vertices */
    int32_t window_ticks_t;      /* ... and t-level sweep */
    int32_t window_slices_b;     /* slices of the widest tick, b-level sweep */
    int32_t window_slices_t;     /* ... and t-level sweep */
    int32_t auto_plan;           /* plan CP_PLAN_AUTO resolves to for a batch of 256 (the choice is made per call) */
    int32_t uploaded;            /* 1 after cp_graph_upload */
    uint64_t blob_bytes;
} cp_graph_info;

/*
 * Validate a graph and pack it (host work only; no GPU is touched).
 *
 *   succ_ptr[n+1], succ_idx[m], succ_t[m]   successor CSR: out-edges of v are
 *       succ_ptr[v] .. succ_ptr[v+1]-1, succ_idx = head vertex, succ_t = t(e)
 *   pred_ptr[n+1], pred_idx[m], pred_eid[m] predecessor CSR: pred_idx = tail vertex,
 *       pred_eid = position of the same edge in the successor arrays
 *   c[n]                                    vertex complexity
 *   level_ptr[L+1], level_vtx[n]            vertices grouped by topological level;
 *       any grouping in which every edge goes to a strictly higher level is accepted
 *
 * All arrays are host memory, borrowed for the call.  succ_idx, succ_t, pred_idx,
 * pred_eid may be NULL when m == 0.  On success *out owns a host object to be
 * released with cp_graph_destroy.
 * Errors: CP_ERR_NULL, CP_ERR_SIZE, CP_ERR_CSR, CP_ERR_LEVELS, CP_ERR_NEGATIVE,
 * CP_ERR_OVERFLOW (longest raw path >= 2^62), CP_ERR_ALLOC.
 */
int cp_graph_create(int32_t n, int64_t m, int32_t L,
                    const int32_t *succ_ptr, const int32_t *succ_idx, const int64_t *succ_t,
                    const int32_t *pred_ptr, const int32_t *pred_idx, const int32_t *pred_eid,
                    const int64_t *c,
                    const int32_t *level_ptr, const int32_t *level_vtx,
                    cp_graph **out);

/* Facts about a created graph. */
int cp_graph_get_info(const cp_graph *g, cp_graph_info *out);

/*
 * Copy the packed graph into caller-owned device memory (>= info.blob_bytes bytes,
 * 256-byte aligned) and wait for the copy.  The memory must stay valid and
 * unmodified until cp_graph_destroy.  Errors: CP_ERR_NULL, CP_ERR_WORKSPACE, CP_ERR_HIP.
 */
int cp_graph_upload(cp_graph *g, void *device_blob, size_t blob_bytes, void *stream);

/* Release the host object (the device blob stays the caller's).  NULL is accepted. */
void cp_graph_destroy(cp_graph *g);

/*
 * Bytes of device workspace cp_eval needs for this batch size, device count,
 * assignment layout, plan (CP_PLAN_AUTO allowed), output layout and tick type.
 */
int cp_eval_workspace_bytes(const cp_graph *g, int32_t batch, int32_t k, int assign_layout,
                            int plan, int out_layout, int tick_dtype, size_t *out_bytes);

/*
 * The plan CP_PLAN_AUTO resolves to for this batch and cost model on the current
 * device (a caller may want to know it to ask for the layout that plan produces
 * directly).  Errors: as cp_eval's argument checks.
 */
int cp_eval_choose_plan(const cp_graph *g, int32_t batch, int32_t k, const int64_t *speeds,
                        const int64_t *bandwidth, int tick_dtype, int *plan_out);

/*
 * Evaluate `batch` partitions.  Only enqueues work on `stream`; it does not wait (with more
 * than 64 devices the cost tables, up to 1 MB, go through eight pinned host buffers shared
 * by the process: the ninth such call in flight waits for the first to have copied its tables).
 *
 *   assignments   device, uint8, [batch][n] or [n][batch] per assign_layout; entries < k
 *   speeds        host, int64 [k], each >= 1
 *   bandwidth     host, int64 [k][k], row = source vertex's device; off-diagonal >= 1
 *   workspace     device, >= cp_eval_workspace_bytes, 256-byte aligned; contents are scratch.
 *                 Two calls that may overlap in time need distinct workspaces.
 *   cp_out        device int64 [batch], or NULL
 *   blevel_out    device ticks, or NULL.  CP_OUT_VERTEX_MAJOR: [n][batch], partition j of vertex v at
 *                 v*batch + j; CP_OUT_PARTITION_MAJOR: [batch][n], at j*n + v
 *   tlevel_out    device ticks, same shape, or NULL
 *   mask_out      device uint64, or NULL.  CP_OUT_VERTEX_MAJOR: [n][ceil(batch/64)], bit i of word w of
 *                 row v is partition 64w+i; CP_OUT_PARTITION_MAJOR: [batch][ceil(n/64)], bit i of word w
 *                 of row j is vertex 64w+i.  Bits past the last partition / vertex are 0.
 *   tick_dtype    CP_TICK_I32 or CP_TICK_I64: element type of blevel_out / tlevel_out
 *   out_layout    CP_OUT_VERTEX_MAJOR or CP_OUT_PARTITION_MAJOR
 *   plan          CP_PLAN_AUTO, or force one (CP_ERR_ARG if it cannot run this graph / cost model)
 *   status_out    device int32, required: CP_STATUS_* after the stream has drained
 *   profile       NULL, or a profile whose next slot receives this call's stage timestamps
 *
 * Dependencies between outputs: mask_out needs cp_out, blevel_out and tlevel_out; cp_out needs
 * blevel_out unless the resident-window plan runs on a graph without far reads (info.window_far_b
 * == 0): it keeps a running maximum, so CP alone costs no output traffic (cp_eval_choose_plan tells
 * which plan CP_PLAN_AUTO takes).  CP_ERR_ARG otherwise.
 * Errors: CP_ERR_NULL, CP_ERR_SIZE, CP_ERR_SPEED, CP_ERR_BANDWIDTH, CP_ERR_OVERFLOW
 * (CP_TICK_I32 with a bound >= 2^31), CP_ERR_WORKSPACE, CP_ERR_STATE, CP_ERR_ARG, CP_ERR_HIP.
 */
int cp_eval(const cp_graph *g, int32_t batch, int32_t k,
            const uint8_t *assignments, int assign_layout,
            const int64_t *speeds, const int64_t *bandwidth,
            void *workspace, size_t workspace_bytes, void *stream,
            int64_t *cp_out, void *blevel_out, void *tlevel_out, uint64_t *mask_out,
            int tick_dtype, int out_layout, int plan, int32_t *status_out, cp_profile *profile);

/*
 * cp_eval for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as cp_eval without `workspace`, `workspace_bytes` and
 * `profile`.  The scratch memory is a fixed array of CP_STATIC_SCRATCH_BYTES bytes that is
 * part of the library's device code (every GPU the library runs on holds one until the
 * process ends), and the cost tables travel as kernel arguments, so the call allocates
 * nothing, copies nothing through the copy engine and records no memset.  (The array's
 * device address is looked up on the first call on a device; make that call outside a
 * capture.)
 *
 * Limits: k <= CP_STATIC_MAX_K (CP_ERR_SIZE) and a workspace need of at most
 * CP_STATIC_SCRATCH_BYTES (CP_ERR_WORKSPACE).  The need is the cost tables
 * ((2k^2 + k) * 8 bytes) plus, depending on how the call goes: n * batch bytes when the
 * wave-column plan reads partition-major assignments; 2 * n * batch ticks more when it
 * writes partition-major outputs; the device ids in sweep order (about n * batch bytes per
 * sweep) when the resident-window plan cannot read them straight from the caller's rows
 * (vertex-major assignments, rows not 16-byte aligned, or a graph whose levels are
 * scattered over the vertex numbers).  A resident-window call on aligned partition-major
 * rows needs the tables only.
 *
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 * (different streams or threads) race; serialise them or use cp_eval with distinct
 * workspaces.  Nothing in the array has to survive between calls.
 */
#define CP_STATIC_SCRATCH_BYTES (32u << 20)
#define CP_STATIC_MAX_K         64
int cp_eval_static(const cp_graph *g, int32_t batch, int32_t k,
                   const uint8_t *assignments, int assign_layout,
                   const int64_t *speeds, const int64_t *bandwidth, void *stream,
                   int64_t *cp_out, void *blevel_out, void *tlevel_out, uint64_t *mask_out,
                   int tick_dtype, int out_layout, int plan, int32_t *status_out);

/*
 * One critical path per partition (paper, section 3.2.2 "compute the critical path";
 * the paper leaves ties open).  Among all source-to-sink paths whose cost equals CP the
 * one with the lexicographically smallest vertex sequence is returned: it starts at the
 * lowest-numbered vertex without predecessors whose b-level equals CP and always moves
 * to the lowest-numbered successor u of v with b(v) = w(v) + x(v->u) + b(u).
 * Only enqueues work on `stream`.
 *
 *   assignments, assign_layout, speeds, bandwidth   as for cp_eval (same values as the
 *                 call that produced blevel and cp)
 *   blevel        device ticks laid out per b_layout (CP_OUT_*), cp device int64 [batch]: outputs of cp_eval
 *   workspace     device, 256-byte aligned, >= cp_eval_workspace_bytes for this batch and k
 *   max_len       row length of path_out, >= the graph's number of levels L
 *   path_out      device int32 [batch][max_len]; unused tail = -1
 *   len_out       device int32 [batch]: vertices on the path
 *   status_out    device int32, as for cp_eval
 * Errors: CP_ERR_NULL, CP_ERR_SIZE (also max_len < L), CP_ERR_ARG, CP_ERR_STATE,
 * CP_ERR_OVERFLOW, CP_ERR_WORKSPACE, CP_ERR_SPEED, CP_ERR_BANDWIDTH, CP_ERR_HIP.
 */
int cp_critical_path(const cp_graph *g, int32_t batch, int32_t k,
                     const uint8_t *assignments, int assign_layout,
                     const int64_t *speeds, const int64_t *bandwidth,
                     const void *blevel, const int64_t *cp, int tick_dtype, int b_layout,
                     void *workspace, size_t workspace_bytes, void *stream,
                     int32_t max_len, int32_t *path_out, int32_t *len_out, int32_t *status_out);

/*
 * PCT priority lists (paper, section 4.1: every device runs, among its executable
 * vertices, the one with the highest PCT; PCT is computed once after partitioning and
 * the schedule is reused).  Per partition, the static priority list of every device:
 * its vertices by descending PCT = b, equal values by ascending vertex number.
 * order_out[j] lists the vertices of device 0, then of device 1, ...;
 * seg_out[j][d] .. seg_out[j][d+1] is device d's range.  Only enqueues work on `stream`.
 *
 *   assignments, assign_layout   as for cp_eval
 *   blevel      device ticks laid out per b_layout (CP_OUT_*): output of cp_eval for these assignments
 *   max_b       an upper bound on every b (for instance the largest CP of the batch); 0 = the
 *               graph's raw path bound.  A tighter bound means fewer sorting passes.  A b
 *               outside [0, max_b] sets CP_STATUS_B_OUT_OF_RANGE.
 *   workspace   device, 256-byte aligned, >= cp_pct_order_workspace_bytes (same batch, k, max_b)
 *   order_out   device int32 [batch][n]
 *   seg_out     device int32 [batch][k+1]
 *   status_out  device int32: CP_STATUS_* flags after the stream has drained
 * Errors: CP_ERR_NULL, CP_ERR_SIZE (also batch * ceil(n / 4096) >= 2^31), CP_ERR_ARG
 * (max_b < 0), CP_ERR_STATE, CP_ERR_OVERFLOW (device bits + bits of max_b > 64, or 32-bit
 * ticks asked for a graph that needs 64), CP_ERR_WORKSPACE, CP_ERR_HIP.
 */
int cp_pct_order_workspace_bytes(const cp_graph *g, int32_t batch, int32_t k, int64_t max_b,
                                 size_t *out_bytes);
int cp_pct_order(const cp_graph *g, int32_t batch, int32_t k,
                 const uint8_t *assignments, int assign_layout,
                 const void *blevel, int tick_dtype, int b_layout, int64_t max_b,
                 void *workspace, size_t workspace_bytes, void *stream,
                 int32_t *order_out, int32_t *seg_out, int32_t *status_out);

/*
 * Validity of `batch` partitions under the placement constraints of the problem
 * statement (paper, section 2, the collocation and the device constraint equations):
 * every collocation pair (v_i, v_j) must share a device, every device constraint
 * (v_i, d_j) must have p(v_i) = d_j.  Needs no graph.  Only enqueues work on `stream`.
 *
 *   n, k          vertices, devices
 *   assignments   device uint8, laid out per assign_layout (CP_ASSIGN_*)
 *   pairs         device int32 [num_pairs][2]; may be NULL when num_pairs = 0
 *   pins          device int32 [num_pins][2] = {vertex, device}; may be NULL when num_pins = 0
 *   valid_out     device uint8 [batch]: 1 if the partition meets every constraint
 *   violations_out  device int32 [batch] or NULL: constraints the partition breaks
 *   status_out    device int32: CP_STATUS_BAD_CONSTRAINT if an index is out of range
 * Errors: CP_ERR_NULL, CP_ERR_SIZE (n < 1, batch < 1, k < 1 or > 255, a negative count), CP_ERR_ARG, CP_ERR_HIP.
 */
int cp_validate(int32_t n, int32_t batch, int32_t k, const uint8_t *assignments, int assign_layout,
                int64_t num_pairs, const int32_t *pairs, int64_t num_pins, const int32_t *pins,
                void *stream, uint8_t *valid_out, int32_t *violations_out, int32_t *status_out);

/* ---- scheduling policies of cp_simulate ---- */
#define CP_POLICY_FIFO 0   /* the vertex that became executable first (paper, section 5.1) */
#define CP_POLICY_PCT  1   /* the vertex with the largest path computation time b (paper, section 4.1) */

/*
 * List-scheduling simulation of one iteration under each of `batch` partitions: the
 * execution time the paper's evaluation plots (section 5).  The scheduling criteria of
 * section 4 are read as follows, in the integer ticks of cp_eval:
 *   - a device runs its own vertices one at a time, without interruption, w(v) ticks each;
 *   - the tensor of an edge (u -> v) is at v's device x(u -> v) ticks after u finishes;
 *     transfers occupy no device and do not compete (section 2 models a rate per device
 *     pair and nothing else);
 *   - v is executable once all its input tensors are there (time 0 without inputs);
 *   - a free device that owns an executable vertex starts one at once, otherwise it waits
 *     for the first of its vertices to become executable;
 *   - CP_POLICY_FIFO takes the vertex that became executable first; among equals the paper
 *     draws at random, here the caller passes the draw: the smaller tie[v] wins;
 *     CP_POLICY_PCT takes the largest b(v), the smaller vertex number among equals.
 * Every vertex must cost at least one tick (c(v) >= 1 for all v, else CP_ERR_ARG): then
 * devices that decide at the same time cannot influence each other and the schedule is
 * unique.  All times must stay below 2^31: the summed execution times on the slowest device plus
 * the longest chain of transfers (bounded by the graph's raw path bound and by L - 1 transfers
 * at the lowest rate), which no makespan exceeds, else CP_ERR_OVERFLOW.
 * One wavefront simulates one partition, one lane per device: k <= 64.
 * Only enqueues work on `stream`.
 *
 *   assignments   device uint8, laid out per assign_layout (CP_ASSIGN_*)
 *   speeds, bandwidth  host, as for cp_eval
 *   policy        CP_POLICY_*
 *   blevel        CP_POLICY_PCT: device ticks as cp_eval wrote them for these assignments
 *                 (tick_dtype, b_layout = CP_OUT_*); values outside [0, 2^31) set
 *                 CP_STATUS_B_OUT_OF_RANGE.  Ignored (may be NULL) under CP_POLICY_FIFO.
 *   tie           CP_POLICY_FIFO: device int32 [n], a permutation of 0 .. n-1 (else
 *                 CP_STATUS_BAD_TIE and makespan -1), or NULL for tie[v] = v.  Ignored under PCT.
 *   workspace     device, 256-byte aligned, >= cp_simulate_workspace_bytes (28 bytes per
 *                 vertex and partition under PCT, 20 under FIFO, plus the cost tables)
 *   makespan_out  device int64 [batch]: the largest finish time; -1 for a partition with a
 *                 device id >= k (CP_STATUS_BAD_DEVICE_ID)
 *   start_out     device int32 [batch][n] (partition-major) or NULL: start time of every vertex
 *   status_out    device int32: CP_STATUS_* flags after the stream has drained
 * Errors: CP_ERR_NULL, CP_ERR_SIZE (k > 64), CP_ERR_ARG, CP_ERR_STATE, CP_ERR_SPEED,
 * CP_ERR_BANDWIDTH, CP_ERR_OVERFLOW, CP_ERR_WORKSPACE, CP_ERR_ALLOC, CP_ERR_HIP.
 */
int cp_simulate_workspace_bytes(const cp_graph *g, int32_t batch, int32_t k, int policy, int with_tie,
                                size_t *out_bytes);
int cp_simulate(const cp_graph *g, int32_t batch, int32_t k,
                const uint8_t *assignments, int assign_layout,
                const int64_t *speeds, const int64_t *bandwidth, int policy,
                const void *blevel, int tick_dtype, int b_layout, const int32_t *tie,
                void *workspace, size_t workspace_bytes, void *stream,
                int64_t *makespan_out, int32_t *start_out, int32_t *status_out);

/*
 * The paper's Critical Path partitioning strategy (section 3.2.2), e.g. as the start of
 * cp_search: the critical path of the ranks (vertex cost c, no devices, no transfers;
 * section 3.2's rank equations) goes to the fastest device (largest s, lowest number on
 * ties); every other vertex, in increasing vertex number, goes to the device d with the
 * smallest load(d) + ceil(c(v) / s[d]) (lowest number on ties), load(d) being the summed
 * execution times of the vertices already on d, the path included (the strategy's load
 * equation in integer ticks).  Memory capacities are not modelled.  The load rule is a
 * chain of n dependent choices: it runs on one wavefront, a few tenths of a microsecond per vertex.
 * Only enqueues work on `stream`.
 *
 *   k <= 64, speeds host int64 [k]
 *   workspace       device, 256-byte aligned, >= cp_seed_workspace_bytes
 *   assignment_out  device uint8 [n]
 *   status_out      device int32 (CP_STATUS_OK unless the inner evaluation reports otherwise)
 * Errors: CP_ERR_NULL, CP_ERR_SIZE (k < 1 or k > 64), CP_ERR_STATE, CP_ERR_WORKSPACE,
 * CP_ERR_SPEED, CP_ERR_HIP.
 */
int cp_seed_workspace_bytes(const cp_graph *g, size_t *out_bytes);
int cp_seed_partition(const cp_graph *g, int32_t k, const int64_t *speeds, void *workspace, size_t workspace_bytes,
                      void *stream, uint8_t *assignment_out, int32_t *status_out);

/*
 * Critical-path move search: a descent over partitions built from the paper's own
 * pieces.  Section 3.2 places the critical path first because it decides the running
 * time; here, from a start partition, every single move of a vertex of the current
 * critical path (cp_critical_path's path) to another device is a candidate; candidate
 * number i * (k-1) + r moves path vertex number i to the r-th device other than its own.
 * All candidates are evaluated with cp_eval in batches of `chunk`; those that break a
 * placement constraint (section 2, as in cp_validate) are left out; the candidate with
 * the smallest CP (lowest number on ties) is taken if it is smaller than the current CP,
 * and the step repeats; otherwise, or after max_moves moves, the search stops.
 * The call blocks: it waits on `stream` between steps.
 *
 *   assignment   device uint8 [n]: in the start partition, out the result
 *   pairs, pins  device, as for cp_validate (NULL with a count of 0)
 *   chunk        candidates per cp_eval call (>= 1); what cp_eval gains from a larger batch
 *                (partitions that share a workgroup's packet stream from 512 on) the search
 *                gains too: a million-vertex graph is searched twice as fast with 1,024
 *                candidates per call as with 256
 *   workspace    device, 256-byte aligned, >= cp_search_workspace_bytes(g, k, chunk)
 *   cp_trace     host int64 [max_moves + 1]: CP of the start, then after each move
 *   moves        host int32 [max_moves][2] = {vertex, new device}, or NULL
 *   num_moves    host: moves made
 *   evaluated    host: candidates evaluated, or NULL
 * Errors: CP_ERR_NULL, CP_ERR_SIZE, CP_ERR_STATE, CP_ERR_WORKSPACE, CP_ERR_ARG (a device id
 * >= k in the start), CP_ERR_SPEED, CP_ERR_BANDWIDTH, CP_ERR_HIP.
 */
int cp_search_workspace_bytes(const cp_graph *g, int32_t k, int32_t chunk, size_t *out_bytes);
int cp_search(const cp_graph *g, int32_t k, const int64_t *speeds, const int64_t *bandwidth,
              uint8_t *assignment, int64_t num_pairs, const int32_t *pairs, int64_t num_pins,
              const int32_t *pins, int32_t max_moves, int32_t chunk, void *workspace, size_t workspace_bytes,
              void *stream, int64_t *cp_trace, int32_t *moves, int32_t *num_moves, int64_t *evaluated);

/*
 * The device-free ranks of section 3.2: upRank (equation for the upward rank), downRank
 * (equation for the downward rank) and totalRank = upRank + downRank (section 3.2.1).
 * Both rank equations add the vertex's own c, so upRank is the b-level and downRank the
 * t-level plus c of the evaluation with a single device of speed 1, which is how they
 * are computed: one cp_eval with batch = 1, k = 1, then one elementwise kernel.
 * Only enqueues work on `stream`.
 *
 *   workspace   device, 256-byte aligned, >= cp_ranks_workspace_bytes
 *   up_out, down_out, total_out   device int64 [n] each; any may be NULL, not all
 * Errors: CP_ERR_NULL, CP_ERR_STATE (graph not uploaded), CP_ERR_WORKSPACE, CP_ERR_HIP.
 */
int cp_ranks_workspace_bytes(const cp_graph *g, size_t *out_bytes);
int cp_ranks(const cp_graph *g, void *workspace, size_t workspace_bytes, void *stream,
             int64_t *up_out, int64_t *down_out, int64_t *total_out);

/*
 * Stage timing with HIP events recorded on the stream the kernels run on.
 * A profile holds `slots` sets of CP_NUM_STAGES+1 events; every cp_eval call that
 * is given the profile fills the next slot (CP_ERR_STATE when full).
 */
int cp_profile_create(int32_t slots, cp_profile **out);
int cp_profile_reset(cp_profile *p);                       /* next call fills slot 0 again */
int cp_profile_count(const cp_profile *p, int32_t *out);   /* slots filled so far */
/* Milliseconds per stage for one filled slot; the stream must have drained.
 * sweep_launches[0], [1] (may be NULL) receive the number of kernel launches the
 * b-level and t-level stages made; {1, 0} for a call that asked for both sweeps means one
 * launch ran both (its time is the b-level stage's). */
int cp_profile_read(const cp_profile *p, int32_t slot, float ms_out[CP_NUM_STAGES],
                    int32_t sweep_launches[2]);
void cp_profile_destroy(cp_profile *p);

/*
 * Diagnostic: the 32-bit multiply-shift constants the kernels would use for
 * ceil(a / divisor) with 0 <= a <= max_dividend:
 *     ceil(a / divisor) == ((a + *dm1) * (uint64)*mul + (a + *dm1)) >> 32.
 * Returns 1 and fills mul, dm1 if that form is exact over the whole range, 0 if it
 * is not (the kernels then divide plainly), or a negative CP_ERR_* code.
 */
int cp_cost_magic(int64_t divisor, int64_t max_dividend, uint32_t *mul, uint32_t *dm1);

/*
 * Diagnostic: the 4-byte table entry some kernels use instead where every divisor of the
 * call is at most 256 and every weight below 2^24:
 *     ceil(a / divisor) == ((a + (e & 0xff)) * (uint64)(e | 0xff) + (a + (e & 0xff))) >> 32.
 * Returns 1 and fills *entry if that form is exact for 0 <= a <= max_dividend, 0 if not,
 * or a negative CP_ERR_* code.
 */
int cp_cost_compact(int64_t divisor, int64_t max_dividend, uint32_t *entry);

/*
 * Diagnostic: the workgroup shape the resident-window plan would launch with for one sweep
 * (tsweep = 0: b-levels, 1: t-levels) of this graph with k devices, on a compute unit with
 * 160 KB of LDS.  shape[0..7] = 16-byte loads per loader lane and tick, loader wavefronts, far
 * wavefronts, compute wavefronts, ticks of prefetch, partitions per workgroup, output stores one
 * compute wavefront issues per tick (1 or 2: the bound the far reads' ordering rests on), LDS
 * bytes per workgroup.  Host only.  Returns CP_OK, CP_ERR_NULL, CP_ERR_ARG (no such shape: the
 * plan does not apply to this graph, device count or tick type).
 */
int cp_window_shape(const cp_graph *g, int32_t k, int tick_dtype, int tsweep, int32_t shape[8]);

/* Human-readable text for a CP_ERR_* code (static storage). */
const char *cp_error_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* CPEVAL_H */
