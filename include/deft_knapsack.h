/*
 * deft_knapsack.h - C ABI of the batched exact 0/1 multiple-knapsack solver
 * for AMD MI355X (gfx950).
 *
 * The solver is the data-parallel core of DeFT's communication scheduler
 * (arXiv 2503.16815): gradient buckets are items weighted by communication
 * time, merged forward/backward computation windows are knapsacks, and many
 * candidate schedules (instances) are solved per call.
 *
 * All array arguments are DEVICE pointers owned by the caller (never retained,
 * never freed by the library).  All integers are int32 unless stated.  The
 * library never prints, throws or aborts: every failure is a return code or a
 * per-instance status.  A handle owns its scratch memory and serves one
 * in-flight batch at a time (not thread-safe; use one handle per stream).
 */
#ifndef DEFT_KNAPSACK_H
#define DEFT_KNAPSACK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct deft_knapsack deft_knapsack_t; /* opaque */

typedef enum {
    DEFT_OK = 0,
    DEFT_ERR_INVALID_ARG = 1, /* NULL pointer, negative count, bad mode, bad data          */
    DEFT_ERR_LIMIT = 2,       /* exceeds a limit given at create time                      */
    DEFT_ERR_OVERFLOW = 3,    /* sum of an instance's values >= 2^31                       */
    DEFT_ERR_OOM = 4,         /* scratch allocation failed                                 */
    DEFT_ERR_DEVICE = 5       /* HIP runtime error, wrong architecture, launch failure     */
} deft_status_t;

enum {
    DEFT_MODE_SEQUENTIAL = 0, /* m knapsacks filled one after the other (Sec. III.B)       */
    DEFT_MODE_JOINT2 = 1,     /* two links, one joint 2-D DP (Sec. III.C, Problem 2)       */
    DEFT_MODE_RECURSIVE = 2,  /* one window, the list shortened from its end (Algorithm 1) */
    DEFT_MODE_GREEDY = 3,     /* the paper's greedy heuristic, SEQUENTIAL layout (Sec. III.C)   */
    DEFT_MODE_GREEDY2 = 4,    /* the same on the JOINT2 layout (one time per link)              */
    DEFT_MODE_CAPACITY_SWEEP = 5 /* one item list at several capacities (Sec. IV.C feedback)    */
};

/* Limits fixed at create time; they size the scratch memory and select the
 * kernel variants.  A limit of 0 disables the corresponding mode.
 *
 * The sequential-mode kernel (lanes per instance, row cells per lane, LDS per
 * workgroup, workgroups per compute unit) is chosen ONCE, here, from max_capacity
 * (and max_items, whose lists must fit the row's LDS), not per call: the host
 * never reads the capacities of a batch, which live in device memory.  Every call
 * on the handle runs that kernel, whatever capacities it holds, so a handle
 * created for max_capacity 38911 solves capacity-900 instances on the
 * 1024-lane, one-workgroup-per-compute-unit kernel, several times slower than
 * a handle created for 1023 would.  Callers with mixed batches should keep one
 * handle per capacity class (<= 1023, 4095, 8191, 10239, 13311, 19967, 26623,
 * 38911 cells; longer rows live in global memory) and route instances by their
 * largest capacity.  deft_knapsack_get_info reports the choice. */
typedef struct {
    int32_t device;        /* HIP device ordinal                                           */
    int32_t max_batch;     /* instances per call                                           */
    int32_t max_items;     /* item_stride upper bound (1..4096)                            */
    int32_t max_knapsacks; /* knap_stride upper bound (1..64)                              */
    int32_t max_capacity;  /* sequential mode: largest capacity (0 = mode unused)          */
    int32_t max_c1;        /* joint mode: largest capacity of link 0 (0 = mode unused)     */
    int32_t max_c2;        /* joint mode: largest capacity of link 1                       */
    uint32_t flags;        /* 0, DEFT_FLAG_VALUES_ARE_WEIGHTS or DEFT_FLAG_SUBSET_SUM      */
} deft_knapsack_config_t;

/*
 * DEFT_FLAG_VALUES_ARE_WEIGHTS: the caller promises that in every instance given to this
 * handle each item's value equals its weight - the paper's own objective (Sec. III.B,
 * Problem 1: the profit of a bucket is its communication time).  Requires 1 <= max_capacity
 * <= 26623 (create returns DEFT_ERR_LIMIT otherwise, also when max_items is too long for the
 * smaller rows' LDS).  The sequential-layout modes (SEQUENTIAL, RECURSIVE, CAPACITY_SWEEP,
 * deft_knapsack_simulate_schedule) then run kernels that keep the DP row as 16-bit cells
 * (row[c] - c lies in [-c, 0]), two per 32-bit word: half the LDS per instance, half the LDS
 * instructions and packed 16-bit arithmetic per cell.  Results are bit-identical to those of a
 * handle without the flag.  An instance that breaks the promise (some value != its weight)
 * gets status DEFT_ERR_INVALID_ARG like any other bad input.  The joint and greedy modes are
 * not affected.
 */
#define DEFT_FLAG_VALUES_ARE_WEIGHTS 1u

/*
 * DEFT_FLAG_SUBSET_SUM: the same promise (every value equals its weight; an instance that
 * breaks it gets DEFT_ERR_INVALID_ARG), 1 <= max_capacity <= 65535.  DEFT_MODE_SEQUENTIAL,
 * DEFT_MODE_RECURSIVE and DEFT_MODE_CAPACITY_SWEEP calls (and with them
 * deft_knapsack_simulate_schedule) then run kernels that
 * treat a window as the subset-sum problem it is (Sec. III.B, Problem 1 with profit = time):
 * the DP row is the set of reachable sums, one bit per cell, an item is one shift-and-or
 * of the set (32 cells per instruction), and the canonical selection - the one the exact DP
 * walks back, smallest mask among the optima - is read off a per-cell record of the first
 * item that reached each sum.  One wavefront per instance, everything in LDS, no scratch
 * memory.  max_items decides the width of that record and with it how many instances share
 * a compute unit: 8-bit cells up to 255 items, 8-bit cells plus one snapshot of the set up
 * to 511, 16-bit cells beyond (create returns DEFT_ERR_LIMIT when set, record and item list
 * exceed a compute unit's LDS).  Algorithm 1's levels are read off the same set (a level's
 * answer is the largest reachable sum not above its remaining time, taken before the item
 * that ends the level is added), and so are the capacity sweep's answers (the final set at
 * the largest capacity, one walk per capacity).  Results are bit-identical to those of a
 * handle without flags.  Where the one more item list those two modes need does not fit
 * the LDS, they run as under DEFT_FLAG_VALUES_ARE_WEIGHTS when max_capacity <= 26623 and on
 * the 32-bit rows above that.  deft_knapsack_get_info reports seq_path 4.
 */
#define DEFT_FLAG_SUBSET_SUM 2u

/*
 * deft_knapsack_create: validate the limits, check that the device is a
 * gfx950, allocate the scratch (keep / choice tables, large rows) on
 * cfg->device and return a handle in *out.
 * Errors: INVALID_ARG (NULL, non-positive limits, unknown flag bits), LIMIT (limits
 * beyond what the library supports), OOM, DEVICE.  *out is NULL on error.
 */
deft_status_t deft_knapsack_create(const deft_knapsack_config_t *cfg, deft_knapsack_t **out);

/*
 * One call = `batch` independent instances.
 *
 * DEFT_MODE_SEQUENTIAL (Sec. III.B, Problem 1, one stage per knapsack):
 *   for s = 0 .. n_knapsacks-1:  j = fill_order[s]  (or s when fill_order is NULL)
 *     solve  max sum v_i x_i  s.t.  sum w_i x_i <= capacities[j],  x in {0,1}
 *     exactly, over the items not yet placed; place the chosen items in j.
 *   Each stage is the textbook exact DP ("NaiveKnapsack" of Algorithm 1); an
 *   item is taken at a capacity only when it strictly improves the value and
 *   the selection is traced back from the last item, so among optimal subsets
 *   the one with the smallest mask sum_t x_t 2^t (t = rank among the offered
 *   items) is returned.  The paper's value is the communication time itself
 *   (values == weights); separate values are accepted.
 *
 * DEFT_MODE_JOINT2 (Sec. III.C, Problem 2 with one weight per link):
 *   max sum_i v_i [a_i != none]  s.t.  sum_{a_i = 0} w0_i <= capacities[0],
 *   sum_{a_i = 1} w1_i <= capacities[1], each item on at most one link.
 *   Exact 2-D DP; per item the tests run skip, link 0, link 1, each replacing
 *   the incumbent only when strictly greater; traced back from the last item.
 *   n_knapsacks must be 2.
 *
 * DEFT_MODE_RECURSIVE (Sec. III.B, Algorithm 1, RecursiveKnapsack):
 *   Items are the list in generation order, capacities[b][0] is the remaining time R.
 *   Level d (d = 0 .. n) keeps the first n - d items and has R minus the drop_time of the
 *   d items left off; a level whose remaining time is negative schedules nothing.  Each
 *   level is solved exactly as a SEQUENTIAL stage (same tie rule); the answer is the
 *   level with the greatest value, and among equal levels the one with the most items
 *   left off (the recursion prefers the shorter list unless the longer one is strictly
 *   better).  All levels come out of one DP sweep: the row after item i is level
 *   n - 1 - i's row.  n_knapsacks must be 1 and knap_stride >= 2:
 *     knap_value[0], knap_load[0]  value and weight scheduled; total_value = knap_value[0]
 *     knap_value[1]                d of the level returned (n if nothing is scheduled)
 *     knap_load[1]                 that level's remaining time (0 if nothing is scheduled)
 *     assignment                   0 for scheduled items, else -1
 *   fill_order is ignored.  Served by every handle with max_capacity > 0 (with rows in
 *   global memory, seq_path 3, at one kernel launch per item).
 *
 * DEFT_MODE_CAPACITY_SWEEP (Sec. IV.C, the feedback mechanism: the Solver is called again
 * with a larger knapsack capacity, up to ten times):
 *   SEQUENTIAL layout, but capacities[b][0 .. n_knapsacks-1] are capacities of ONE knapsack,
 *   in any order; each is Problem 1 over the whole item list, solved exactly as a
 *   SEQUENTIAL stage (same tie rule).  One DP sweep at the largest capacity answers all of
 *   them: the value at capacity c is cell c of the final row and the selection is walked
 *   back from (last item, c).  n_knapsacks <= 31.
 *     knap_value[j], knap_load[j]  value and weight scheduled at capacities[b][j]
 *     assignment[i]                bit j set iff item i is scheduled at capacities[b][j]
 *                                  (0 = nowhere; also for slots >= n_items and faulted
 *                                  instances)
 *     total_value                  the value at the largest capacity
 *   fill_order is ignored.  Served by every handle with max_capacity > 0.
 *
 * DEFT_MODE_GREEDY / DEFT_MODE_GREEDY2 (Sec. III.C, the heuristic of the paper's Solver;
 * here so that the exact modes can be compared with it on the same inputs):
 *   knapsacks sorted by capacity, ascending (equal capacities: lower id first); items
 *   sorted by weight (the bucket's time), descending (equal weights: lower index first);
 *   each knapsack in that order goes through the items in that order and takes every
 *   item not placed yet that fits what is left of it.  Values only add up; they play no
 *   part in the order.  GREEDY takes the SEQUENTIAL layout (fill_order ignored), GREEDY2
 *   the JOINT2 layout (n_knapsacks must be 2; link j goes through the items in the order
 *   of its own weights).  Outputs as in SEQUENTIAL.  Served by any handle whose limits
 *   cover the layout (max_capacity > 0, or max_c1 / max_c2 > 0).
 *
 * Layout (row-major, device memory):
 *   n_items     [batch]                      0 <= n_items[b] <= item_stride
 *   n_knapsacks [batch]                      0 <= n_knapsacks[b] <= knap_stride
 *   weights     SEQUENTIAL, RECURSIVE, GREEDY, CAPACITY_SWEEP [batch][item_stride]   each >= 1
 *               JOINT2, GREEDY2 [batch][2][item_stride]   row 0 = link 0, row 1 = link 1
 *   values      [batch][item_stride]         each >= 0, sum per instance < 2^31
 *   capacities  [batch][knap_stride]         indexed by knapsack id, each >= 0
 *   fill_order  [batch][knap_stride] or NULL a permutation of 0..n_knapsacks[b]-1
 *   drop_time   RECURSIVE [batch][item_stride] each >= 0 (unused, may be NULL, otherwise)
 * Outputs (every slot of every row is written):
 *   total_value [batch] int64                sum of knap_value
 *   knap_value  [batch][knap_stride]         value placed in knapsack j (unused slots 0)
 *   knap_load   [batch][knap_stride]         weight placed in knapsack j (<= capacity)
 *   assignment  [batch][item_stride]         knapsack id, or -1 (also for slots >= n_items)
 *   status      [batch]                      deft_status_t of the instance
 * A faulted instance (status != DEFT_OK: bad n/m, w < 1, v < 0, capacity < 0,
 * fill_order not a permutation, drop_time < 0, RECURSIVE with n_knapsacks != 1,
 * CAPACITY_SWEEP with n_knapsacks > 31 -> INVALID_ARG; capacity above the create-time
 * limit -> LIMIT; value sum >= 2^31 -> OVERFLOW; in that precedence) gets
 * total_value 0, knap_value/knap_load 0 and assignment -1; other instances are
 * unaffected.
 */
typedef struct {
    int32_t mode;        /* DEFT_MODE_*                                                    */
    int32_t batch;       /* 0 .. max_batch (0 is a no-op)                                  */
    int32_t item_stride; /* 1 .. max_items                                                 */
    int32_t knap_stride; /* 1 .. max_knapsacks (>= 2 for JOINT2 and RECURSIVE)             */
    const int32_t *n_items;
    const int32_t *n_knapsacks;
    const int32_t *weights;
    const int32_t *values;
    const int32_t *capacities;
    const int32_t *fill_order; /* may be NULL */
    int64_t *total_value;
    int32_t *knap_value;
    int32_t *knap_load;
    int32_t *assignment;
    int32_t *status;
    void *stream; /* hipStream_t; NULL = the default stream */
    const int32_t *drop_time; /* RECURSIVE mode only */
} deft_knapsack_batch_t;

/*
 * deft_knapsack_solve_batch: enqueue the whole solve (all stages, traceback
 * included) on batch->stream and return without waiting; outputs are valid once
 * the stream has been synchronised.  Host-checkable faults (NULL handle / batch
 * / required array, batch < 0, strides < 1, bad mode) return INVALID_ARG, counts
 * above the create-time limits or a mode whose limit was 0 return LIMIT, a failed
 * launch returns DEVICE; in all these cases nothing was enqueued.
 * The call only launches kernels (no allocation, no memset, no host read of device data),
 * so with profiling off it may be recorded into a HIP graph and replayed.
 */
deft_status_t deft_knapsack_solve_batch(deft_knapsack_t *h, const deft_knapsack_batch_t *batch);

/*
 * The current and the future task queue of Sec. III.B (Cases 1-4), simulated for
 * `iterations` iterations over `batch` independent candidate schedules.  A candidate is
 * n_buckets communication times (in the order of Algorithm 1's list: the last bucket is
 * the first one the list loses), the time each bucket takes off the remaining time when
 * it is left off that list, and a forward and a backward window.  Every iteration has a
 * forward stage and then a backward stage, during which its buckets are generated:
 *   forward stage, current queue not empty (Case 1): Problem 1 over the current queue,
 *     capacity = forward window;
 *   backward stage, current queue not empty and longer than the backward window (Case 2):
 *     Problem 1 over it, capacity = backward window; the new buckets join the future queue
 *     (merged with what waits there);
 *   backward stage, current queue not empty and fitting (Case 3): all of it is
 *     synchronised first; the new buckets join the future queue; Algorithm 1 over the
 *     future queue with what is left of the window; what it leaves becomes the current
 *     queue;
 *   backward stage, current queue empty (Case 4): Algorithm 1 over the new buckets merged
 *     with the future queue, with the whole window; what it leaves becomes the current
 *     queue.
 * A queue that empties is complete; at the end of each iteration all complete gradients
 * are applied in one parameter update.  Each stage's problem is solved exactly as
 * DEFT_MODE_SEQUENTIAL / DEFT_MODE_RECURSIVE solve it (value = communication time).
 *
 * Inputs (device, int32):  comm_time [batch][n_buckets] >= 1 (sum per candidate < 2^31),
 *   drop_time [batch][n_buckets] >= 0, forward_time [batch], backward_time [batch]
 *   (0 .. max_capacity).
 * Outputs (device, int32, every slot written; s = 0 forward, 1 backward):
 *   stage_case  [batch][iterations][2]  0 = nothing to solve, else the case number
 *   stage_count [batch][iterations][2]  buckets synchronised in the stage
 *   stage_time  [batch][iterations][2]  their communication time (<= the window)
 *   update_k    [batch][iterations]     iterations of gradients applied at the end of
 *                                       iteration t (0 = no update)
 *   tail        [batch][2]              iterations still held by the current / the future
 *                                       queue after the last iteration
 *   status      [batch]                 INVALID_ARG (time < 1, drop time < 0, window < 0),
 *                                       LIMIT (window above max_capacity), OVERFLOW; such a
 *                                       candidate's other outputs are 0
 * The call enqueues everything on `stream` and returns; its first use on a handle
 * allocates the queue state (sized for max_batch x max_items; OOM if that fails).
 * Host-side errors: INVALID_ARG (NULL, batch < 0, n_buckets < 1, iterations < 1), LIMIT
 * (above the create-time limits, iterations > 4096, max_knapsacks < 2, max_capacity == 0),
 * DEVICE.
 */
typedef struct {
    int32_t batch;
    int32_t n_buckets;
    int32_t iterations;
    const int32_t *comm_time;
    const int32_t *drop_time;
    const int32_t *forward_time;
    const int32_t *backward_time;
    int32_t *stage_case;
    int32_t *stage_count;
    int32_t *stage_time;
    int32_t *update_k;
    int32_t *tail;
    int32_t *status;
    void *stream; /* hipStream_t; NULL = the default stream */
} deft_schedule_batch_t;

deft_status_t deft_knapsack_simulate_schedule(deft_knapsack_t *h, const deft_schedule_batch_t *s);

/*
 * deft_knapsack_solve_batch_static: DEFT_MODE_SEQUENTIAL for callers that cannot
 * allocate device memory: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No handle: what a handle would own (keep table,
 * offered-item lists) lives in one device array of DEFT_STATIC_SCRATCH_BYTES that is part
 * of the library image; every GPU the library runs on holds its own copy until the
 * process ends.  The call never calls hipMalloc / hipFree or any allocating routine; its
 * first use on a device looks up that device's copy of the array and, per kernel, sets
 * the kernel's dynamic-LDS attribute (neither allocates).  It runs the same kernels as
 * deft_knapsack_solve_batch with rows resident in LDS and returns the same outputs.
 *   device        HIP device ordinal (< 64) the arrays of `batch` live on
 *   max_capacity  1 .. 38911: upper bound of every capacity in the batch; it selects
 *                 the kernel exactly as deft_knapsack_config_t.max_capacity does, and an
 *                 instance with a larger capacity gets status DEFT_ERR_LIMIT
 *   batch         as for deft_knapsack_solve_batch; mode must be DEFT_MODE_SEQUENTIAL,
 *                 drop_time is ignored
 * Size limit: batch * item_stride * W + batch * knap_stride * ceil8(item_stride) * 16 bytes
 * must not exceed DEFT_STATIC_SCRATCH_BYTES, where W = 4 * lanes * ceil(cells / 32) of the
 * kernel chosen (256 bytes for max_capacity <= 1023, 1024 <= 4095 and <= 8191, 2048 <=
 * 10239 and <= 13311, 3072 <= 19967, 4096 <= 26623, 8192 <= 38911).  Larger calls, and
 * max_capacity above 38911, return DEFT_ERR_LIMIT with nothing enqueued.
 * Errors otherwise as deft_knapsack_solve_batch (INVALID_ARG also for another mode, a bad
 * device ordinal or max_capacity < 1; DEVICE when the device is not a gfx950).
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap in
 * time (different streams, or a captured graph replayed while another call runs) race.
 * Calls on one stream are ordered and safe; nothing in the array carries over from call
 * to call, and nothing in it needs clearing.
 */
#define DEFT_STATIC_SCRATCH_BYTES (64 * 1024 * 1024)
deft_status_t deft_knapsack_solve_batch_static(int32_t device, int32_t max_capacity,
                                               const deft_knapsack_batch_t *batch);

/* deft_knapsack_destroy: free the scratch and the handle.  NULL is a no-op. */
void deft_knapsack_destroy(deft_knapsack_t *h);

/* ---- introspection and measurement (not part of the paper's method) ------ */

typedef struct {
    int64_t scratch_bytes;     /* device memory owned by the handle                        */
    int32_t seq_path;          /* 0 none, 1 wavefront-per-instance LDS, 2 workgroup-per-
                                  instance LDS, 3 rows in global memory, 4 bit-set rows
                                  (DEFT_FLAG_SUBSET_SUM; what SEQUENTIAL, RECURSIVE and
                                  CAPACITY_SWEEP calls run on)                             */
    int32_t seq_threads;       /* threads cooperating on one instance                      */
    int32_t seq_cells_per_thread;
    int32_t seq_lds_bytes;     /* LDS per workgroup                                        */
    int32_t seq_workgroups_per_cu; /* co-resident workgroups reported by the runtime       */
    int32_t joint_path;        /* 0 none, 1 rows in global memory                          */
    int32_t compute_units;
} deft_knapsack_info_t;

/* Fill *info for a live handle.  INVALID_ARG on NULL. */
deft_status_t deft_knapsack_get_info(const deft_knapsack_t *h, deft_knapsack_info_t *info);

typedef struct {
    float total_ms;        /* summed duration of the profiled calls (first to last launch) */
    float sweep_ms;        /* summed duration of the DP sweep kernel launches              */
    int32_t sweep_launches;
    float other_ms;        /* total_ms - sweep_ms: set-up, traceback, launch gaps          */
    int64_t streamed_row_cells; /* sequential mode with rows in global memory, persistent
                              sweep: row cells read from plus row cells written to global
                              memory by the sweeps, summed over instances and stages (a
                              pass over a row may serve two items); 0 on the other paths   */
    int64_t swept_cell_updates; /* rows in LDS (seq_path 1 or 2): cell-updates the sweeps
                              evaluated, C - w + 1 for every item a stage's sweep went
                              through (stages settled without a sweep and the items after
                              a full row add nothing); 0 on the other paths               */
} deft_knapsack_profile_t;

/* Turn HIP-event timing of solve calls on (1) or off (0); off by default.
 * Events are recorded on each call's stream; nothing waits until they are read. */
deft_status_t deft_knapsack_set_profiling(deft_knapsack_t *h, int32_t enable);

/* Wait for the last profiled call to finish, return the sums over every call
 * made since profiling was enabled or last read, and start a new sum.
 * INVALID_ARG if profiling is off or no call has been made since. */
deft_status_t deft_knapsack_get_profile(deft_knapsack_t *h, deft_knapsack_profile_t *out);

/* What the device delivers, measured: for the benchmark's report of nominal and
 * measured peaks.  Allocates and frees 2 GiB of device memory, launches on the default
 * stream and waits; takes about a second. */
typedef struct {
    float lds_read_gbs;        /* conflict-free 4-byte LDS reads, every compute unit busy       */
    float lds_read_write_gbs;  /* the DP sweep's mix: one shifted 4-byte read and one 4-byte
                                  write (addressed by lane) per cell; bytes read + written      */
    float hbm_copy_gbs;        /* 1 GiB device-to-device copy kernel; bytes read + written      */
    float hbm_read_gbs;        /* 1 GiB read-only kernel                                        */
    float hbm_write_gbs;       /* 1 GiB fill kernel                                             */
    int32_t compute_units;
    int32_t clock_mhz_reported; /* the runtime's maximum shader clock                           */
} deft_knapsack_peaks_t;

/* INVALID_ARG (NULL, bad ordinal), DEVICE (not a gfx950, runtime failure), OOM. */
deft_status_t deft_knapsack_measure_peaks(int32_t device, deft_knapsack_peaks_t *out);

/* Static string for a status code ("DEFT_OK", ...); never NULL. */
const char *deft_knapsack_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* DEFT_KNAPSACK_H */
