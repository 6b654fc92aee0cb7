// Internal interface between the C ABI (api.hip) and the kernel files.
// Nothing here is visible to users of include/deft_knapsack.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <functional>

#include "../../include/deft_knapsack.h"

namespace deft {

// Arguments of one solve call as the kernels see them (all device pointers).
struct BatchArgs {
    int32_t mode;  // DEFT_MODE_*
    int32_t batch, item_stride, knap_stride;
    int32_t max_capacity, max_c1, max_c2;  // create-time limits (per-instance LIMIT status)
    const int32_t *n_items, *n_knapsacks, *weights, *values, *capacities, *fill_order;
    const int32_t *drop_time;  // recursive mode only
    int64_t *total_value;
    int32_t *knap_value, *knap_load, *assignment, *status;
};

// ---- sequential mode, capacity row resident in LDS (seq_lds.hip) ------------
// One instance is owned by `threads` lanes (64 = one wavefront, several
// instances per workgroup; otherwise one workgroup).  Each lane keeps
// `cells_per_thread` row cells in registers.
struct SeqLdsPlan {
    int32_t packed16;          // 1: rows of 16-bit cells (values equal weights, capacities <= 26623)
    int32_t variant;           // index into the compiled (threads, cells_per_thread) table
    int32_t threads;           // T
    int32_t cells_per_thread;  // K
    int32_t keep_words;        // 32-bit keep words per lane and item: ceil(K / 32)
    int32_t guard_cells;       // cells below the row: 8 scratch words, then INT_MIN
    int32_t row_cells;         // LDS row length (multiple of 64, covers max_capacity)
    int32_t n_pad;             // entries per offered-item list (multiple of 8, >= max_items)
    int32_t lds_bytes;         // dynamic LDS per workgroup
    int32_t wg_threads;        // workgroup size
    int32_t inst_per_wg;       // instances per workgroup
    int32_t wg_per_cu;         // co-resident workgroups: the runtime's answer, capped by LDS granules
    int64_t keep_words_per_inst;  // max_items * keep_words * T
    int64_t keep_bytes;        // keep table of the whole batch
    int64_t scratch_bytes;     // keep table + one offered-item list per instance and stage
};

// Picks the variant for the limits; returns false when no LDS variant fits.
// packed16: the kernels with rows of 16-bit cells (every value equals its weight).
bool seq_lds_plan(int32_t max_capacity, int32_t max_items, int32_t max_knapsacks, int32_t max_batch,
                  int32_t lds_per_wg_bytes, bool packed16, SeqLdsPlan *plan);
// Sets the kernel's dynamic-LDS attribute and queries occupancy.
hipError_t seq_lds_prepare(SeqLdsPlan *plan);
// `swept_cells` (device, may be null): every stage adds the cell-updates its sweep evaluated.
hipError_t seq_lds_launch(const SeqLdsPlan &plan, const BatchArgs &args, void *scratch,
                          hipStream_t stream, unsigned long long *swept_cells);
// The kernels with rows of 16-bit cells (seq_lds_p16.hip, seq_lds_p16_rec.hip); the launchers
// above forward to them when the plan says packed16.
hipError_t seq_lds_p16_prepare(const SeqLdsPlan &plan, int *wg_per_cu);
hipError_t seq_lds_p16_launch(const SeqLdsPlan &plan, const BatchArgs &args, void *scratch,
                              hipStream_t stream, unsigned long long *swept_cells);
hipError_t seq_lds_p16_rec_prepare(const SeqLdsPlan &plan);
hipError_t seq_lds_p16_rec_launch(const SeqLdsPlan &plan, const BatchArgs &args, void *scratch,
                                  hipStream_t stream, unsigned long long *swept_cells);
// Algorithm 1 (recursive mode) under the same plan and scratch (seq_lds_rec.hip).
hipError_t seq_lds_rec_prepare(const SeqLdsPlan &plan);
hipError_t seq_lds_rec_launch(const SeqLdsPlan &plan, const BatchArgs &args, void *scratch,
                              hipStream_t stream, unsigned long long *swept_cells);

// ---- sequential layout, value = weight, one bit per cell (seq_bits_kernel.h) -----
// One wavefront per instance; the reachable sums as a bit set in registers and LDS, the
// selection from a per-cell "first item that reached this sum" array in LDS.  No scratch.
struct SeqBitsPlan {
    int32_t variant;         // index into the compiled words-per-lane table
    int32_t words_per_lane;  // K: capacities up to 2048 K - 1
    int32_t row_words;       // 64 K
    int32_t first_ints;      // LDS ints of the per-cell array (8-bit cells for at most 255 items, else 16-bit)
    int32_t n_pad;           // entries of the stage's item list in LDS
    int32_t lds_bytes;       // dynamic LDS per workgroup (= per instance)
    int32_t lds_bytes_rec;   // the same for the Algorithm 1 kernels (0: they do not fit)
};
bool seq_bits_plan(int32_t max_capacity, int32_t max_items, int32_t lds_per_wg_bytes, SeqBitsPlan *plan);
hipError_t seq_bits_prepare(const SeqBitsPlan &plan);
hipError_t seq_bits_launch(const SeqBitsPlan &plan, const BatchArgs &args, hipStream_t stream);
hipError_t seq_bits_rec_prepare(const SeqBitsPlan &plan);  // DEFT_MODE_RECURSIVE (seq_bits_rec.hip)
hipError_t seq_bits_rec_launch(const SeqBitsPlan &plan, const BatchArgs &args, hipStream_t stream);

// ---- per-call HIP-event timing (profile.hip) ---------------------------------
class Profiler {
public:
    void reset() { ncall_ = nsweep_ = 0; failed_ = false; }
    bool begin(hipStream_t st);        // start of a profiled call
    void sweep_begin(hipStream_t st);  // brackets one launch of the DP sweep kernel
    void sweep_end(hipStream_t st);
    void end(hipStream_t st);
    // waits for the last recorded call, sums every call since reset(), resets
    deft_status_t read(deft_knapsack_profile_t *out);
    void destroy();

private:
    struct Pool {
        hipEvent_t *ev = nullptr;
        int cap = 0;
        hipEvent_t get(int i);  // event i, created on demand; nullptr on failure
        void destroy();
    };
    void record(Pool &p, int idx, hipStream_t st);
    Pool call_, sweep_;
    int ncall_ = 0, nsweep_ = 0;  // events used (two per call / per launch)
    bool failed_ = false;
};

// ---- sequential mode, rows in global memory (seq_global.hip) -------------------
// For capacities whose row does not fit LDS.  One launch per offered item: the
// row ping-pongs between two global buffers, keep bits go out as 64-bit words.
struct SeqGlobalPlan {
    int32_t threads, cells_per_thread;
    int32_t row_len;           // int32 cells per row buffer (multiple of the tile)
    int32_t keep_words;        // 64-bit keep words per item
    int32_t max_items, max_batch;
    int32_t ring_segs;         // persistent sweep: 256-cell segments of the old row resident in LDS
    int32_t lds_bytes;         // its dynamic LDS
    int32_t persistent_min_batch;  // batches at least this large take the persistent sweep
    int64_t scratch_bytes;     // rows + keep + offered-item lists + per-instance state
};
void seq_global_plan(int32_t max_capacity, int32_t max_items, int32_t max_batch, int32_t lds_per_wg_bytes,
                     int32_t compute_units, SeqGlobalPlan *plan);
hipError_t seq_global_prepare(const SeqGlobalPlan &plan);
// `streamed_cells` (device, may be null): the persistent sweep adds the row cells it fetched.
hipError_t seq_global_launch(const SeqGlobalPlan &plan, const BatchArgs &args, void *scratch,
                             hipStream_t stream, Profiler *prof, unsigned long long *streamed_cells);

// ---- joint two-link mode, table in global memory (joint2.hip) -----------------
struct JointPlan {
    int32_t pitch;             // int32 cells per table row (multiple of 64)
    int32_t rows;              // max_c1 + 1
    int32_t lds_pitch;         // int32 cells per LDS row: max_c2 + 1
    int32_t ring_rows;         // old rows resident in LDS
    int32_t lds_bytes;         // dynamic LDS of the sweep kernel
    int32_t max_items, max_batch;
    int64_t scratch_bytes;
};
void joint_plan(int32_t max_c1, int32_t max_c2, int32_t max_items, int32_t max_batch, int32_t lds_per_wg_bytes,
                JointPlan *plan);
hipError_t joint_prepare(const JointPlan &plan);
hipError_t joint_launch(const JointPlan &plan, const BatchArgs &args, void *scratch, hipStream_t stream,
                        Profiler *prof);

// ---- the two task queues over several iterations (schedule_sim.hip) -------------
// Arguments of one simulation call as the kernels see them (all device pointers).
struct ScheduleArgs {
    int32_t batch, n_buckets, iterations, max_capacity;
    const int32_t *comm_time, *drop_time, *forward_time, *backward_time;
    int32_t *stage_case, *stage_count, *stage_time, *update_k, *tail, *status;
};
// Bytes of the handle-owned buffers (queue state and the per-stage solver problem).
int64_t schedule_sim_bytes(int32_t max_batch, int32_t max_items);
// Enqueues the whole simulation: per stage a set-up kernel, the solver (`solve` enqueues one
// batch in args.mode = DEFT_MODE_SEQUENTIAL or DEFT_MODE_RECURSIVE on the handle's path), a
// kernel that applies the answer.
hipError_t schedule_sim_launch(const ScheduleArgs &args, void *sim_buffers, hipStream_t stream,
                               const std::function<hipError_t(const BatchArgs &)> &solve);

// ---- the paper's greedy heuristic (greedy.hip) ----------------------------------
// No scratch memory.  per_link: the two-link weight layout.
hipError_t greedy_prepare(int32_t max_items);
hipError_t greedy_launch(const BatchArgs &args, bool per_link, hipStream_t stream);

}  // namespace deft
