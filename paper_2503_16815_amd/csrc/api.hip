// C ABI of the solver: argument validation, scratch ownership, kernel choice
// and launch sequencing.  See include/deft_knapsack.h for the contract.
#include <hip/hip_runtime.h>

#include <cstring>
#include <initializer_list>
#include <new>
#include <vector>

#include "kernels.h"

using namespace deft;

namespace {

constexpr int32_t kMaxItems = 4096;
constexpr int32_t kMaxKnapsacks = 64;
constexpr int32_t kMaxBatch = 1 << 20;
constexpr int32_t kMaxCapacity = 1 << 24;
constexpr int32_t kMaxJointCapacity = 4095;
constexpr int32_t kMaxIterations = 4096;
constexpr int32_t kMaxPacked16Capacity = 26623;  // the longest row of 16-bit cells that is compiled
constexpr int32_t kMaxSubsetSumCapacity = 65535;  // the longest bit-set row that is compiled

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard()
    {
        if (ok && prev >= 0) (void)hipSetDevice(prev);
    }
};

}  // namespace

struct deft_knapsack {
    deft_knapsack_config_t cfg{};
    int compute_units = 0;
    int64_t scratch_bytes = 0;

    int seq_path = 0;  // 0 none, 1 wave LDS, 2 workgroup LDS, 3 global rows
    SeqLdsPlan lds_plan{};
    void *keep = nullptr;  // LDS path: keep table, then the offered-item lists
    SeqGlobalPlan glob_plan{};
    void *glob_scratch = nullptr;
    unsigned long long *glob_streamed = nullptr;  // device counter read by get_profile
    unsigned long long *lds_swept = nullptr;      // device counter read by get_profile (LDS path)

    bool use_bits = false;        // SEQUENTIAL mode runs on the bit-set kernels (DEFT_FLAG_SUBSET_SUM)
    bool use_bits_rec = false;    // and so do RECURSIVE and CAPACITY_SWEEP
    SeqBitsPlan bits_plan{};

    void *sim_buffers = nullptr;  // task-queue simulation: allocated by its first call

    int joint_path = 0;
    JointPlan joint_plan{};
    void *joint_scratch = nullptr;

    bool profiling = false;
    Profiler prof;
};

namespace {

void free_handle(deft_knapsack *h)
{
    if (!h) return;
    DeviceGuard g(h->cfg.device);
    if (h->keep) (void)hipFree(h->keep);
    if (h->glob_scratch) (void)hipFree(h->glob_scratch);
    if (h->glob_streamed) (void)hipFree(h->glob_streamed);
    if (h->lds_swept) (void)hipFree(h->lds_swept);
    if (h->joint_scratch) (void)hipFree(h->joint_scratch);
    if (h->sim_buffers) (void)hipFree(h->sim_buffers);
    h->prof.destroy();
    delete h;
}

deft_status_t alloc(void **p, int64_t bytes, int64_t *total)
{
    *p = nullptr;
    if (bytes <= 0) return DEFT_OK;
    hipError_t e = hipMalloc(p, (size_t)bytes);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return DEFT_ERR_OOM;
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    *total += bytes;
    return DEFT_OK;
}

}  // namespace

extern "C" deft_status_t deft_knapsack_create(const deft_knapsack_config_t *cfg, deft_knapsack_t **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return DEFT_ERR_INVALID_ARG;
    if ((cfg->flags & ~(uint32_t)(DEFT_FLAG_VALUES_ARE_WEIGHTS | DEFT_FLAG_SUBSET_SUM)) != 0 || cfg->device < 0 || cfg->max_batch < 1 || cfg->max_items < 1 ||
        cfg->max_knapsacks < 1 || cfg->max_capacity < 0 || cfg->max_c1 < 0 || cfg->max_c2 < 0)
        return DEFT_ERR_INVALID_ARG;
    const bool want_seq = cfg->max_capacity > 0;
    const bool want_joint = cfg->max_c1 > 0 || cfg->max_c2 > 0;
    if (!want_seq && !want_joint) return DEFT_ERR_INVALID_ARG;
    if (cfg->max_items > kMaxItems || cfg->max_knapsacks > kMaxKnapsacks || cfg->max_batch > kMaxBatch ||
        cfg->max_capacity > kMaxCapacity || cfg->max_c1 > kMaxJointCapacity ||
        cfg->max_c2 > kMaxJointCapacity)
        return DEFT_ERR_LIMIT;
    if (want_joint && cfg->max_knapsacks < 2) return DEFT_ERR_INVALID_ARG;
    const bool subset_sum = (cfg->flags & DEFT_FLAG_SUBSET_SUM) != 0;
    if (subset_sum && (!want_seq || cfg->max_capacity > kMaxSubsetSumCapacity)) return DEFT_ERR_LIMIT;
    // what a subset-sum handle does not run on the bit-set kernels (the greedy mode; Algorithm 1
    // and the capacity sweep where their extra list does not fit the LDS) runs on rows of 16-bit
    // cells where those reach, on the 32-bit rows beyond
    const bool packed16 = (cfg->flags & DEFT_FLAG_VALUES_ARE_WEIGHTS) != 0 ||
                          (subset_sum && cfg->max_capacity <= kMaxPacked16Capacity);
    if ((cfg->flags & DEFT_FLAG_VALUES_ARE_WEIGHTS) != 0 && (!want_seq || cfg->max_capacity > kMaxPacked16Capacity))
        return DEFT_ERR_LIMIT;

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    if (cfg->device >= ndev) return DEFT_ERR_INVALID_ARG;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, cfg->device) != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return DEFT_ERR_DEVICE;

    DeviceGuard g(cfg->device);
    if (!g.ok) return DEFT_ERR_DEVICE;

    deft_knapsack *h = new (std::nothrow) deft_knapsack;
    if (!h) return DEFT_ERR_OOM;
    h->cfg = *cfg;
    h->compute_units = prop.multiProcessorCount;

    deft_status_t st = DEFT_OK;
    if (want_seq) {
        const int lds_wg = (int)prop.sharedMemPerBlockOptin > 0 ? (int)prop.sharedMemPerBlockOptin
                                                                : (int)prop.sharedMemPerBlock;
        if (seq_lds_plan(cfg->max_capacity, cfg->max_items, cfg->max_knapsacks, cfg->max_batch, lds_wg, packed16,
                         &h->lds_plan) &&
            seq_lds_prepare(&h->lds_plan) == hipSuccess && seq_lds_rec_prepare(h->lds_plan) == hipSuccess) {
            h->seq_path = h->lds_plan.threads == 64 ? 1 : 2;
            st = alloc(&h->keep, h->lds_plan.scratch_bytes, &h->scratch_bytes);
            if (st == DEFT_OK) {
                void *c = nullptr;
                st = alloc(&c, 8, &h->scratch_bytes);
                h->lds_swept = static_cast<unsigned long long *>(c);
                if (st == DEFT_OK && hipMemset(c, 0, 8) != hipSuccess) {
                    (void)hipGetLastError();
                    st = DEFT_ERR_DEVICE;
                }
            }
        } else if (packed16) {
            (void)hipGetLastError();
            st = DEFT_ERR_LIMIT;   // (an item list too long for the packed row's LDS)
        } else {
            (void)hipGetLastError();
            h->seq_path = 3;
            seq_global_plan(cfg->max_capacity, cfg->max_items, cfg->max_batch, lds_wg, h->compute_units,
                            &h->glob_plan);
            if (seq_global_prepare(h->glob_plan) != hipSuccess) {
                (void)hipGetLastError();
                st = DEFT_ERR_DEVICE;
            } else {
                st = alloc(&h->glob_scratch, h->glob_plan.scratch_bytes, &h->scratch_bytes);
                if (st == DEFT_OK) {
                    void *c = nullptr;
                    st = alloc(&c, 8, &h->scratch_bytes);
                    h->glob_streamed = static_cast<unsigned long long *>(c);
                    if (st == DEFT_OK && hipMemset(c, 0, 8) != hipSuccess) {
                        (void)hipGetLastError();
                        st = DEFT_ERR_DEVICE;
                    }
                }
            }
        }
    }
    if (st == DEFT_OK && subset_sum) {
        const int lds_wg = (int)prop.sharedMemPerBlockOptin > 0 ? (int)prop.sharedMemPerBlockOptin
                                                                : (int)prop.sharedMemPerBlock;
        if (!seq_bits_plan(cfg->max_capacity, cfg->max_items, lds_wg, &h->bits_plan)) {
            st = DEFT_ERR_LIMIT;  // (an item list too long for the LDS beside the row)
        } else if (seq_bits_prepare(h->bits_plan) != hipSuccess) {
            (void)hipGetLastError();
            st = DEFT_ERR_DEVICE;
        } else if (h->bits_plan.lds_bytes_rec > 0 && seq_bits_rec_prepare(h->bits_plan) != hipSuccess) {
            (void)hipGetLastError();
            st = DEFT_ERR_DEVICE;
        } else {
            h->use_bits = true;
            h->use_bits_rec = h->bits_plan.lds_bytes_rec > 0;
        }
    }
    if (st == DEFT_OK && want_joint) {
        h->joint_path = 1;
        const int lds_wg = (int)prop.sharedMemPerBlockOptin > 0 ? (int)prop.sharedMemPerBlockOptin
                                                                : (int)prop.sharedMemPerBlock;
        joint_plan(cfg->max_c1, cfg->max_c2, cfg->max_items, cfg->max_batch, lds_wg, &h->joint_plan);
        if (joint_prepare(h->joint_plan) != hipSuccess) {
            (void)hipGetLastError();
            st = DEFT_ERR_DEVICE;
        } else {
            st = alloc(&h->joint_scratch, h->joint_plan.scratch_bytes, &h->scratch_bytes);
        }
    }
    if (st == DEFT_OK && greedy_prepare(cfg->max_items) != hipSuccess) {
        (void)hipGetLastError();
        st = DEFT_ERR_DEVICE;
    }
    if (st != DEFT_OK) {
        free_handle(h);
        return st;
    }
    *out = h;
    return DEFT_OK;
}

extern "C" deft_status_t deft_knapsack_solve_batch(deft_knapsack_t *h, const deft_knapsack_batch_t *b)
{
    if (!h || !b) return DEFT_ERR_INVALID_ARG;
    if (b->mode < DEFT_MODE_SEQUENTIAL || b->mode > DEFT_MODE_CAPACITY_SWEEP) return DEFT_ERR_INVALID_ARG;
    if (b->batch < 0 || b->item_stride < 1 || b->knap_stride < 1) return DEFT_ERR_INVALID_ARG;
    const bool two_link = b->mode == DEFT_MODE_JOINT2 || b->mode == DEFT_MODE_GREEDY2;
    if ((two_link || b->mode == DEFT_MODE_RECURSIVE) && b->knap_stride < 2) return DEFT_ERR_INVALID_ARG;
    if (b->mode == DEFT_MODE_RECURSIVE && !b->drop_time) return DEFT_ERR_INVALID_ARG;
    if (!b->n_items || !b->n_knapsacks || !b->weights || !b->values || !b->capacities || !b->total_value ||
        !b->knap_value || !b->knap_load || !b->assignment || !b->status)
        return DEFT_ERR_INVALID_ARG;
    if (b->batch > h->cfg.max_batch || b->item_stride > h->cfg.max_items ||
        b->knap_stride > h->cfg.max_knapsacks)
        return DEFT_ERR_LIMIT;
    if (!two_link && h->seq_path == 0) return DEFT_ERR_LIMIT;
    if (two_link && h->joint_path == 0) return DEFT_ERR_LIMIT;
    // Algorithm 1 and the capacity sweep have kernels of their own on the LDS-resident row and
    // ride on the sequential mode's kernels when rows live in global memory
    const bool on_lds = h->seq_path == 1 || h->seq_path == 2;
    const bool probing = b->mode == DEFT_MODE_RECURSIVE || b->mode == DEFT_MODE_CAPACITY_SWEEP;
    if (b->batch == 0) return DEFT_OK;

    DeviceGuard g(h->cfg.device);
    if (!g.ok) return DEFT_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(b->stream);

    BatchArgs a;
    a.mode = b->mode;
    a.batch = b->batch;
    a.item_stride = b->item_stride;
    a.knap_stride = b->knap_stride;
    a.max_capacity = h->cfg.max_capacity;
    a.max_c1 = h->cfg.max_c1;
    a.max_c2 = h->cfg.max_c2;
    a.n_items = b->n_items;
    a.n_knapsacks = b->n_knapsacks;
    a.weights = b->weights;
    a.values = b->values;
    a.capacities = b->capacities;
    a.fill_order = b->mode == DEFT_MODE_SEQUENTIAL ? b->fill_order : nullptr;
    a.drop_time = b->mode == DEFT_MODE_RECURSIVE ? b->drop_time : nullptr;
    a.total_value = b->total_value;
    a.knap_value = b->knap_value;
    a.knap_load = b->knap_load;
    a.assignment = b->assignment;
    a.status = b->status;

    Profiler *prof = h->profiling ? &h->prof : nullptr;
    if (prof && !prof->begin(st)) return DEFT_ERR_DEVICE;

    hipError_t e = hipSuccess;
    if (b->mode == DEFT_MODE_SEQUENTIAL && h->use_bits) {
        if (prof) prof->sweep_begin(st);
        e = seq_bits_launch(h->bits_plan, a, st);
        if (prof) prof->sweep_end(st);
    } else if ((b->mode == DEFT_MODE_RECURSIVE || b->mode == DEFT_MODE_CAPACITY_SWEEP) && h->use_bits_rec) {
        if (prof) prof->sweep_begin(st);
        e = seq_bits_rec_launch(h->bits_plan, a, st);
        if (prof) prof->sweep_end(st);
    } else if (b->mode == DEFT_MODE_SEQUENTIAL || (probing && !on_lds)) {
        if (h->seq_path == 3) {
            e = seq_global_launch(h->glob_plan, a, h->glob_scratch, st, prof, h->glob_streamed);
        } else {
            if (prof) prof->sweep_begin(st);
            e = seq_lds_launch(h->lds_plan, a, h->keep, st, prof ? h->lds_swept : nullptr);
            if (prof) prof->sweep_end(st);
        }
    } else if (b->mode == DEFT_MODE_GREEDY || b->mode == DEFT_MODE_GREEDY2) {
        if (prof) prof->sweep_begin(st);
        e = greedy_launch(a, two_link, st);
        if (prof) prof->sweep_end(st);
    } else if (probing) {  // on the LDS-resident row
        if (prof) prof->sweep_begin(st);
        e = seq_lds_rec_launch(h->lds_plan, a, h->keep, st, prof ? h->lds_swept : nullptr);
        if (prof) prof->sweep_end(st);
    } else {
        e = joint_launch(h->joint_plan, a, h->joint_scratch, st, prof);
    }
    if (prof) prof->end(st);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    return DEFT_OK;
}

extern "C" deft_status_t deft_knapsack_simulate_schedule(deft_knapsack_t *h, const deft_schedule_batch_t *s)
{
    if (!h || !s) return DEFT_ERR_INVALID_ARG;
    if (s->batch < 0 || s->n_buckets < 1 || s->iterations < 1) return DEFT_ERR_INVALID_ARG;
    if (!s->comm_time || !s->drop_time || !s->forward_time || !s->backward_time || !s->stage_case ||
        !s->stage_count || !s->stage_time || !s->update_k || !s->tail || !s->status)
        return DEFT_ERR_INVALID_ARG;
    if (s->batch > h->cfg.max_batch || s->n_buckets > h->cfg.max_items || s->iterations > kMaxIterations ||
        h->cfg.max_knapsacks < 2)
        return DEFT_ERR_LIMIT;
    if (h->seq_path == 0) return DEFT_ERR_LIMIT;
    if (s->batch == 0) return DEFT_OK;

    DeviceGuard g(h->cfg.device);
    if (!g.ok) return DEFT_ERR_DEVICE;
    if (!h->sim_buffers) {
        const deft_status_t rc = alloc(&h->sim_buffers, schedule_sim_bytes(h->cfg.max_batch, h->cfg.max_items),
                                       &h->scratch_bytes);
        if (rc != DEFT_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(s->stream);
    ScheduleArgs a;
    a.batch = s->batch;
    a.n_buckets = s->n_buckets;
    a.iterations = s->iterations;
    a.max_capacity = h->cfg.max_capacity;
    a.comm_time = s->comm_time;
    a.drop_time = s->drop_time;
    a.forward_time = s->forward_time;
    a.backward_time = s->backward_time;
    a.stage_case = s->stage_case;
    a.stage_count = s->stage_count;
    a.stage_time = s->stage_time;
    a.update_k = s->update_k;
    a.tail = s->tail;
    a.status = s->status;

    Profiler *prof = h->profiling ? &h->prof : nullptr;
    if (prof && !prof->begin(st)) return DEFT_ERR_DEVICE;
    const auto solve = [&](const BatchArgs &x) -> hipError_t {
        if ((h->use_bits && x.mode == DEFT_MODE_SEQUENTIAL) || (h->use_bits_rec && x.mode == DEFT_MODE_RECURSIVE)) {
            if (prof) prof->sweep_begin(st);
            const hipError_t rc = x.mode == DEFT_MODE_SEQUENTIAL ? seq_bits_launch(h->bits_plan, x, st)
                                                                 : seq_bits_rec_launch(h->bits_plan, x, st);
            if (prof) prof->sweep_end(st);
            return rc;
        }
        if (h->seq_path == 3) return seq_global_launch(h->glob_plan, x, h->glob_scratch, st, prof, h->glob_streamed);
        if (prof) prof->sweep_begin(st);
        const hipError_t rc = x.mode == DEFT_MODE_SEQUENTIAL
                                  ? seq_lds_launch(h->lds_plan, x, h->keep, st, prof ? h->lds_swept : nullptr)
                                  : seq_lds_rec_launch(h->lds_plan, x, h->keep, st, prof ? h->lds_swept : nullptr);
        if (prof) prof->sweep_end(st);
        return rc;
    };
    const hipError_t e = schedule_sim_launch(a, h->sim_buffers, st, solve);
    if (prof) prof->end(st);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    return DEFT_OK;
}

extern "C" void deft_knapsack_destroy(deft_knapsack_t *h) { free_handle(h); }

extern "C" deft_status_t deft_knapsack_get_info(const deft_knapsack_t *h, deft_knapsack_info_t *info)
{
    if (!h || !info) return DEFT_ERR_INVALID_ARG;
    std::memset(info, 0, sizeof(*info));
    info->scratch_bytes = h->scratch_bytes;
    info->seq_path = h->seq_path;
    if (h->seq_path == 1 || h->seq_path == 2) {
        info->seq_threads = h->lds_plan.threads;
        info->seq_cells_per_thread = h->lds_plan.cells_per_thread;
        info->seq_lds_bytes = h->lds_plan.lds_bytes;
        info->seq_workgroups_per_cu = h->lds_plan.wg_per_cu;
    } else if (h->seq_path == 3) {
        info->seq_threads = h->glob_plan.threads;
        info->seq_cells_per_thread = h->glob_plan.cells_per_thread;
    }
    if (h->use_bits) {  // what SEQUENTIAL calls run on
        info->seq_path = 4;
        info->seq_threads = 64;
        info->seq_cells_per_thread = h->bits_plan.words_per_lane * 32;
        info->seq_lds_bytes = h->bits_plan.lds_bytes;
        info->seq_workgroups_per_cu = 0;
    }
    info->joint_path = h->joint_path;
    info->compute_units = h->compute_units;
    return DEFT_OK;
}

extern "C" deft_status_t deft_knapsack_set_profiling(deft_knapsack_t *h, int32_t enable)
{
    if (!h) return DEFT_ERR_INVALID_ARG;
    h->profiling = enable != 0;
    h->prof.reset();
    for (unsigned long long *counter : {h->glob_streamed, h->lds_swept}) {
        if (!counter) continue;
        DeviceGuard g(h->cfg.device);
        if (!g.ok || hipMemset(counter, 0, 8) != hipSuccess) {
            (void)hipGetLastError();
            return DEFT_ERR_DEVICE;
        }
    }
    return DEFT_OK;
}

extern "C" deft_status_t deft_knapsack_get_profile(deft_knapsack_t *h, deft_knapsack_profile_t *out)
{
    if (!h || !out || !h->profiling) return DEFT_ERR_INVALID_ARG;
    DeviceGuard g(h->cfg.device);
    if (!g.ok) return DEFT_ERR_DEVICE;
    deft_status_t rc = h->prof.read(out);   // waits for the last profiled call
    out->streamed_row_cells = 0;
    out->swept_cell_updates = 0;
    if (rc != DEFT_OK) return rc;
    for (int which = 0; which < 2; ++which) {
        unsigned long long *counter = which == 0 ? h->glob_streamed : h->lds_swept;
        if (!counter) continue;
        unsigned long long v = 0;
        if (hipMemcpy(&v, counter, 8, hipMemcpyDeviceToHost) != hipSuccess || hipMemset(counter, 0, 8) != hipSuccess) {
            (void)hipGetLastError();
            return DEFT_ERR_DEVICE;
        }
        (which == 0 ? out->streamed_row_cells : out->swept_cell_updates) = (int64_t)v;
    }
    return rc;
}

extern "C" const char *deft_knapsack_status_string(int32_t s)
{
    switch (s) {
    case DEFT_OK: return "DEFT_OK";
    case DEFT_ERR_INVALID_ARG: return "DEFT_ERR_INVALID_ARG";
    case DEFT_ERR_LIMIT: return "DEFT_ERR_LIMIT";
    case DEFT_ERR_OVERFLOW: return "DEFT_ERR_OVERFLOW";
    case DEFT_ERR_OOM: return "DEFT_ERR_OOM";
    case DEFT_ERR_DEVICE: return "DEFT_ERR_DEVICE";
    default: return "DEFT_ERR_UNKNOWN";
    }
}
