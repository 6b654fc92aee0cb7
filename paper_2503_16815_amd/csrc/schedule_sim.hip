// The two task queues of Sec. III.B (Cases 1-4) simulated over several iterations for a
// batch of candidate schedules, entirely on the device: per stage a small kernel turns
// each candidate's queue state into one knapsack problem (the list, the window, and
// whether the stage is a plain knapsack or Algorithm 1), the solver runs on all candidates
// at once, and a second small kernel applies the answer to the queues and
// writes the stage's record.  Nothing is read back by the host between stages.
//
// Forward stages are plain knapsacks for every candidate and run in the sequential mode.
// In a backward stage some candidates pose a plain knapsack and others Algorithm 1; all go
// to the recursive mode, a plain knapsack as a list whose drop times exceed any window,
// so that only the whole list has a non-negative remaining time.
#include "kernels.h"

namespace deft {

namespace {

constexpr int kPlainDrop = 1 << 30;  // above every window (windows are <= 2^24)

enum StateWord { kStatus = 0, kCurK, kFutK, kDoneK, kKind, kFirstCount, kFirstTime, kListK, kStateWords };
enum StageKind { kNothing = 0, kPlain = 1, kAlgorithm1 = 2 };

struct SimBuffers {
    uint8_t *cur;        // [batch][n]  bucket in the current task queue?
    int32_t *state;      // [batch][kStateWords]
    int32_t *n_items, *n_knap, *w, *drop, *cap, *map;   // solver inputs ([batch], [batch][n], cap [batch][2])
    int64_t *total;
    int32_t *kv, *kl, *asg, *status;                    // solver outputs
};

__device__ __forceinline__ int wave_sum(int x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off);
    return __shfl(x, 0);
}
__device__ __forceinline__ long long wave_sum64(long long x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off);
    return __shfl(x, 0);
}

// One wavefront per candidate: input checks, empty queues, cleared records.
__global__ void __launch_bounds__(64) sim_init(ScheduleArgs s, SimBuffers buf)
{
    const int b = blockIdx.x, lane = threadIdx.x, n = s.n_buckets;
    const int32_t *comm = s.comm_time + (size_t)b * n, *drop = s.drop_time + (size_t)b * n;
    int bad = 0;
    long long sum = 0;
    for (int i = lane; i < n; i += 64) {
        const int c = comm[i];
        if (c < 1 || drop[i] < 0) bad = 1; else sum += c;
        buf.cur[(size_t)b * n + i] = 0;
    }
    bad = __ballot(bad != 0) != 0ull;
    sum = wave_sum64(sum);
    const int f = s.forward_time[b], w = s.backward_time[b];
    int status = DEFT_OK;
    if (bad || f < 0 || w < 0) status = DEFT_ERR_INVALID_ARG;
    else if (f > s.max_capacity || w > s.max_capacity) status = DEFT_ERR_LIMIT;
    else if (sum >= (1ll << 31)) status = DEFT_ERR_OVERFLOW;
    if (lane < kStateWords) buf.state[(size_t)b * kStateWords + lane] = lane == kStatus ? status : 0;
    for (int x = lane; x < 2 * s.iterations; x += 64) {
        s.stage_case[(size_t)b * 2 * s.iterations + x] = 0;
        s.stage_count[(size_t)b * 2 * s.iterations + x] = 0;
        s.stage_time[(size_t)b * 2 * s.iterations + x] = 0;
    }
    for (int t = lane; t < s.iterations; t += 64) s.update_k[(size_t)b * s.iterations + t] = 0;
    if (lane < 2) s.tail[(size_t)b * 2 + lane] = 0;
    if (lane == 0) {
        s.status[b] = status;
        buf.n_knap[b] = 1;
        buf.n_items[b] = 0;
        buf.cap[(size_t)b * 2] = 0;
        buf.cap[(size_t)b * 2 + 1] = 0;
    }
}

// Before a stage: which case applies, and the knapsack problem it poses.
__global__ void __launch_bounds__(64) sim_prep(ScheduleArgs s, SimBuffers buf, int stage)
{
    const int b = blockIdx.x, lane = threadIdx.x, n = s.n_buckets;
    int32_t *st = buf.state + (size_t)b * kStateWords;
    if (st[kStatus] != DEFT_OK) return;  // the empty problem written by sim_init stays
    const int32_t *comm = s.comm_time + (size_t)b * n, *drop = s.drop_time + (size_t)b * n;
    uint8_t *cur = buf.cur + (size_t)b * n;
    int32_t *lw = buf.w + (size_t)b * n, *ld = buf.drop + (size_t)b * n, *map = buf.map + (size_t)b * n;

    int in_cur = 0;
    long long cur_time = 0;
    for (int i = lane; i < n; i += 64)
        if (cur[i]) { ++in_cur; cur_time += comm[i]; }
    in_cur = wave_sum(in_cur);
    cur_time = wave_sum64(cur_time);
    const int window = stage == 0 ? s.forward_time[b] : s.backward_time[b];

    int kind = kNothing, items = 0, capacity = 0;
    if (in_cur > 0 && (stage == 0 || cur_time > window)) {
        // Case 1 / Case 2: plain knapsack over the current task queue, in bucket order
        kind = kPlain;
        capacity = window;
        for (int i0 = 0; i0 < n; i0 += 64) {
            const int i = i0 + lane;
            const bool in = i < n && cur[i];
            const unsigned long long m = __ballot(in);
            if (in) {
                const int pos = items + __popcll(m & ((1ull << lane) - 1ull));
                lw[pos] = comm[i];
                ld[pos] = kPlainDrop;
                map[pos] = i;
            }
            items += __popcll(m);
        }
    } else if (stage == 1) {
        // Case 3 (the current queue fits and goes first) / Case 4 (it is empty): Algorithm 1
        // over this iteration's buckets merged with the future queue, with what is left
        kind = kAlgorithm1;
        capacity = window - (int)cur_time;
        items = n;
        for (int i = lane; i < n; i += 64) {
            lw[i] = comm[i];
            ld[i] = drop[i];
            map[i] = i;
            cur[i] = 0;
        }
        if (lane == 0) {
            st[kFirstCount] = in_cur;
            st[kFirstTime] = (int)cur_time;
            if (in_cur > 0) st[kDoneK] += st[kCurK];
            st[kListK] = st[kFutK] + 1;
            st[kFutK] = 0;
        }
    }
    if (lane == 0) {
        st[kKind] = kind;
        buf.n_items[b] = items;
        buf.cap[(size_t)b * 2] = capacity;
    }
}

// After a stage: the answer applied to the queues, the stage's record, the update.
__global__ void __launch_bounds__(64) sim_post(ScheduleArgs s, SimBuffers buf, int t, int stage)
{
    const int b = blockIdx.x, lane = threadIdx.x, n = s.n_buckets;
    int32_t *st = buf.state + (size_t)b * kStateWords;
    if (st[kStatus] != DEFT_OK) return;
    if (buf.status[b] != DEFT_OK) {  // the solver refused the instance (never expected)
        if (lane == 0) { st[kStatus] = DEFT_ERR_DEVICE; s.status[b] = DEFT_ERR_DEVICE; }
        return;
    }
    uint8_t *cur = buf.cur + (size_t)b * n;
    const int32_t *asg = buf.asg + (size_t)b * n, *map = buf.map + (size_t)b * n;
    const int kind = st[kKind], items = buf.n_items[b];
    const size_t rec = ((size_t)b * s.iterations + t) * 2 + stage;

    int got = 0;
    if (kind == kPlain) {
        for (int p = lane; p < items; p += 64)
            if (asg[p] == 0) { cur[map[p]] = 0; ++got; }
    } else if (kind == kAlgorithm1) {
        for (int i = lane; i < n; i += 64) {
            const bool take = asg[i] == 0;
            cur[i] = take ? 0 : 1;  // what Algorithm 1 leaves is the new current queue
            got += take;
        }
    }
    got = wave_sum(got);
    if (lane == 0) {
        const int load = buf.kl[(size_t)b * 2];
        if (kind == kPlain) {
            s.stage_case[rec] = stage == 0 ? 1 : 2;
            s.stage_count[rec] = got;
            s.stage_time[rec] = load;
            if (stage == 1) st[kFutK] += 1;  // the new buckets wait in the future queue
            if (got == items) { st[kDoneK] += st[kCurK]; st[kCurK] = 0; }
        } else if (kind == kAlgorithm1) {
            s.stage_case[rec] = st[kFirstCount] > 0 ? 3 : 4;
            s.stage_count[rec] = st[kFirstCount] + got;
            s.stage_time[rec] = st[kFirstTime] + load;
            st[kCurK] = st[kListK];
            if (got == n) { st[kDoneK] += st[kCurK]; st[kCurK] = 0; }
        }
        if (stage == 1) {  // end of the iteration: everything complete is applied in one update
            s.update_k[(size_t)b * s.iterations + t] = st[kDoneK];
            st[kDoneK] = 0;
            if (t == s.iterations - 1) {
                s.tail[(size_t)b * 2] = st[kCurK];
                s.tail[(size_t)b * 2 + 1] = st[kFutK];
            }
        }
    }
}

SimBuffers carve(void *base, int64_t batch, int64_t n)
{
    // 64-bit totals first, then the int32 arrays, then the byte flags
    char *p = static_cast<char *>(base);
    SimBuffers b{};
    auto take = [&](int64_t bytes) { char *q = p; p += (bytes + 255) & ~(int64_t)255; return q; };
    b.total = reinterpret_cast<int64_t *>(take(batch * 8));
    b.state = reinterpret_cast<int32_t *>(take(batch * kStateWords * 4));
    b.n_items = reinterpret_cast<int32_t *>(take(batch * 4));
    b.n_knap = reinterpret_cast<int32_t *>(take(batch * 4));
    b.cap = reinterpret_cast<int32_t *>(take(batch * 2 * 4));
    b.kv = reinterpret_cast<int32_t *>(take(batch * 2 * 4));
    b.kl = reinterpret_cast<int32_t *>(take(batch * 2 * 4));
    b.status = reinterpret_cast<int32_t *>(take(batch * 4));
    b.w = reinterpret_cast<int32_t *>(take(batch * n * 4));
    b.drop = reinterpret_cast<int32_t *>(take(batch * n * 4));
    b.map = reinterpret_cast<int32_t *>(take(batch * n * 4));
    b.asg = reinterpret_cast<int32_t *>(take(batch * n * 4));
    b.cur = reinterpret_cast<uint8_t *>(take(batch * n));
    return b;
}

}  // namespace

int64_t schedule_sim_bytes(int32_t max_batch, int32_t max_items)
{
    const int64_t b = max_batch, n = max_items;
    return b * (8 + kStateWords * 4 + 4 + 4 + 8 + 8 + 8 + 4) + b * n * 17 + 13 * 256;
}

hipError_t schedule_sim_launch(const ScheduleArgs &s, void *sim_buffers, hipStream_t st,
                               const std::function<hipError_t(const BatchArgs &)> &solve)
{
    const SimBuffers buf = carve(sim_buffers, s.batch, s.n_buckets);
    BatchArgs a{};
    a.mode = DEFT_MODE_RECURSIVE;
    a.batch = s.batch;
    a.item_stride = s.n_buckets;
    a.knap_stride = 2;
    a.max_capacity = s.max_capacity;
    a.n_items = buf.n_items;
    a.n_knapsacks = buf.n_knap;
    a.weights = buf.w;
    a.values = buf.w;  // the value of a bucket is its communication time
    a.capacities = buf.cap;
    a.fill_order = nullptr;
    a.drop_time = buf.drop;
    a.total_value = buf.total;
    a.knap_value = buf.kv;
    a.knap_load = buf.kl;
    a.assignment = buf.asg;
    a.status = buf.status;

    const dim3 grid((unsigned)s.batch), block(64);
    hipLaunchKernelGGL(sim_init, grid, block, 0, st, s, buf);
    for (int t = 0; t < s.iterations; ++t) {
        for (int stage = 0; stage < 2; ++stage) {
            hipLaunchKernelGGL(sim_prep, grid, block, 0, st, s, buf, stage);
            // forward stages are plain knapsacks for every candidate (Case 1): the sequential
            // mode solves them, with its shortcuts; backward stages mix plain knapsacks and
            // Algorithm 1 and go to the recursive mode
            a.mode = stage == 0 ? DEFT_MODE_SEQUENTIAL : DEFT_MODE_RECURSIVE;
            const hipError_t e = solve(a);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(sim_post, grid, block, 0, st, s, buf, t, stage);
        }
    }
    return hipGetLastError();
}

}  // namespace deft
