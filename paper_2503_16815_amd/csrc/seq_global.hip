// Sequential multiple-knapsack solve for capacities whose row does not fit LDS
// (Sec. III.B, Problem 1 per window).  The row lives in global memory in two
// buffers; offered item q reads buffer q & 1 and writes the other:
//   new[c] = max(old[c], old[c - w] + v)   for c >= w,   new[c] = old[c] below,
// with the take bit (old[c - w] + v > old[c]) collected per 64 cells by a
// wavefront ballot and stored as one 64-bit keep word.  The first offered item
// of a stage reads zeros instead of a buffer.  One launch per offered-item
// rank (the host cannot know how many items each instance still offers, so it
// launches item_stride of them; a workgroup whose instance has fewer exits).
// Traffic per cell: 4 B read + 4 B write + 1/8 B keep (the shifted read hits
// cache lines another wavefront has just fetched).
#include "instance_check.h"

namespace deft {

namespace {

constexpr int kThreads = 256;
constexpr int kIter = 32;                       // 64-cell groups per wavefront
constexpr int kWaveCells = 64 * kIter;          // 2048
constexpr int kTileCells = kWaveCells * (kThreads / 64);

// per-instance state kept between launches
struct InstState {
    int32_t status, n_act, knap, cap;
    int64_t total;
};

struct Scratch {
    int32_t *rows;      // [batch][2][row_len]
    uint64_t *keep;     // [batch][max_items][keep_words]
    int32_t *act;       // [batch][max_items]
    InstState *state;   // [batch]
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

Scratch carve(const SeqGlobalPlan &p, void *base, int32_t max_batch)
{
    char *c = static_cast<char *>(base);
    Scratch s;
    s.rows = reinterpret_cast<int32_t *>(c);
    c += align256((size_t)max_batch * 2 * p.row_len * 4);
    s.keep = reinterpret_cast<uint64_t *>(c);
    c += align256((size_t)max_batch * p.max_items * p.keep_words * 8);
    s.act = reinterpret_cast<int32_t *>(c);
    c += align256((size_t)max_batch * p.max_items * 4);
    s.state = reinterpret_cast<InstState *>(c);
    return s;
}

__global__ void __launch_bounds__(kThreads) sg_init(BatchArgs a, InstState *state)
{
    const int inst = blockIdx.x;
    const int status = check_instance(a, inst, false);
    clear_outputs(a, inst, status);
    if (threadIdx.x == 0) {
        state[inst].status = status;
        state[inst].n_act = 0;
        state[inst].total = 0;
    }
}

// Stage s: knapsack id, capacity and the ascending list of offered items
// (not yet placed, weight <= capacity).
__global__ void __launch_bounds__(64) sg_stage_setup(BatchArgs a, int s, InstState *state, int32_t *act,
                                                     int max_items)
{
    const int inst = blockIdx.x, lane = threadIdx.x;
    InstState *st = &state[inst];
    const int m = a.n_knapsacks[inst];
    if (st->status != DEFT_OK || s >= m) {
        if (lane == 0) st->n_act = 0, st->knap = -1;
        return;
    }
    const int n = a.n_items[inst];
    const int j = a.fill_order ? a.fill_order[(size_t)inst * a.knap_stride + s] : s;
    const int C = a.capacities[(size_t)inst * a.knap_stride + j];
    const int32_t *W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *asg = a.assignment + (size_t)inst * a.item_stride;
    int32_t *list = act + (size_t)inst * max_items;
    int cnt = 0;
    for (int i0 = 0; i0 < n; i0 += 64) {
        const int i = i0 + lane;
        const bool f = i < n && asg[i] < 0 && W[i] <= C;
        const unsigned long long mask = __ballot(f);
        if (f) list[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = i;
        cnt += __popcll(mask);
    }
    if (lane == 0) { st->n_act = cnt; st->knap = j; st->cap = C; }
}

// Offered item q of every instance: one pass over the row.
__global__ void __launch_bounds__(kThreads)
sg_sweep(BatchArgs a, int q, const InstState *__restrict__ state, const int32_t *__restrict__ act,
         int32_t *rows, uint64_t *keep, int row_len, int keep_words, int max_items, int tiles)
{
    const int inst = blockIdx.x / tiles, tile = blockIdx.x % tiles;
    const InstState st = state[inst];
    if (q >= st.n_act) return;
    const int C = st.cap;
    const int lane = threadIdx.x & 63;
    const int wave_base = (tile * (kThreads / 64) + (threadIdx.x >> 6)) * kWaveCells;
    if (wave_base > C) return;
    const int t = act[(size_t)inst * max_items + q];
    const int w = a.weights[(size_t)inst * a.item_stride + t];
    const int v = a.values[(size_t)inst * a.item_stride + t];
    const int32_t *__restrict__ src = rows + ((size_t)inst * 2 + (q & 1)) * row_len;
    int32_t *__restrict__ dst = rows + ((size_t)inst * 2 + ((q & 1) ^ 1)) * row_len;
    uint64_t *kw = keep + ((size_t)inst * max_items + t) * keep_words + wave_base / 64;
    const bool first = q == 0;

    unsigned long long mine = 0;
#pragma unroll 8
    for (int i = 0; i < kIter; ++i) {
        const int c = wave_base + i * 64 + lane;
        const int own = first ? 0 : src[c];
        int cand = INT_MIN;
        if (c >= w) cand = (first ? 0 : src[c - w]) + v;
        const bool take = cand > own;
        dst[c] = take ? cand : own;
        const unsigned long long mask = __ballot(take);
        if (lane == i) mine = mask;
    }
    if (lane < kIter) kw[lane] = mine;
}

// One thread per instance walks the keep words back from (last offered item, C).
__global__ void __launch_bounds__(64)
sg_traceback(BatchArgs a, InstState *state, const int32_t *__restrict__ act, const int32_t *rows,
             const uint64_t *keep, int row_len, int keep_words, int max_items)
{
    const int inst = blockIdx.x * 64 + threadIdx.x;
    if (inst >= a.batch) return;
    InstState *st = &state[inst];
    if (st->status != DEFT_OK || st->knap < 0) return;
    const int nact = st->n_act, C = st->cap, j = st->knap;
    const int32_t *W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *list = act + (size_t)inst * max_items;
    int value = 0;
    if (nact > 0) value = rows[((size_t)inst * 2 + (nact & 1)) * row_len + C];
    int c = C;
    for (int q = nact - 1; q >= 0; --q) {
        const int t = list[q];
        const int w = W[t];
        if (w <= c) {
            const uint64_t word = keep[((size_t)inst * max_items + t) * keep_words + (c >> 6)];
            if ((word >> (c & 63)) & 1ull) {
                a.assignment[(size_t)inst * a.item_stride + t] = j;
                c -= w;
            }
        }
    }
    a.knap_value[(size_t)inst * a.knap_stride + j] = value;
    a.knap_load[(size_t)inst * a.knap_stride + j] = C - c;
    st->total += value;
    a.total_value[inst] = st->total;
}

}  // namespace

void seq_global_plan(int32_t max_capacity, int32_t max_items, int32_t max_batch, SeqGlobalPlan *p)
{
    p->threads = kThreads;
    p->cells_per_thread = kIter;
    const int64_t cells = (int64_t)max_capacity + 1;
    p->row_len = (int32_t)((cells + kWaveCells - 1) / kWaveCells * kWaveCells);
    p->keep_words = p->row_len / 64;
    p->max_items = max_items;
    p->max_batch = max_batch;
    p->scratch_bytes = (int64_t)(align256((size_t)max_batch * 2 * p->row_len * 4) +
                                 align256((size_t)max_batch * max_items * p->keep_words * 8) +
                                 align256((size_t)max_batch * max_items * 4) +
                                 align256((size_t)max_batch * sizeof(InstState)));
}

hipError_t seq_global_launch(const SeqGlobalPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                             Profiler *prof)
{
    const Scratch s = carve(p, scratch, p.max_batch);
    hipLaunchKernelGGL(sg_init, dim3(a.batch), dim3(kThreads), 0, st, a, s.state);
    const int tiles = p.row_len / kTileCells + (p.row_len % kTileCells ? 1 : 0);
    for (int stage = 0; stage < a.knap_stride; ++stage) {
        hipLaunchKernelGGL(sg_stage_setup, dim3(a.batch), dim3(64), 0, st, a, stage, s.state, s.act,
                           p.max_items);
        for (int q = 0; q < a.item_stride; ++q) {
            if (prof) prof->sweep_begin(st);
            hipLaunchKernelGGL(sg_sweep, dim3((unsigned)tiles * (unsigned)a.batch), dim3(kThreads), 0, st, a, q,
                               s.state, s.act, s.rows, s.keep, p.row_len, p.keep_words, p.max_items, tiles);
            if (prof) prof->sweep_end(st);
        }
        hipLaunchKernelGGL(sg_traceback, dim3((a.batch + 63) / 64), dim3(64), 0, st, a, s.state, s.act,
                           s.rows, s.keep, p.row_len, p.keep_words, p.max_items);
    }
    return hipGetLastError();
}

}  // namespace deft
