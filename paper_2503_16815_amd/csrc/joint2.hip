// Joint two-link solve (Sec. III.C, Problem 2 with one weight per link) with
// the (C1+1) x (C2+1) table in global memory.  Item q reads table q & 1 and
// writes the other:
//   new[a][b] = max(old[a][b], old[a - w0][b] + v, old[a][b - w1] + v)
// tested in that order, each replacing the incumbent only when strictly
// greater.  The 2-bit choice is stored as two bit planes (took link 0 / took
// link 1), one 64-bit ballot word per 64 consecutive b.  The first item reads
// zeros instead of a table.  One launch per item rank up to item_stride.
#include "instance_check.h"

namespace deft {

namespace {

constexpr int kThreads = 256;
constexpr int kTasksPerWave = 8;   // (row, 64-column segment) pairs per wavefront

struct InstState {
    int32_t status, n, c1, c2;
};

struct Scratch {
    int32_t *tab;       // [batch][2][rows][pitch]
    uint64_t *choice;   // [batch][max_items][rows][pitch / 64][2]
    InstState *state;   // [batch]
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

Scratch carve(const JointPlan &p, void *base)
{
    char *c = static_cast<char *>(base);
    Scratch s;
    s.tab = reinterpret_cast<int32_t *>(c);
    c += align256((size_t)p.max_batch * 2 * p.rows * p.pitch * 4);
    s.choice = reinterpret_cast<uint64_t *>(c);
    c += align256((size_t)p.max_batch * p.max_items * p.rows * (p.pitch / 64) * 16);
    s.state = reinterpret_cast<InstState *>(c);
    return s;
}

__global__ void __launch_bounds__(kThreads) jt_init(BatchArgs a, InstState *state)
{
    const int inst = blockIdx.x;
    const int status = check_instance(a, inst, true);
    clear_outputs(a, inst, status);
    if (threadIdx.x == 0) {
        InstState st;
        st.status = status;
        st.n = status == DEFT_OK ? a.n_items[inst] : 0;
        st.c1 = status == DEFT_OK ? a.capacities[(size_t)inst * a.knap_stride] : -1;
        st.c2 = status == DEFT_OK ? a.capacities[(size_t)inst * a.knap_stride + 1] : -1;
        state[inst] = st;
    }
}

__global__ void __launch_bounds__(kThreads)
jt_sweep(BatchArgs a, int q, const InstState *__restrict__ state, int32_t *tab, uint64_t *choice, int rows,
         int pitch, int max_items, int wgs_per_inst)
{
    const int inst = blockIdx.x / wgs_per_inst, wg = blockIdx.x % wgs_per_inst;
    const InstState st = state[inst];
    if (q >= st.n) return;
    const int lane = threadIdx.x & 63;
    const int segs = pitch / 64;
    const int w0 = a.weights[(size_t)inst * 2 * a.item_stride + q];
    const int w1 = a.weights[(size_t)inst * 2 * a.item_stride + a.item_stride + q];
    const int v = a.values[(size_t)inst * a.item_stride + q];
    const size_t tsz = (size_t)rows * pitch;
    const int32_t *__restrict__ src = tab + ((size_t)inst * 2 + (q & 1)) * tsz;
    int32_t *__restrict__ dst = tab + ((size_t)inst * 2 + ((q & 1) ^ 1)) * tsz;
    uint64_t *ch = choice + ((size_t)inst * max_items + q) * ((size_t)rows * segs * 2);
    const bool first = q == 0;
    const int task0 = (wg * (kThreads / 64) + (threadIdx.x >> 6)) * kTasksPerWave;
#pragma unroll 2
    for (int i = 0; i < kTasksPerWave; ++i) {
        const int task = task0 + i;
        const int ar = task / segs, sg = task % segs;
        if (ar > st.c1 || sg * 64 > st.c2) continue;
        const int b = sg * 64 + lane;
        const size_t at = (size_t)ar * pitch + b;
        int best = first ? 0 : src[at];
        bool t0 = false, t1 = false;
        if (ar >= w0) {
            const int cand = (first ? 0 : src[at - (size_t)w0 * pitch]) + v;
            if (cand > best) { best = cand; t0 = true; }
        }
        if (b >= w1) {
            const int cand = (first ? 0 : src[at - w1]) + v;
            if (cand > best) { best = cand; t0 = false; t1 = true; }
        }
        dst[at] = best;
        const unsigned long long m0 = __ballot(t0), m1 = __ballot(t1);
        if (lane < 2) ch[((size_t)ar * segs + sg) * 2 + lane] = lane ? m1 : m0;
    }
}

__global__ void __launch_bounds__(64)
jt_traceback(BatchArgs a, const InstState *__restrict__ state, const int32_t *tab, const uint64_t *choice,
             int rows, int pitch, int max_items)
{
    const int inst = blockIdx.x * 64 + threadIdx.x;
    if (inst >= a.batch) return;
    const InstState st = state[inst];
    if (st.status != DEFT_OK) return;
    const int segs = pitch / 64;
    const int32_t *W0 = a.weights + (size_t)inst * 2 * a.item_stride;
    const int32_t *W1 = W0 + a.item_stride;
    const int32_t *V = a.values + (size_t)inst * a.item_stride;
    int total = 0;
    if (st.n > 0) total = tab[((size_t)inst * 2 + (st.n & 1)) * ((size_t)rows * pitch) + (size_t)st.c1 * pitch + st.c2];
    int ar = st.c1, b = st.c2, val0 = 0, val1 = 0;
    for (int i = st.n - 1; i >= 0; --i) {
        const uint64_t *ch = choice + ((size_t)inst * max_items + i) * ((size_t)rows * segs * 2) +
                             ((size_t)ar * segs + (b >> 6)) * 2;
        const unsigned bit = b & 63;
        if ((ch[0] >> bit) & 1ull) {
            a.assignment[(size_t)inst * a.item_stride + i] = 0;
            ar -= W0[i];
            val0 += V[i];
        } else if ((ch[1] >> bit) & 1ull) {
            a.assignment[(size_t)inst * a.item_stride + i] = 1;
            b -= W1[i];
            val1 += V[i];
        }
    }
    int32_t *kv = a.knap_value + (size_t)inst * a.knap_stride;
    int32_t *kl = a.knap_load + (size_t)inst * a.knap_stride;
    kv[0] = val0; kv[1] = val1;
    kl[0] = st.c1 - ar; kl[1] = st.c2 - b;
    a.total_value[inst] = total;
}

}  // namespace

void joint_plan(int32_t max_c1, int32_t max_c2, int32_t max_items, int32_t max_batch, JointPlan *p)
{
    p->rows = max_c1 + 1;
    p->pitch = (max_c2 + 1 + 63) / 64 * 64;
    p->max_items = max_items;
    p->max_batch = max_batch;
    p->scratch_bytes = (int64_t)(align256((size_t)max_batch * 2 * p->rows * p->pitch * 4) +
                                 align256((size_t)max_batch * max_items * p->rows * (p->pitch / 64) * 16) +
                                 align256((size_t)max_batch * sizeof(InstState)));
}

hipError_t joint_launch(const JointPlan &p, const BatchArgs &a, void *scratch, hipStream_t st, Profiler *prof)
{
    const Scratch s = carve(p, scratch);
    hipLaunchKernelGGL(jt_init, dim3(a.batch), dim3(kThreads), 0, st, a, s.state);
    const int tasks = p.rows * (p.pitch / 64);
    const int per_wg = kTasksPerWave * (kThreads / 64);
    const int wgs = (tasks + per_wg - 1) / per_wg;
    for (int q = 0; q < a.item_stride; ++q) {
        if (prof) prof->sweep_begin(st);
        hipLaunchKernelGGL(jt_sweep, dim3((unsigned)wgs * (unsigned)a.batch), dim3(kThreads), 0, st, a, q, s.state,
                           s.tab, s.choice, p.rows, p.pitch, p.max_items, wgs);
        if (prof) prof->sweep_end(st);
    }
    hipLaunchKernelGGL(jt_traceback, dim3((a.batch + 63) / 64), dim3(64), 0, st, a, s.state, s.tab, s.choice,
                       p.rows, p.pitch, p.max_items);
    return hipGetLastError();
}

}  // namespace deft
