// The greedy heuristic of the paper's own Solver (Sec. III.C), batched: capacities sorted
// ascending, bucket times sorted descending, then every knapsack from the smallest up
// takes, longest bucket first, whatever still fits.  It is here to be compared with the
// exact solvers on the same inputs, not to be fast: one 256-thread workgroup per
// instance sorts the times in LDS (bitonic, 64-bit keys = time and index, so that equal
// times keep their index order) and its first wavefront does the placement, which is a
// chain of dependent decisions (each item sees what the ones before it left).
#include "instance_check.h"

namespace deft {

namespace {

constexpr int kThreads = 256;
constexpr int kIndexBits = 12;  // item indices < 4096
constexpr int kMaxKnap = 64;

// LDS: [P keys of 8 bytes][item_stride placed flags, one byte each, padded to 8][64 ints: knapsack order]
__global__ void __launch_bounds__(kThreads) greedy_kernel(BatchArgs a, int per_link, int key_slots, int flag_bytes)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(lds_raw);
    unsigned char *placed = lds_raw + (size_t)key_slots * 8;
    int32_t *order = reinterpret_cast<int32_t *>(placed + flag_bytes);

    const int inst = blockIdx.x, tid = threadIdx.x;
    const int status = check_instance(a, inst, per_link != 0);
    clear_outputs(a, inst, status);
    if (status != DEFT_OK) return;  // uniform

    const int n = a.n_items[inst], m = a.n_knapsacks[inst];
    const int32_t *W = a.weights + (size_t)inst * (per_link ? 2 : 1) * a.item_stride;
    const int32_t *V = a.values + (size_t)inst * a.item_stride;
    const int32_t *cap = a.capacities + (size_t)inst * a.knap_stride;
    int32_t *out_asg = a.assignment + (size_t)inst * a.item_stride;

    for (int i = tid; i < flag_bytes; i += kThreads) placed[i] = 0;
    // knapsack ids by capacity, ascending, equal capacities by id: rank by counting
    if (tid < m) {
        const int c = cap[tid];
        int rank = 0;
        for (int j = 0; j < m; ++j) {
            const int cj = cap[j];
            rank += (cj < c || (cj == c && j < tid)) ? 1 : 0;
        }
        order[rank] = tid;
    }
    int P = 64;  // keys sorted: the power of two covering n
    while (P < n) P <<= 1;
    __syncthreads();

    long long total = 0;
    for (int s = 0; s < m; ++s) {
        const int j = order[s];
        const int32_t *time = per_link ? W + (size_t)j * a.item_stride : W;
        if (s == 0 || per_link) {
            // key = time * 4096 + (4095 - index): descending keys = descending time, ascending index
            for (int t = tid; t < P; t += kThreads)
                keys[t] = t < n ? ((unsigned long long)(uint32_t)time[t] << kIndexBits) |
                                      (unsigned long long)((1 << kIndexBits) - 1 - t)
                                : 0ull;  // below every real key (times are >= 1)
            __syncthreads();
            for (int k = 2; k <= P; k <<= 1) {
                for (int d = k >> 1; d > 0; d >>= 1) {
                    for (int t = tid; t < P; t += kThreads) {
                        const int u = t ^ d;
                        if (u > t) {
                            const unsigned long long x = keys[t], y = keys[u];
                            const bool falling = (t & k) == 0;
                            if (falling ? x < y : x > y) {
                                keys[t] = y;
                                keys[u] = x;
                            }
                        }
                    }
                    __syncthreads();
                }
            }
        }
        if (tid < 64) {
            int left = cap[j];  // uniform across the wavefront
            long long value = 0;
            for (int base = 0; base < n && left > 0; base += 64) {
                const int t = base + tid;
                const unsigned long long key = t < n ? keys[t] : 0ull;
                const int w = (int)(key >> kIndexBits);
                const int idx = (1 << kIndexBits) - 1 - (int)(key & ((1u << kIndexBits) - 1));
                const bool open = t < n && placed[idx] == 0;
                // what is left only shrinks: a lane that does not fit now never will in this chunk
                unsigned long long cand = __ballot(open && w <= left);
                unsigned long long taken = 0;
                while (cand) {
                    const int l = __builtin_ctzll(cand);
                    cand &= cand - 1;
                    const int wl = __builtin_amdgcn_readlane(w, l);
                    if (wl <= left) {
                        left -= wl;
                        taken |= 1ull << l;
                    }
                }
                if ((taken >> tid) & 1ull) {
                    placed[idx] = 1;
                    out_asg[idx] = j;
                    value += V[idx];
                }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) value += __shfl_down(value, off);
            value = __shfl(value, 0);
            if (tid == 0) {
                a.knap_value[(size_t)inst * a.knap_stride + j] = (int32_t)value;
                a.knap_load[(size_t)inst * a.knap_stride + j] = cap[j] - left;
            }
            total += value;
        }
        __syncthreads();  // the flags are set and the keys are free to be rebuilt
    }
    if (tid == 0) a.total_value[inst] = total;
}

int key_slots_for(int item_stride)
{
    int p = 64;
    while (p < item_stride) p <<= 1;
    return p;
}

}  // namespace

hipError_t greedy_prepare(int32_t max_items)
{
    const int lds = key_slots_for(max_items) * 8 + ((max_items + 7) & ~7) + kMaxKnap * 4;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&greedy_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

hipError_t greedy_launch(const BatchArgs &a, bool per_link, hipStream_t st)
{
    if (a.item_stride > (1 << kIndexBits) || a.knap_stride > kMaxKnap) return hipErrorInvalidValue;
    const int key_slots = key_slots_for(a.item_stride);
    const int flag_bytes = (a.item_stride + 7) & ~7;
    const size_t lds = (size_t)key_slots * 8 + flag_bytes + kMaxKnap * 4;
    hipLaunchKernelGGL(greedy_kernel, dim3((unsigned)a.batch), dim3(kThreads), lds, st, a, per_link ? 1 : 0,
                       key_slots, flag_bytes);
    return hipGetLastError();
}

}  // namespace deft
