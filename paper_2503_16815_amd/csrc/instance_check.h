// Per-instance input checks shared by the set-up kernels of the global-memory
// paths.  Run by one 256-thread workgroup per instance.  Returns the instance's
// deft_status_t (same value in every thread).  Precedence: invalid data, then
// create-time limits, then value-sum overflow.
#pragma once

#include "kernels.h"

namespace deft {

__device__ inline int check_instance(const BatchArgs &a, int inst, bool joint)
{
    __shared__ uint32_t s_flags;
    __shared__ uint32_t s_seen[2];
    __shared__ unsigned long long s_vsum;
    const int tid = threadIdx.x, nt = blockDim.x;
    if (tid == 0) { s_flags = 0; s_seen[0] = s_seen[1] = 0; s_vsum = 0; }
    __syncthreads();
    const int n = a.n_items[inst], m = a.n_knapsacks[inst];
    uint32_t flags = 0;
    unsigned long long vs = 0;
    const bool counts_ok = n >= 0 && n <= a.item_stride && m >= 0 && m <= a.knap_stride && (!joint || m == 2) &&
                           (a.mode != DEFT_MODE_CAPACITY_SWEEP || m <= 31) && (a.mode != DEFT_MODE_RECURSIVE || m == 1);
    if (!counts_ok) {
        flags = 1;
    } else {
        const size_t wstride = joint ? 2 * (size_t)a.item_stride : (size_t)a.item_stride;
        const int32_t *W = a.weights + (size_t)inst * wstride;
        const int32_t *V = a.values + (size_t)inst * a.item_stride;
        const int32_t *cap = a.capacities + (size_t)inst * a.knap_stride;
        for (int i = tid; i < n; i += nt) {
            const int v = V[i];
            bool bad = W[i] < 1 || v < 0;
            if (joint) bad = bad || W[a.item_stride + i] < 1;
            if (a.mode == DEFT_MODE_RECURSIVE) bad = bad || a.drop_time[(size_t)inst * a.item_stride + i] < 0;
            if (bad) flags |= 1; else vs += (unsigned)v;
        }
        for (int j = tid; j < m; j += nt) {
            const int c = cap[j];
            const int lim = joint ? (j == 0 ? a.max_c1 : a.max_c2) : a.max_capacity;
            if (c < 0) flags |= 1; else if (c > lim) flags |= 2;
            if (!joint && a.fill_order) {
                const int o = a.fill_order[(size_t)inst * a.knap_stride + j];
                if (o < 0 || o >= m) {
                    flags |= 1;
                } else {
                    const uint32_t bit = 1u << (o & 31);
                    if (atomicOr(&s_seen[o >> 5], bit) & bit) flags |= 1;
                }
            }
        }
    }
    if (flags) atomicOr(&s_flags, flags);
    if (vs) atomicAdd(&s_vsum, vs);
    __syncthreads();
    int status = DEFT_OK;
    if (s_flags & 1) status = DEFT_ERR_INVALID_ARG;
    else if (s_flags & 2) status = DEFT_ERR_LIMIT;
    else if (s_vsum >= (1ull << 31)) status = DEFT_ERR_OVERFLOW;
    return status;
}

// Clears every output slot of the instance and records its status (assignment: no knapsack,
// or, for the capacity sweep, the empty mask).
__device__ inline void clear_outputs(const BatchArgs &a, int inst, int status)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int none = a.mode == DEFT_MODE_CAPACITY_SWEEP ? 0 : -1;
    for (int i = tid; i < a.item_stride; i += nt) a.assignment[(size_t)inst * a.item_stride + i] = none;
    for (int j = tid; j < a.knap_stride; j += nt) {
        a.knap_value[(size_t)inst * a.knap_stride + j] = 0;
        a.knap_load[(size_t)inst * a.knap_stride + j] = 0;
    }
    if (tid == 0) {
        a.total_value[inst] = 0;
        a.status[inst] = status;
    }
}

}  // namespace deft
