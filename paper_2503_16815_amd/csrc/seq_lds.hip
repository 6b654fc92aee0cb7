// Sequential multiple-knapsack solve with the capacity row resident in LDS.
//
// One launch solves every stage of every instance (Sec. III.B: Problem 1 per
// window, windows filled one after the other).  An instance is owned by T
// lanes.  Cell c of the row lives in lane (c mod T), register slot (c div T),
// and a copy lives in LDS so that the shifted operand row[c - w] can be read
// by whichever lane needs it.  Per offered item:
//   phase 1  every lane reads row[c - w] for its cells          (LDS, 4 B/cell)
//   barrier
//   phase 2  cand = row[c - w] + v; take = cand > row[c];
//            row[c] = max(row[c], cand) kept in registers and written back
//            (LDS, 4 B/cell); take bits are shifted into one 32-bit word per
//            32 register slots and stored to the keep table (HBM, 1/8 B/cell)
//   barrier
// The textbook reverse sweep (c from C down to w) exists to read old values
// only; reading everything before the barrier gives the same result.
// Cells below w are not touched: a wavefront skips 64-cell segments that lie
// wholly below w or above C; in the one segment that straddles w the lanes
// below w read a guard zone holding INT_MIN, which can never win.
//
// After the last item of a stage the same lanes trace the selection back
// from (last offered item, C) through the keep words just written and mark
// the chosen items, which the next stage then leaves out.
#include <limits.h>

#include "kernels.h"

namespace deft {

namespace {

constexpr int kGuardCells = 64;

template <int T>
__device__ __forceinline__ void lds_sync()
{
    if constexpr (T == 64) {
        // one wavefront: LDS executes its instructions in order; only the
        // compiler has to be kept from reordering
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
    } else {
        // waits for LDS traffic only: keep-table stores stay in flight
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    }
}

// Makes the keep words written by all lanes of the instance visible to the
// lanes that trace back (global memory, through L2; L1 is bypassed on read).
template <int T>
__device__ __forceinline__ void global_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    if constexpr (T == 64) {
        __builtin_amdgcn_wave_barrier();
    } else {
        __builtin_amdgcn_s_barrier();
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// bits = 2 * bits + (cand > own): compare into vcc, add-with-carry.
__device__ __forceinline__ uint32_t shift_in_take(uint32_t bits, int cand, int own)
{
    uint32_t out;
    asm("v_cmp_gt_i32 vcc, %2, %3\n\tv_addc_co_u32 %0, vcc, %1, %1, vcc"
        : "=v"(out)
        : "v"(bits), "v"(cand), "v"(own)
        : "vcc");
    return out;
}

struct LdsLayout {
    int32_t row_cells, n_pad, ints_per_inst;
};

template <int T, int K>
__global__ void __launch_bounds__(T == 64 ? 256 : T)
seq_lds_kernel(BatchArgs a, LdsLayout lay, uint32_t *__restrict__ keep, int64_t keep_words_per_inst)
{
    extern __shared__ __align__(16) int32_t lds_raw[];
    constexpr int NW = (K + 31) / 32;
    constexpr int LOG_T = (T == 64) ? 6 : (T == 256) ? 8 : (T == 512) ? 9 : 10;
    static_assert((1 << LOG_T) == T, "T must be 64, 256, 512 or 1024");

    const int sub = (T == 64) ? (int)(threadIdx.x >> 6) : 0;
    const int tid = (T == 64) ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
    const int inst = (T == 64) ? (int)blockIdx.x * 4 + sub : (int)blockIdx.x;
    if (inst >= a.batch) return;  // whole wavefront (T == 64) or never (grid == batch)

    int32_t *guard = lds_raw + (size_t)sub * lay.ints_per_inst;
    int32_t *row = guard + kGuardCells;
    int16_t *asg = reinterpret_cast<int16_t *>(row + lay.row_cells);
    int16_t *act = asg + lay.n_pad;
    int32_t *misc = reinterpret_cast<int32_t *>(act + lay.n_pad);
    // misc: [0] fault flags, [1] offered-item count, [2..3] value sum, [4..5] fill-order seen mask

    const int n = a.n_items[inst];
    const int m = a.n_knapsacks[inst];
    const int32_t *__restrict__ W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *__restrict__ V = a.values + (size_t)inst * a.item_stride;
    const int32_t *__restrict__ cap = a.capacities + (size_t)inst * a.knap_stride;
    const int32_t *__restrict__ ord =
        a.fill_order ? a.fill_order + (size_t)inst * a.knap_stride : nullptr;
    int32_t *out_asg = a.assignment + (size_t)inst * a.item_stride;
    int32_t *out_kv = a.knap_value + (size_t)inst * a.knap_stride;
    int32_t *out_kl = a.knap_load + (size_t)inst * a.knap_stride;
    uint32_t *kp = keep + (size_t)inst * keep_words_per_inst;

    // ---- per-instance validation -------------------------------------------
    if (tid < 6) misc[tid] = 0;
    if (tid < kGuardCells) guard[tid] = INT_MIN;
    for (int i = tid; i < lay.n_pad; i += T) asg[i] = -1;
    lds_sync<T>();
    {
        uint32_t flags = 0;
        unsigned long long vs = 0;
        const bool counts_ok = n >= 0 && n <= a.item_stride && m >= 0 && m <= a.knap_stride;
        if (!counts_ok) {
            flags = 1;
        } else {
            for (int i = tid; i < n; i += T) {
                const int w = W[i], v = V[i];
                if (w < 1 || v < 0) flags |= 1; else vs += (unsigned)v;
            }
            for (int j = tid; j < m; j += T) {
                const int c = cap[j];
                if (c < 0) flags |= 1; else if (c > a.max_capacity) flags |= 2;
                if (ord) {
                    const int o = ord[j];
                    if (o < 0 || o >= m) {
                        flags |= 1;
                    } else {
                        const uint32_t bit = 1u << (o & 31);
                        const uint32_t old = atomicOr(reinterpret_cast<uint32_t *>(&misc[4 + (o >> 5)]), bit);
                        if (old & bit) flags |= 1;
                    }
                }
            }
        }
        if (flags) atomicOr(reinterpret_cast<uint32_t *>(&misc[0]), flags);
        if (vs) atomicAdd(reinterpret_cast<unsigned long long *>(&misc[2]), vs);
    }
    lds_sync<T>();
    int status = DEFT_OK;
    {
        const uint32_t flags = (uint32_t)misc[0];
        const unsigned long long vs = *reinterpret_cast<unsigned long long *>(&misc[2]);
        if (flags & 1) status = DEFT_ERR_INVALID_ARG;
        else if (flags & 2) status = DEFT_ERR_LIMIT;
        else if (vs >= (1ull << 31)) status = DEFT_ERR_OVERFLOW;
    }
    status = uniform(status);
    if (tid == 0) {
        for (int j = 0; j < a.knap_stride; ++j) { out_kv[j] = 0; out_kl[j] = 0; }
        a.status[inst] = status;
    }
    if (status != DEFT_OK) {
        for (int i = tid; i < a.item_stride; i += T) out_asg[i] = -1;
        if (tid == 0) a.total_value[inst] = 0;
        return;
    }

    // ---- stages ----------------------------------------------------------------
    const int wave_first = tid & ~63;  // first lane index of this wavefront within the instance
    long long total = 0;
    for (int s = 0; s < m; ++s) {
        const int j = uniform(ord ? ord[s] : s);
        const int C = uniform(cap[j]);

        // offered items: not yet placed and able to fit at all, ascending index
        if (tid < 64) {
            int cnt = 0;
            for (int i0 = 0; i0 < n; i0 += 64) {
                const int i = i0 + tid;
                const bool f = i < n && asg[i] < 0 && W[i] <= C;
                const unsigned long long mask = __ballot(f);
                if (f) act[cnt + __popcll(mask & ((1ull << tid) - 1ull))] = (int16_t)i;
                cnt += __popcll(mask);
            }
            if (tid == 0) misc[1] = cnt;
        }

        // 64-cell segments [k*T + wave_first, +64) with k < kmax hold cells <= C
        const int kmax = uniform(C >= wave_first ? ((C - wave_first) >> LOG_T) + 1 : 0);
        int own[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            own[k] = 0;
            if (k < kmax) row[k * T + tid] = 0;
        }
        lds_sync<T>();
        const int nact = uniform(misc[1]);

        for (int q = 0; q < nact; ++q) {
            const int t = uniform(act[q]);
            const int w = uniform(W[t]);
            const int v = uniform(V[t]);
            // first segment of this wavefront that reaches cell w
            const int kmin = uniform(max(0, w - wave_first - 63 + T - 1) >> LOG_T);
            const int32_t *src = row + (tid - w);
            int rd[K];
#pragma unroll
            for (int k = K - 1; k >= 0; --k)
                if (k >= kmin && k < kmax) rd[k] = src[k * T];
            lds_sync<T>();

            uint32_t bits[NW];
#pragma unroll
            for (int x = 0; x < NW; ++x) bits[x] = 0;
#pragma unroll
            for (int k = K - 1; k >= 0; --k) {
                if (k >= kmin && k < kmax) {
                    const int cand = rd[k] + v;
                    bits[k >> 5] = shift_in_take(bits[k >> 5], cand, own[k]);
                    own[k] = max(own[k], cand);
                    row[k * T + tid] = own[k];
                }
            }
            // the lowest processed slot of word x sits at bit 0: move it to its place
#pragma unroll
            for (int x = 0; x < NW; ++x) {
                const int sh = kmin - 32 * x;
                if (sh > 0) bits[x] = sh < 32 ? bits[x] << sh : 0u;
                kp[((size_t)t * NW + x) * T + tid] = bits[x];
            }
            lds_sync<T>();
        }

        const int value = uniform(row[C]);

        // ---- traceback ------------------------------------------------------------
        global_sync<T>();
        if (tid == 0) {
            int c = C;
            for (int q = nact - 1; q >= 0; --q) {
                const int t = act[q];
                const int w = W[t];
                if (w <= c) {
                    const int k = c >> LOG_T, lane = c & (T - 1);
                    const uint32_t word = __hip_atomic_load(
                        &kp[((size_t)t * NW + (k >> 5)) * T + lane], __ATOMIC_RELAXED,
                        __HIP_MEMORY_SCOPE_AGENT);
                    if ((word >> (k & 31)) & 1u) {
                        asg[t] = (int16_t)j;
                        c -= w;
                    }
                }
            }
            out_kv[j] = value;
            out_kl[j] = C - c;
        }
        total += value;
        lds_sync<T>();
    }

    for (int i = tid; i < a.item_stride; i += T) out_asg[i] = asg[i];
    if (tid == 0) a.total_value[inst] = total;
}

struct Variant {
    int threads, cells;
    const void *fn;
};

#define DEFT_VARIANT(T, K) { T, K, reinterpret_cast<const void *>(&seq_lds_kernel<T, K>) }
const Variant kVariants[] = {
    DEFT_VARIANT(64, 16),    // capacity <= 1023: one wavefront per instance, four per workgroup
    DEFT_VARIANT(256, 16),   // <= 4095
    DEFT_VARIANT(256, 32),   // <= 8191
    DEFT_VARIANT(256, 51),   // <= 13055
    DEFT_VARIANT(512, 51),   // <= 26111
    DEFT_VARIANT(1024, 40),  // <= 40959 (if LDS allows)
};
#undef DEFT_VARIANT
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

template <int T, int K>
hipError_t launch_one(const SeqLdsPlan &p, const BatchArgs &a, uint32_t *keep, hipStream_t st)
{
    const LdsLayout lay{p.row_cells, p.n_pad, p.lds_bytes / p.inst_per_wg / 4};
    const unsigned grid = (unsigned)((a.batch + p.inst_per_wg - 1) / p.inst_per_wg);
    hipLaunchKernelGGL((seq_lds_kernel<T, K>), dim3(grid), dim3(p.wg_threads), (size_t)p.lds_bytes, st,
                       a, lay, keep, p.keep_words_per_inst);
    return hipGetLastError();
}

}  // namespace

bool seq_lds_plan(int32_t max_capacity, int32_t max_items, int32_t lds_per_cu_bytes,
                  int32_t lds_per_wg_bytes, SeqLdsPlan *plan)
{
    (void)lds_per_cu_bytes;
    const int64_t nseg = (int64_t)max_capacity / 64 + 1;
    const int32_t n_pad = (max_items + 3) & ~3;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        const int64_t seg_per_slot = v.threads / 64;
        if (nseg > (int64_t)v.cells * seg_per_slot) continue;
        const int64_t row_cells = nseg * 64;
        const int64_t per_inst = (kGuardCells + row_cells) * 4 + (int64_t)n_pad * 4 + 8 * 4;
        const int inst_per_wg = v.threads == 64 ? 4 : 1;
        const int64_t lds = per_inst * inst_per_wg;
        if (lds > lds_per_wg_bytes) continue;
        plan->variant = i;
        plan->threads = v.threads;
        plan->cells_per_thread = v.cells;
        plan->keep_words = (v.cells + 31) / 32;
        plan->row_cells = (int32_t)row_cells;
        plan->n_pad = n_pad;
        plan->lds_bytes = (int32_t)lds;
        plan->wg_threads = v.threads == 64 ? 256 : v.threads;
        plan->inst_per_wg = inst_per_wg;
        plan->wg_per_cu = 0;
        plan->keep_words_per_inst = (int64_t)max_items * plan->keep_words * v.threads;
        return true;
    }
    return false;
}

hipError_t seq_lds_prepare(SeqLdsPlan *plan)
{
    const void *fn = kVariants[plan->variant].fn;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, plan->lds_bytes);
    if (e != hipSuccess) return e;
    int nb = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, plan->wg_threads, (size_t)plan->lds_bytes);
    if (e != hipSuccess) return e;
    plan->wg_per_cu = nb;
    return nb > 0 ? hipSuccess : hipErrorInvalidConfiguration;
}

hipError_t seq_lds_launch(const SeqLdsPlan &p, const BatchArgs &a, uint32_t *keep, hipStream_t st)
{
    switch (p.variant) {
    case 0: return launch_one<64, 16>(p, a, keep, st);
    case 1: return launch_one<256, 16>(p, a, keep, st);
    case 2: return launch_one<256, 32>(p, a, keep, st);
    case 3: return launch_one<256, 51>(p, a, keep, st);
    case 4: return launch_one<512, 51>(p, a, keep, st);
    case 5: return launch_one<1024, 40>(p, a, keep, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace deft
