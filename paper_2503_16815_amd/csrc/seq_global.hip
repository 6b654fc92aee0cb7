// Sequential multiple-knapsack solve for capacities whose row does not fit LDS
// (Sec. III.B, Problem 1 per window).  The row lives in global memory in two
// buffers; offered item q reads buffer q & 1 and writes the other:
//   new[c] = max(old[c], old[c - w] + v)   for c >= w,   new[c] = old[c] below,
// with the take bit (old[c - w] + v > old[c]) collected per 64 cells by a
// wavefront ballot and stored as one 64-bit keep word.  The first offered item
// of a stage reads zeros instead of a buffer.
// Two ways to run a stage's sweeps:
//  * batches with at least one instance per two compute units: one persistent
//    workgroup per instance walks all offered items; the row streams once per
//    item through a ring in LDS, so each old cell is fetched from global memory
//    exactly once and both operands of a cell come from LDS (sg_sweep_all);
//  * smaller batches: one launch per offered-item rank, the row cut into tiles
//    over many workgroups (sg_sweep; the host cannot know how many items each
//    instance still offers, so it launches item_stride of them and a workgroup
//    whose instance has fewer exits); the shifted read hits cache lines another
//    wavefront has just fetched.
// Traffic per cell: 4 B read + 4 B write + 1/8 B keep.
#include <limits.h>

#include <type_traits>

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

constexpr int kAllThreads = 1024;   // persistent sweep: one workgroup per instance
constexpr int kAllWaves = kAllThreads / 64;
constexpr int kAllLoadWaves = 2;    // wavefronts that only move old cells from global memory into LDS
constexpr int kAllComputeWaves = kAllWaves - kAllLoadWaves;
constexpr int kSegCells = 256;      // one task / one 16-byte-per-lane LDS-direct load

typedef __attribute__((address_space(3))) int32_t lds_i32;
typedef const __attribute__((address_space(1))) int32_t global_ci32;

// Block hand-over barriers of sg_sweep_all: a loading wavefront arrives when its LDS-direct
// loads have landed, a computing wavefront when its LDS reads have (its row and keep stores
// stay in flight until the end of the item).  Asm, because the compiler puts a wait for all
// vector memory in front of every barrier it knows of once a kernel has LDS-direct loads.
__device__ __forceinline__ void barrier_after_loads() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void barrier_after_lds_reads() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// All offered items of one stage, one workgroup per instance.  The row is walked in
// ascending blocks of R segments (256 cells each).  Segment g lives in ring slot
// g % ring_segs; the ring holds the block being computed, the block being loaded and the
// cells up to w below the current block: 2 R + ceil(w / 256) + 1 <= ring_segs.  Heavier
// items read their shifted operand from global memory (separate instantiation).
// A compute task is one segment: lane l covers cells seg*256 + 64 j + l, j = 0..3, so the
// v_cmp masks are the keep words of the segment.
__global__ void __launch_bounds__(kAllThreads)
sg_sweep_all(BatchArgs a, const InstState *__restrict__ state, const int32_t *__restrict__ act, int32_t *rows,
             uint64_t *keep, int row_len, int keep_words, int max_items, int ring_segs)
{
    extern __shared__ __align__(16) int32_t ring[];  // [ring_segs][256]
    const int inst = blockIdx.x;
    const InstState st = state[inst];
    if (st.status != DEFT_OK || st.knap < 0 || st.n_act <= 0) return;
    const int C = st.cap;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool loader = wave < kAllLoadWaves;
    const int nseg = C / kSegCells + 1;  // segments holding cells 0 .. C (all inside row_len)
    const int ring_cells = ring_segs * kSegCells;
    const int32_t *W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *V = a.values + (size_t)inst * a.item_stride;
    const int32_t *list = act + (size_t)inst * max_items;

    // the first offered item sees an all-zero row: the ring is cleared once and not loaded
    for (int i = threadIdx.x; i < ring_cells; i += kAllThreads) ring[i] = 0;
    __syncthreads();

    for (int q = 0; q < st.n_act; ++q) {
        const int t = list[q];
        const int w = W[t], v = V[t];
        const int32_t *__restrict__ src = rows + ((size_t)inst * 2 + (q & 1)) * row_len;
        int32_t *__restrict__ dst = rows + ((size_t)inst * 2 + ((q & 1) ^ 1)) * row_len;
        uint64_t *kw = keep + ((size_t)inst * max_items + t) * keep_words;
        const bool first = q == 0;
        const int wsegs = (w + kSegCells - 1) / kSegCells + 1;  // segments the shifted operand reaches back
        const bool shifted_in_ring = wsegs + 2 <= ring_segs;
        const int R = max(1, (shifted_in_ring ? ring_segs - wsegs : ring_segs) / 2);

        // segments [lo, lo + R) of the old row -> ring; slot_lo = lo % ring_segs
        auto load_segs = [&](int lo, int slot_lo) {
            if (first) return;
            const int ns = min(R, nseg - lo);
            for (int g = wave; g < ns; g += kAllLoadWaves) {
                int slot = slot_lo + g;
                if (slot >= ring_segs) slot -= ring_segs;
                __builtin_amdgcn_global_load_lds((global_ci32 *)(src + (size_t)(lo + g) * kSegCells + lane * 4),
                                                 (lds_i32 *)(ring + (size_t)slot * kSegCells), 16, 0, 0);
            }
        };

        // One task = one segment.  IN_RING: the shifted operand comes from the ring.
        // KIND 0: the whole segment lies at or above w; 1: w falls inside it (cells below w
        // keep their value); 2: the whole segment lies below w (copied through).
        auto task = [&](auto in_ring_tag, auto kind_tag, int seg, int slot) {
            constexpr bool IN_RING = decltype(in_ring_tag)::value;
            constexpr int KIND = decltype(kind_tag)::value;
            const int32_t *own = ring + (size_t)slot * kSegCells + lane;
            const int c0 = seg * kSegCells + lane;
            int cen[4], sh[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) cen[j] = own[j * 64];
            if (KIND != 2) {
                if (IN_RING) {
                    // ring position of the segment's first cell minus w, brought into [0, ring_cells)
                    int base = slot * kSegCells - w;
                    base += base < 0 ? ring_cells : 0;
                    if (base + kSegCells <= ring_cells) {
                        // the 256 shifted cells are contiguous in the ring: immediate offsets
                        const int32_t *shp = ring + base + lane;
#pragma unroll
                        for (int j = 0; j < 4; ++j) sh[j] = shp[j * 64];
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            unsigned o = (unsigned)(base + lane + j * 64);
                            o = min(o, o - (unsigned)ring_cells);  // wraps past the ring's end
                            sh[j] = ring[o];
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int c = c0 + j * 64;
                        sh[j] = (c >= w && !first) ? src[c - w] : 0;
                    }
                }
            }
            unsigned long long m[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int best = cen[j];
                m[j] = 0;
                if (KIND != 2) {
                    int cand = sh[j] + v;
                    if (KIND == 1 || !IN_RING) cand = c0 + j * 64 < w ? INT_MIN : cand;
                    m[j] = __ballot(cand > best);
                    best = max(best, cand);
                }
                dst[(size_t)c0 + j * 64] = best;
            }
            if (lane < 4) {
                unsigned long long wsel = 0;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (jj == lane) wsel = m[jj];
                kw[seg * 4 + lane] = wsel;
            }
        };

        if (loader) {
            load_segs(0, 0);
            barrier_after_loads();
        } else {
            barrier_after_lds_reads();
        }
        int slot_lo = 0;  // lo % ring_segs
        for (int lo = 0; lo < nseg; lo += R) {
            int slot_next = slot_lo + R;
            if (slot_next >= ring_segs) slot_next -= ring_segs;
            if (loader) {
                if (lo + R < nseg) load_segs(lo + R, slot_next);
                barrier_after_loads();  // the next block is in the ring
            } else {
                const int ns = min(R, nseg - lo);
                const std::true_type yes{};
                const std::false_type no{};
                for (int g = wave - kAllLoadWaves; g < ns; g += kAllComputeWaves) {
                    const int seg = lo + g;
                    int slot = slot_lo + g;
                    if (slot >= ring_segs) slot -= ring_segs;
                    const int c_first = seg * kSegCells;
                    if (c_first >= w) {
                        if (shifted_in_ring) task(yes, std::integral_constant<int, 0>{}, seg, slot);
                        else task(no, std::integral_constant<int, 0>{}, seg, slot);
                    } else if (c_first + kSegCells > w) {
                        if (shifted_in_ring) task(yes, std::integral_constant<int, 1>{}, seg, slot);
                        else task(no, std::integral_constant<int, 1>{}, seg, slot);
                    } else {
                        task(yes, std::integral_constant<int, 2>{}, seg, slot);
                    }
                }
                barrier_after_lds_reads();  // this block's slots may be reused
            }
            slot_lo = slot_next;
        }
        // the next item reads what this one wrote (other wavefronts' cells included)
        __threadfence_block();
        __syncthreads();
    }
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

void seq_global_plan(int32_t max_capacity, int32_t max_items, int32_t max_batch, int32_t lds_per_wg_bytes,
                     int32_t compute_units, SeqGlobalPlan *p)
{
    p->threads = kThreads;
    p->cells_per_thread = kIter;
    p->ring_segs = lds_per_wg_bytes / (kSegCells * 4);
    p->lds_bytes = p->ring_segs * kSegCells * 4;
    // one workgroup per instance pays once the batch covers at least half the compute units
    p->persistent_min_batch = p->ring_segs >= 8 ? (compute_units + 1) / 2 : INT_MAX;
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

hipError_t seq_global_prepare(const SeqGlobalPlan &p)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&sg_sweep_all),
                               hipFuncAttributeMaxDynamicSharedMemorySize, p.lds_bytes);
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
        if (a.batch >= p.persistent_min_batch) {
            if (prof) prof->sweep_begin(st);
            hipLaunchKernelGGL(sg_sweep_all, dim3((unsigned)a.batch), dim3(kAllThreads), (size_t)p.lds_bytes, st, a,
                               s.state, s.act, s.rows, s.keep, p.row_len, p.keep_words, p.max_items, p.ring_segs);
            if (prof) prof->sweep_end(st);
        } else {
            for (int q = 0; q < a.item_stride; ++q) {
                if (prof) prof->sweep_begin(st);
                hipLaunchKernelGGL(sg_sweep, dim3((unsigned)tiles * (unsigned)a.batch), dim3(kThreads), 0, st, a, q,
                                   s.state, s.act, s.rows, s.keep, p.row_len, p.keep_words, p.max_items, tiles);
                if (prof) prof->sweep_end(st);
            }
        }
        hipLaunchKernelGGL(sg_traceback, dim3((a.batch + 63) / 64), dim3(64), 0, st, a, s.state, s.act,
                           s.rows, s.keep, p.row_len, p.keep_words, p.max_items);
    }
    return hipGetLastError();
}

}  // namespace deft
