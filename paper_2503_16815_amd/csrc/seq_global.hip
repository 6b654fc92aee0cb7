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
    int32_t buf;   // row buffer holding the stage's final row; -1: the parity of n_act says
    // Algorithm 1: the best level met so far (its value, the length of its list, its remaining time)
    int32_t best_value, best_length, best_remain;
};

struct Scratch {
    int32_t *rows;      // [batch][2][row_len]
    uint64_t *keep;     // [batch][max_items][keep_words]
    int32_t *act;       // [batch][max_items]
    int32_t *probe;     // [batch][max_items]  Algorithm 1: remaining time of the level that ends before entry q
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
    s.probe = reinterpret_cast<int32_t *>(c);
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
// Algorithm 1 (one stage): the whole list is offered in its order, and entry q gets the
// remaining time of the level that ends before it, R - sum of drop_time over the entries
// from q on (-1 if negative), from a suffix sum taken 64 entries at a time from the end.
__global__ void __launch_bounds__(64) sg_levels_setup(BatchArgs a, InstState *state, int32_t *act, int32_t *probe,
                                                      int max_items)
{
    const int inst = blockIdx.x, lane = threadIdx.x;
    InstState *st = &state[inst];
    if (st->status != DEFT_OK) {
        if (lane == 0) st->n_act = 0, st->knap = -1, st->buf = -1;
        return;
    }
    const int n = a.n_items[inst];
    const int C = a.capacities[(size_t)inst * a.knap_stride];
    const int32_t *drop = a.drop_time + (size_t)inst * a.item_stride;
    long long behind = 0;
    for (int i0 = (n - 1) & ~63; i0 >= 0 && n > 0; i0 -= 64) {
        const int i = i0 + lane;
        long long x = i < n ? drop[i] : 0;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long y = __shfl_down(x, off);
            if (lane + off < 64) x += y;
        }
        if (i < n) {
            const long long left = (long long)C - (x + behind);
            act[(size_t)inst * max_items + i] = i;
            probe[(size_t)inst * max_items + i] = left < 0 ? -1 : (int)left;
        }
        behind += __shfl(x, 0);
    }
    if (lane == 0) {
        st->n_act = n; st->knap = 0; st->cap = C; st->buf = -1;
        st->best_value = 0; st->best_length = 0; st->best_remain = 0;
    }
}

__global__ void __launch_bounds__(64) sg_stage_setup(BatchArgs a, int s, InstState *state, int32_t *act,
                                                     int max_items)
{
    const int inst = blockIdx.x, lane = threadIdx.x;
    InstState *st = &state[inst];
    const int m = a.n_knapsacks[inst];
    if (st->status != DEFT_OK || s >= m) {
        if (lane == 0) st->n_act = 0, st->knap = -1, st->buf = -1;
        return;
    }
    const int n = a.n_items[inst];
    // Capacity sweep (Sec. IV.C feedback): one stage, swept at the largest of the instance's
    // capacities; every item is offered and nothing is settled here (the smaller capacities
    // are read off the same final row).
    const bool caps_sweep = a.mode == DEFT_MODE_CAPACITY_SWEEP;
    const int j = caps_sweep ? 0 : a.fill_order ? a.fill_order[(size_t)inst * a.knap_stride + s] : s;
    int C = a.capacities[(size_t)inst * a.knap_stride + j];
    if (caps_sweep)
        for (int x = 1; x < m; ++x) C = max(C, a.capacities[(size_t)inst * a.knap_stride + x]);
    const int32_t *W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *asg = a.assignment + (size_t)inst * a.item_stride;
    int32_t *list = act + (size_t)inst * max_items;
    int cnt = 0;
    long long offered_weight = 0;
    for (int i0 = 0; i0 < n; i0 += 64) {
        const int i = i0 + lane;
        const bool f = i < n && (caps_sweep || asg[i] < 0) && W[i] <= C;
        const unsigned long long mask = __ballot(f);
        if (f) {
            list[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = i;
            offered_weight += W[i];
        }
        cnt += __popcll(mask);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) offered_weight += __shfl_down(offered_weight, off);
    offered_weight = __shfl(offered_weight, 0);
    if (!caps_sweep && offered_weight <= C) {
        // Nothing is offered, or everything offered fits together: the DP and its walk would
        // take exactly the offered items of positive value (at every step of the walk the
        // capacity left still holds all earlier items, and a zero-value item never strictly
        // improves a cell).  The stage is settled here; no sweep, no walk.
        const int32_t *V = a.values + (size_t)inst * a.item_stride;
        long long vsum = 0, lsum = 0;
        for (int i = lane; i < n; i += 64) {
            const int w = W[i], v = V[i];
            if (asg[i] < 0 && w <= C && v > 0) {
                a.assignment[(size_t)inst * a.item_stride + i] = j;
                vsum += v;
                lsum += w;
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            vsum += __shfl_down(vsum, off);
            lsum += __shfl_down(lsum, off);
        }
        if (lane == 0) {
            a.knap_value[(size_t)inst * a.knap_stride + j] = (int)vsum;
            a.knap_load[(size_t)inst * a.knap_stride + j] = (int)lsum;
            st->total += vsum;
            a.total_value[inst] = st->total;
            st->n_act = 0, st->knap = -1, st->buf = -1;
        }
        return;
    }
    if (lane == 0) { st->n_act = cnt; st->knap = j; st->cap = C; st->buf = -1; }
}

// Offered item q of every instance: one pass over the row.
__global__ void __launch_bounds__(kThreads)
sg_sweep(BatchArgs a, int q, InstState *state, const int32_t *__restrict__ act, const int32_t *__restrict__ probe,
         int32_t *rows, uint64_t *keep, int row_len, int keep_words, int max_items, int tiles)
{
    const int inst = blockIdx.x / tiles, tile = blockIdx.x % tiles;
    const InstState st = state[inst];
    if (q >= st.n_act) return;
    const int C = st.cap;
    if (a.mode == DEFT_MODE_RECURSIVE && tile == 0 && threadIdx.x == 0 && q > 0) {
        // Algorithm 1: the row before item q is the row of the level that ends here; a
        // shallower level replaces the best one only when strictly greater.  (Nobody else
        // touches the instance's best level during this launch; before the first item the
        // row is all zero and cannot win.)
        const int at = probe[(size_t)inst * max_items + q];
        if (at >= 0) {
            const int level_value = rows[((size_t)inst * 2 + (q & 1)) * row_len + at];
            if (level_value > st.best_value) {
                state[inst].best_value = level_value;
                state[inst].best_length = q;
                state[inst].best_remain = at;
            }
        }
    }
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
constexpr int kMaxItemsPerPass = 3; // temporal blocking depth of the persistent sweep
constexpr int kMinBlockSegs = 14;   // smallest block worth an extra level: one task per computing wavefront

typedef __attribute__((address_space(3))) int32_t lds_i32;
typedef const __attribute__((address_space(1))) int32_t global_ci32;

// Block hand-over barriers of sg_sweep_all: a loading wavefront arrives when its LDS-direct
// loads have landed, a computing wavefront when its LDS reads have (its row and keep stores
// stay in flight until the end of the item).  Asm, because the compiler puts a wait for all
// vector memory in front of every barrier it knows of once a kernel has LDS-direct loads.
__device__ __forceinline__ void barrier_after_loads() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void barrier_after_lds_reads() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// All offered items of one stage, one workgroup per instance.  The row is walked in
// ascending blocks of R segments (256 cells each); a ring of LDS segments holds the part
// of the old row the block needs (segment g in slot g % ring size), so that every old cell
// is fetched from global memory once and both operands of a cell come from LDS.
//
// Two kinds of pass over the row:
//  * one item: old row in buffer `cur`, new row into the other buffer.  The ring holds the
//    block being computed, the block being loaded and the cells up to w below:
//    2 R + ceil(w / 256) + 1 <= ring_segs.  Items too heavy for that read their shifted
//    operand from global memory (separate instantiation).
//  * g = 2 or 3 items (temporal blocking): the rows between the items exist only in LDS.
//    Ring 0 holds the old row (2 R + s0 segments), ring l the row after item l - 1
//    (R + sl + 1 segments), sl = ceil(wl / 256) + 1; per block, level l computes item l's
//    block from ring l into ring l + 1, and the last level stores it - into the buffer
//    being read, behind the loads - so a cell-update costs 1/g of the HBM traffic.
// A compute task is one segment: lane l covers cells seg*256 + 64 j + l, j = 0..3, so the
// v_cmp masks are the keep words of the segment.
__global__ void __launch_bounds__(kAllThreads)
sg_sweep_all(BatchArgs a, InstState *__restrict__ state, const int32_t *__restrict__ act, int32_t *rows,
             uint64_t *keep, int row_len, int keep_words, int max_items, int ring_segs,
             unsigned long long *streamed_cells)
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
    const int32_t *W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *V = a.values + (size_t)inst * a.item_stride;
    const int32_t *list = act + (size_t)inst * max_items;
    int32_t *const buf0 = rows + (size_t)inst * 2 * row_len;
    const std::true_type yes{};
    const std::false_type no{};

    // the first offered item sees an all-zero row: the ring is cleared once and not loaded
    for (int i = threadIdx.x; i < ring_segs * kSegCells; i += kAllThreads) ring[i] = 0;
    __syncthreads();

    // segments [lo, lo + n) of `src` -> ring slots slot_lo .. of a ring of rn segments at rbase
    auto load_segs = [&](const int32_t *src, int lo, int n, int rbase, int rn, int slot_lo) {
        for (int g = wave; g < n; g += kAllLoadWaves) {
            int slot = slot_lo + g;
            if (slot >= rn) slot -= rn;
            __builtin_amdgcn_global_load_lds((global_ci32 *)(src + (size_t)(lo + g) * kSegCells + lane * 4),
                                             (lds_i32 *)(ring + (size_t)(rbase + slot) * kSegCells), 16, 0, 0);
        }
    };

    // One task = one segment `seg`, held in slot `slot` of the source ring (rn segments at
    // segment offset rbase).  IN_RING: the shifted operand comes from the ring, else from
    // `src` in global memory.  KIND 0: the whole segment lies at or above w; 1: w falls
    // inside it (cells below w keep their value); 2: the whole segment lies below w (copied
    // through).  TO_LDS: the new cells go to slot `oslot` of the ring at obase, else to `dst`.
    auto task = [&](auto in_ring_tag, auto kind_tag, auto to_lds_tag, int rbase, int rn, int w, int v, int seg,
                    int slot, const int32_t *src, bool first, int32_t *dst, int obase, int oslot, uint64_t *kw) {
        constexpr bool IN_RING = decltype(in_ring_tag)::value;
        constexpr int KIND = decltype(kind_tag)::value;
        constexpr bool TO_LDS = decltype(to_lds_tag)::value;
        const int32_t *rg = ring + (size_t)rbase * kSegCells;
        const int rcells = rn * kSegCells;
        const int32_t *own = rg + (size_t)slot * kSegCells + lane;
        const int c0 = seg * kSegCells + lane;
        int cen[4], sh[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) cen[j] = own[j * 64];
        if (KIND != 2) {
            if (IN_RING) {
                // ring position of the segment's first cell minus w, brought into [0, rcells)
                int base = slot * kSegCells - w;
                base += base < 0 ? rcells : 0;
                if (base + kSegCells <= rcells) {
                    // the 256 shifted cells are contiguous in the ring: immediate offsets
                    const int32_t *shp = rg + base + lane;
#pragma unroll
                    for (int j = 0; j < 4; ++j) sh[j] = shp[j * 64];
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        unsigned o = (unsigned)(base + lane + j * 64);
                        o = min(o, o - (unsigned)rcells);  // wraps past the ring's end
                        sh[j] = rg[o];
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
        int32_t *lds_out = ring + (size_t)(obase + oslot) * kSegCells + lane;
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
            if (TO_LDS) lds_out[j * 64] = best;
            else dst[(size_t)c0 + j * 64] = best;
        }
        if (lane < 4) {
            unsigned long long wsel = 0;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (jj == lane) wsel = m[jj];
            kw[seg * 4 + lane] = wsel;
        }
    };
    // picks the KIND for the segment
    auto run_task = [&](auto in_ring_tag, auto to_lds_tag, int rbase, int rn, int w, int v, int seg, int slot,
                        const int32_t *src, bool first, int32_t *dst, int obase, int oslot, uint64_t *kw) {
        const int c_first = seg * kSegCells;
        if (c_first >= w)
            task(in_ring_tag, std::integral_constant<int, 0>{}, to_lds_tag, rbase, rn, w, v, seg, slot, src, first, dst,
                 obase, oslot, kw);
        else if (c_first + kSegCells > w)
            task(in_ring_tag, std::integral_constant<int, 1>{}, to_lds_tag, rbase, rn, w, v, seg, slot, src, first, dst,
                 obase, oslot, kw);
        else
            task(yes, std::integral_constant<int, 2>{}, to_lds_tag, rbase, rn, w, v, seg, slot, src, first, dst, obase,
                 oslot, kw);
    };

    int cur = 0;  // buffer holding the row before item q (all zeros for q == 0, wherever it is)
    int q = 0;
    int row_transfers = 0;  // rows read from plus rows written to global memory
    while (q < st.n_act) {
        const bool first = q == 0;
        row_transfers += first ? 1 : 2;  // every pass writes the row, all but the stage's first read it
        int32_t *src = buf0 + (size_t)cur * row_len;
        // the next up to kMaxItemsPerPass items: weight, value, reach in segments, keep row
        int w[kMaxItemsPerPass], v[kMaxItemsPerPass], sg[kMaxItemsPerPass];
        uint64_t *kw[kMaxItemsPerPass];
#pragma unroll
        for (int l = 0; l < kMaxItemsPerPass; ++l) {
            const int t = list[min(q + l, st.n_act - 1)];
            w[l] = W[t];
            v[l] = V[t];
            sg[l] = (w[l] + kSegCells - 1) / kSegCells + 1;  // segments the shifted operand reaches back
            kw[l] = keep + ((size_t)inst * max_items + t) * keep_words;
        }
        // as many items per pass as leave blocks of at least kMinBlockSegs segments:
        // (g + 1) R + sum of reaches + (g - 1) <= ring_segs
        int g = 1, R = 0;
        {
            int reach = sg[0];
#pragma unroll
            for (int l = 1; l < kMaxItemsPerPass; ++l) {
                reach += sg[l];
                const int r = (ring_segs - l - reach) / (l + 2);
                if (q + l < st.n_act && r >= kMinBlockSegs) { g = l + 1; R = r; }
            }
        }
        if (g >= 2) {
            // ---- g items per pass: ring 0 holds the old row (2 R + reach of item 0), ring l
            // the row after item l - 1 (R + reach of item l + 1); level l reads ring l and
            // writes ring l + 1, the last level stores to the buffer being read ------------
            int rbase[kMaxItemsPerPass], rn[kMaxItemsPerPass], slot[kMaxItemsPerPass];
            {
                int at = 0;
#pragma unroll
                for (int l = 0; l < kMaxItemsPerPass; ++l) {
                    rbase[l] = at;
                    rn[l] = l == 0 ? 2 * R + sg[0] : R + sg[l] + 1;
                    at += rn[l];
                    slot[l] = 0;  // lo % rn[l]
                }
            }
            if (loader) {
                if (!first) load_segs(src, 0, min(R, nseg), 0, rn[0], 0);
                barrier_after_loads();
            } else {
                barrier_after_lds_reads();
            }
            for (int lo = 0; lo < nseg; lo += R) {
                int slot_next[kMaxItemsPerPass];
#pragma unroll
                for (int l = 0; l < kMaxItemsPerPass; ++l) {
                    slot_next[l] = slot[l] + R;
                    if (slot_next[l] >= rn[l]) slot_next[l] -= rn[l];
                }
                const int ns = min(R, nseg - lo);
                if (loader) {
                    if (!first && lo + R < nseg) load_segs(src, lo + R, min(R, nseg - lo - R), 0, rn[0], slot_next[0]);
                    for (int l = 0; l + 1 < g; ++l) barrier_after_lds_reads();  // (levels of this block)
                    barrier_after_loads();  // the next block of the old row is in ring 0
                } else {
#pragma unroll
                    for (int l = 0; l < kMaxItemsPerPass; ++l) {
                        if (l < g) {
                            const bool last = l + 1 == g;
                            for (int i = wave - kAllLoadWaves; i < ns; i += kAllComputeWaves) {
                                int s_in = slot[l] + i;
                                if (s_in >= rn[l]) s_in -= rn[l];
                                if (last) {
                                    run_task(yes, no, rbase[l], rn[l], w[l], v[l], lo + i, s_in, src, first && l == 0, src, 0,
                                             0, kw[l]);
                                } else {
                                    int s_out = slot[l + 1 < kMaxItemsPerPass ? l + 1 : l] + i;
                                    const int rn_out = rn[l + 1 < kMaxItemsPerPass ? l + 1 : l];
                                    if (s_out >= rn_out) s_out -= rn_out;
                                    run_task(yes, yes, rbase[l], rn[l], w[l], v[l], lo + i, s_in, src, first && l == 0, src,
                                             rbase[l + 1 < kMaxItemsPerPass ? l + 1 : l], s_out, kw[l]);
                                }
                            }
                            barrier_after_lds_reads();  // level l of the block is complete
                        }
                    }
                }
#pragma unroll
                for (int l = 0; l < kMaxItemsPerPass; ++l) slot[l] = slot_next[l];
            }
            q += g;  // the new row replaced the old one in buffer `cur`
        } else {
            // ---- one item per pass --------------------------------------------------
            int32_t *dst = buf0 + (size_t)(cur ^ 1) * row_len;
            const int wA = w[0], vA = v[0], sA = sg[0];
            uint64_t *kwA = kw[0];
            const bool shifted_in_ring = sA + 2 <= ring_segs;
            const int R1 = max(1, (shifted_in_ring ? ring_segs - sA : ring_segs) / 2);
            if (loader) {
                if (!first) load_segs(src, 0, min(R1, nseg), 0, ring_segs, 0);
                barrier_after_loads();
            } else {
                barrier_after_lds_reads();
            }
            int slot_lo = 0;  // lo % ring_segs
            for (int lo = 0; lo < nseg; lo += R1) {
                int slot_next = slot_lo + R1;
                if (slot_next >= ring_segs) slot_next -= ring_segs;
                if (loader) {
                    if (!first && lo + R1 < nseg)
                        load_segs(src, lo + R1, min(R1, nseg - lo - R1), 0, ring_segs, slot_next);
                    barrier_after_loads();  // the next block is in the ring
                } else {
                    const int ns = min(R1, nseg - lo);
                    for (int i = wave - kAllLoadWaves; i < ns; i += kAllComputeWaves) {
                        int sl = slot_lo + i;
                        if (sl >= ring_segs) sl -= ring_segs;
                        if (shifted_in_ring)
                            run_task(yes, no, 0, ring_segs, wA, vA, lo + i, sl, src, first, dst, 0, 0, kwA);
                        else
                            run_task(no, no, 0, ring_segs, wA, vA, lo + i, sl, src, first, dst, 0, 0, kwA);
                    }
                    barrier_after_lds_reads();  // this block's slots may be reused
                }
                slot_lo = slot_next;
            }
            cur ^= 1;
            q += 1;
        }
        // the next pass reads what this one wrote (other wavefronts' cells included)
        __threadfence_block();
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        state[inst].buf = cur;
        if (streamed_cells) atomicAdd(streamed_cells, (unsigned long long)row_transfers * nseg * kSegCells);
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
    if (nact > 0) value = rows[((size_t)inst * 2 + (st->buf >= 0 ? st->buf : (nact & 1))) * row_len + C];
    int c = C, from = nact - 1;
    const bool levels = a.mode == DEFT_MODE_RECURSIVE;
    int length = nact;
    if (levels) {  // the whole list is the last level met; the walk starts at the best level's end
        if (value > st->best_value) { st->best_value = value; st->best_length = nact; st->best_remain = C; }
        value = st->best_value;
        length = st->best_length;
        from = length - 1;
        c = st->best_remain;
    }
    const int start = c;
    for (int q = from; q >= 0; --q) {
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
    a.knap_load[(size_t)inst * a.knap_stride + j] = start - c;
    if (levels) {  // slot 1 reports the level: items left off the list, its remaining time
        a.knap_value[(size_t)inst * a.knap_stride + 1] = a.n_items[inst] - length;
        a.knap_load[(size_t)inst * a.knap_stride + 1] = value > 0 ? start : 0;
    }
    st->total += value;
    a.total_value[inst] = st->total;
}

// Capacity sweep: one thread per (instance, capacity) reads the value at its capacity off the
// final row and walks the keep words back from (last offered item, that capacity); an item's
// output word collects the capacities at which it is taken.
__global__ void __launch_bounds__(64)
sg_traceback_caps(BatchArgs a, InstState *state, const int32_t *__restrict__ act, const int32_t *rows,
                  const uint64_t *keep, int row_len, int keep_words, int max_items)
{
    const int idx = blockIdx.x * 64 + threadIdx.x;
    const int inst = idx / a.knap_stride, j = idx % a.knap_stride;
    if (inst >= a.batch) return;
    const InstState *st = &state[inst];
    if (st->status != DEFT_OK || st->knap < 0 || j >= a.n_knapsacks[inst]) return;
    const int nact = st->n_act, C = a.capacities[(size_t)inst * a.knap_stride + j];
    const int32_t *W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *list = act + (size_t)inst * max_items;
    int value = 0;
    if (nact > 0) value = rows[((size_t)inst * 2 + (st->buf >= 0 ? st->buf : (nact & 1))) * row_len + C];
    int c = C;
    for (int q = nact - 1; q >= 0; --q) {
        const int t = list[q];
        const int w = W[t];
        if (w <= c) {
            const uint64_t word = keep[((size_t)inst * max_items + t) * keep_words + (c >> 6)];
            if ((word >> (c & 63)) & 1ull) {
                atomicOr(reinterpret_cast<unsigned int *>(&a.assignment[(size_t)inst * a.item_stride + t]), 1u << j);
                c -= w;
            }
        }
    }
    a.knap_value[(size_t)inst * a.knap_stride + j] = value;
    a.knap_load[(size_t)inst * a.knap_stride + j] = C - c;
    if (C == st->cap) a.total_value[inst] = value;  // the largest capacity (equal ones agree)
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
                                 2 * align256((size_t)max_batch * max_items * 4) +
                                 align256((size_t)max_batch * sizeof(InstState)));
}

hipError_t seq_global_prepare(const SeqGlobalPlan &p)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&sg_sweep_all),
                               hipFuncAttributeMaxDynamicSharedMemorySize, p.lds_bytes);
}

hipError_t seq_global_launch(const SeqGlobalPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                             Profiler *prof, unsigned long long *streamed_cells)
{
    const Scratch s = carve(p, scratch, p.max_batch);
    hipLaunchKernelGGL(sg_init, dim3(a.batch), dim3(kThreads), 0, st, a, s.state);
    const int tiles = p.row_len / kTileCells + (p.row_len % kTileCells ? 1 : 0);
    const bool caps_sweep = a.mode == DEFT_MODE_CAPACITY_SWEEP, levels = a.mode == DEFT_MODE_RECURSIVE;
    const int stages = caps_sweep || levels ? 1 : a.knap_stride;
    for (int stage = 0; stage < stages; ++stage) {
        if (levels)
            hipLaunchKernelGGL(sg_levels_setup, dim3(a.batch), dim3(64), 0, st, a, s.state, s.act, s.probe, p.max_items);
        else
            hipLaunchKernelGGL(sg_stage_setup, dim3(a.batch), dim3(64), 0, st, a, stage, s.state, s.act, p.max_items);
        // Algorithm 1 reads one cell of every intermediate row, so it takes the sweeps that
        // leave each of them in global memory (one launch per item)
        if (a.batch >= p.persistent_min_batch && !levels) {
            if (prof) prof->sweep_begin(st);
            hipLaunchKernelGGL(sg_sweep_all, dim3((unsigned)a.batch), dim3(kAllThreads), (size_t)p.lds_bytes, st, a,
                               s.state, s.act, s.rows, s.keep, p.row_len, p.keep_words, p.max_items, p.ring_segs,
                               prof ? streamed_cells : nullptr);
            if (prof) prof->sweep_end(st);
        } else {
            for (int q = 0; q < a.item_stride; ++q) {
                if (prof) prof->sweep_begin(st);
                hipLaunchKernelGGL(sg_sweep, dim3((unsigned)tiles * (unsigned)a.batch), dim3(kThreads), 0, st, a, q,
                                   s.state, s.act, s.probe, s.rows, s.keep, p.row_len, p.keep_words, p.max_items,
                                   tiles);
                if (prof) prof->sweep_end(st);
            }
        }
        if (caps_sweep) {
            const unsigned walks = (unsigned)a.batch * (unsigned)a.knap_stride;
            hipLaunchKernelGGL(sg_traceback_caps, dim3((walks + 63) / 64), dim3(64), 0, st, a, s.state, s.act, s.rows,
                               s.keep, p.row_len, p.keep_words, p.max_items);
        } else {
            hipLaunchKernelGGL(sg_traceback, dim3((a.batch + 63) / 64), dim3(64), 0, st, a, s.state, s.act,
                               s.rows, s.keep, p.row_len, p.keep_words, p.max_items);
        }
    }
    return hipGetLastError();
}

}  // namespace deft
