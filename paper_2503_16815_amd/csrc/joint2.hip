// Joint two-link solve (Sec. III.C, Problem 2 with one weight per link).  The
// (C1+1) x (C2+1) table does not fit LDS, so it lives in global memory (two
// copies, item q reads copy q & 1 and writes the other) and streams through an
// LDS window once per item:
//   new[a][b] = max(old[a][b], old[a - w0][b] + v, old[a][b - w1] + v)
// tested in that order, each replacing the incumbent only when strictly
// greater.  One workgroup owns an instance for all its items.  It walks the
// rows in ascending blocks; each old row is fetched from global memory exactly
// once, as the block's own rows, into a ring of LDS rows, where it stays until
// the rows w0 above it have used it as their shifted operand; the b-shifted
// operand comes from the same LDS row.  Per cell: 4 B read + 4 B written +
// 1/4 B of choice bits to HBM, 4 B written + 12 B read in LDS.
// The 2-bit choice is stored as two bit planes (took link 0 / took link 1),
// one 64-bit ballot word per 64 consecutive b.  The first item reads zeros
// instead of a table.
#include <limits.h>

#include <type_traits>

#include "instance_check.h"

namespace deft {

namespace {

constexpr int kThreads = 256;

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

constexpr int kSweepThreads = 1024;  // one workgroup per instance
constexpr int kSweepWaves = kSweepThreads / 64;
constexpr int kLoadWaves = 3;        // wavefronts that only move old rows from global memory into LDS
constexpr int kComputeWaves = kSweepWaves - kLoadWaves;

// Block hand-over barriers.  A loading wavefront arrives when its LDS-direct loads have
// landed (they count as vector memory); a computing wavefront arrives when its LDS reads
// have, while its table stores stay in flight (they are awaited once, at the end of the
// item).  Written as asm because the compiler, seeing LDS-direct loads in the kernel, puts
// a wait for all vector memory in front of every barrier it knows about.
__device__ __forceinline__ void barrier_after_loads()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ void barrier_after_lds_reads()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

typedef __attribute__((address_space(3))) int32_t lds_i32;
typedef const __attribute__((address_space(1))) int32_t global_ci32;

// Roles: the first kLoadWaves wavefronts copy the next block's old rows from global
// memory straight into the LDS ring (no registers in between, so dozens of 256-byte
// loads are in flight per wavefront); the others compute the current block from the ring
// and store the new rows and the choice bits, and never wait on memory.  One barrier per
// block hands the freshly loaded block over.
// A compute task is one row x 256 columns: lane l covers columns tile*256 + 64 j + l,
// j = 0..3, so every global and LDS access of a wavefront is 64 consecutive words and the
// ballot over j is the choice word of segment tile*4 + j.
__global__ void __launch_bounds__(kSweepThreads)
jt_sweep_all(BatchArgs a, const InstState *__restrict__ state, int32_t *tab, uint64_t *choice, int rows, int pitch,
             int max_items, int ring_rows, int lds_pitch)
{
    extern __shared__ __align__(16) int32_t ring[];  // [ring_rows][lds_pitch], row a lives in slot a % ring_rows
    const int inst = blockIdx.x;
    const InstState st = state[inst];
    if (st.status != DEFT_OK || st.n <= 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool loader = wave < kLoadWaves;
    const int segs = pitch / 64;
    const int ncol = st.c2 + 1, nrow = st.c1 + 1;
    const int ntile = (ncol + 255) / 256;
    // A last tile of a single column (capacities that are multiples of 256: C2 + 1 columns)
    // is not worth a task of its own: the task of the tile before it takes the column along
    // in one lane.
    const bool lone_column = ncol > 256 && (ncol & 255) == 1;
    const int ntile_tasks = lone_column ? ntile - 1 : ntile;
    const size_t tsz = (size_t)rows * pitch;
    const int32_t *W0 = a.weights + (size_t)inst * 2 * a.item_stride;
    const int32_t *W1 = W0 + a.item_stride;
    const int32_t *V = a.values + (size_t)inst * a.item_stride;

    // the first item sees an all-zero table: the ring is cleared once and not loaded
    for (int i = threadIdx.x; i < ring_rows * lds_pitch; i += kSweepThreads) ring[i] = 0;
    __syncthreads();

    for (int q = 0; q < st.n; ++q) {
        const int w0 = W0[q], w1 = W1[q], v = V[q];
        const int32_t *__restrict__ src = tab + ((size_t)inst * 2 + (q & 1)) * tsz;
        int32_t *__restrict__ dst = tab + ((size_t)inst * 2 + ((q & 1) ^ 1)) * tsz;
        uint64_t *ch = choice + ((size_t)inst * max_items + q) * ((size_t)rows * segs * 2);
        const bool first = q == 0;
        // The ring holds the block being computed, the next block being loaded and the w0
        // rows below the current block: 2 R + w0 <= ring_rows.  Heavier items read their
        // row-shifted operand from global memory instead.
        const bool shifted_in_ring = 2 + w0 <= ring_rows;
        const int R = max(1, (shifted_in_ring ? ring_rows - w0 : ring_rows) / 2);

        // rows [lo, lo + R) of the old table -> ring; slot_lo = lo % ring_rows.  The
        // (row, segment) pairs are dealt round-robin to the loading wavefronts.
        auto load_rows = [&](int lo, int slot_lo) {
            if (first) return;
            const int nr = min(R, nrow - lo);
            // whole rows, dealt round-robin to the loading wavefronts; a row is ntile parts of
            // 256 columns, 16 bytes per lane.  Kept lean: a loading wavefront shares its SIMD with
            // computing ones, so the instructions it spends per load bound the rate it loads at.
            for (int r = wave; r < nr; r += kLoadWaves) {
                int slot = slot_lo + r;
                if (slot >= ring_rows) slot -= ring_rows;
                const int32_t *g = src + (size_t)(lo + r) * pitch + lane * 4;
                int32_t *l = ring + (size_t)slot * lds_pitch;
                // a lane's four columns may run past the instance's last column, never past the
                // row pitch of the table or of the ring (both are multiples of four)
                for (int part = 0; part < ntile; ++part) {
                    if (part * 256 + lane * 4 < ncol)
                        __builtin_amdgcn_global_load_lds((global_ci32 *)(g + part * 256), (lds_i32 *)(l + part * 256), 16, 0, 0);
                }
            }
        };

        if (loader) {
            load_rows(0, 0);
            barrier_after_loads();
        } else {
            barrier_after_lds_reads();
        }
        int slot_a0 = 0;  // a0 % ring_rows
        for (int a0 = 0; a0 < nrow; a0 += R) {
            int slot_next = slot_a0 + R;
            if (slot_next >= ring_rows) slot_next -= ring_rows;
            if (loader) {
                if (a0 + R < nrow) load_rows(a0 + R, slot_next);
                barrier_after_loads();  // the next block is in the ring
            } else {
                // One task.  IN_RING: the row-shifted operand comes from the ring; otherwise
                // (items heavier than the ring allows) from global memory, which makes every
                // task wait on vector memory: kept apart so that the common path never does.
                // MASK_B: some column of the tile lies below w1 and must not take link 1.
                // The first item needs no special case: the ring holds zeros while it runs.
                // HAS0: the row has a row-shifted operand (ar >= w0).  FULL: all four 64-column
                // segments of the tile exist and no column needs clamping (straight-line code).
                auto task = [&](auto in_ring_tag, auto mask_b_tag, auto has0_tag, auto full_tag, int ar, int slot,
                                int tile, bool with_lone_column) {
                    constexpr bool IN_RING = decltype(in_ring_tag)::value;
                    constexpr bool MASK_B = decltype(mask_b_tag)::value;
                    constexpr bool has0 = decltype(has0_tag)::value;
                    constexpr bool FULL = decltype(full_tag)::value;
                    const int32_t *own_row = ring + (size_t)slot * lds_pitch;
                    int sh_slot = slot - w0;  // only used when w0 < ring_rows
                    if (sh_slot < 0) sh_slot += ring_rows;
                    const int32_t *sh_row = ring + (size_t)(IN_RING ? sh_slot : 0) * lds_pitch;
                    const int col0 = tile * 256 + lane;
                    const int nj = FULL ? 4 : min(4, (ncol - tile * 256 + 63) >> 6);  // segments of the tile that exist
                    int32_t *out = dst + (size_t)ar * pitch + col0;
                    int cen[4], sh[4], bs[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (j < nj) {
                            const int col = FULL ? col0 + j * 64 : min(col0 + j * 64, ncol - 1);
                            const int idx = col - w1;
                            cen[j] = own_row[col];
                            bs[j] = own_row[MASK_B ? max(idx, 0) : idx];
                            if (has0) {
                                if (IN_RING) sh[j] = sh_row[col];
                                else sh[j] = first ? 0 : src[(size_t)(ar - w0) * pitch + col];
                            }
                        }
                    }
                    unsigned long long m0[4], m1[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        m0[j] = 0;
                        m1[j] = 0;
                        if (j < nj) {
                            const int col = col0 + j * 64;
                            int best = cen[j];
                            if (has0) {
                                const int cand0 = sh[j] + v;
                                m0[j] = __ballot(cand0 > best);
                                best = max(best, cand0);
                            }
                            int cand1 = bs[j] + v;
                            if (MASK_B) cand1 = col < w1 ? INT_MIN : cand1;
                            m1[j] = __ballot(cand1 > best);
                            best = max(best, cand1);
                            m0[j] &= ~m1[j];
                            // (streaming store: the new table is next read a whole table's worth of
                            // traffic per compute unit later; measured 9.1 -> 8.4 ms on the two-link batch)
                            if (FULL || col < ncol) __builtin_nontemporal_store(best, &out[j * 64]);
                        }
                    }
                    // lanes 0..7 store the eight ballot words of the tile's four segments (bits of
                    // columns past the instance's last one are never looked at)
                    const int j = lane >> 1;
                    if (lane < 8 && j < nj) {
                        unsigned long long wsel = 0;
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj)
                            if (jj == j) wsel = (lane & 1) ? m1[jj] : m0[jj];
                        ch[((size_t)ar * segs + tile * 4 + j) * 2 + (lane & 1)] = wsel;
                    }
                    if (with_lone_column && lane == 0) {  // the row's last column, same tests in the same order
                        const int col = ncol - 1;
                        int best = own_row[col];
                        unsigned long long t0 = 0, t1 = 0;
                        if (has0) {
                            const int cand0 =
                                (IN_RING ? sh_row[col] : (first ? 0 : src[(size_t)(ar - w0) * pitch + col])) + v;
                            t0 = cand0 > best;
                            best = max(best, cand0);
                        }
                        const int cand1 = col >= w1 ? own_row[col - w1] + v : INT_MIN;
                        t1 = cand1 > best;
                        best = max(best, cand1);
                        t0 &= ~t1;
                        dst[(size_t)ar * pitch + col] = best;
                        ch[((size_t)ar * segs + (col >> 6)) * 2] = t0;
                        ch[((size_t)ar * segs + (col >> 6)) * 2 + 1] = t1;
                    }
                };
                const int nr = min(R, nrow - a0);
                int r = 0, tile = wave - kLoadWaves;
                while (true) {
                    while (tile >= ntile_tasks) { tile -= ntile_tasks; ++r; }
                    if (r >= nr) break;
                    int slot = slot_a0 + r;
                    if (slot >= ring_rows) slot -= ring_rows;
                    const bool mask_b = tile * 256 < w1, has0 = a0 + r >= w0, full = tile * 256 + 256 <= ncol;
                    const bool lone = lone_column && tile == ntile_tasks - 1;
                    const std::true_type yes{};
                    const std::false_type no{};
                    const int ar = a0 + r;
                    auto run = [&](auto in_ring, auto mask, auto has, auto is_full) {
                        task(in_ring, mask, has, is_full, ar, slot, tile, lone);
                    };
                    if (!shifted_in_ring || !full) {  // rare shapes: one general instance each
                        if (!shifted_in_ring) {
                            if (has0) run(no, yes, yes, no); else run(no, yes, no, no);
                        } else {
                            if (has0) run(yes, yes, yes, no); else run(yes, yes, no, no);
                        }
                    } else if (has0) {
                        if (mask_b) run(yes, yes, yes, yes); else run(yes, no, yes, yes);
                    } else {
                        if (mask_b) run(yes, yes, no, yes); else run(yes, no, no, yes);
                    }
                    tile += kComputeWaves;
                }
                barrier_after_lds_reads();  // this block's slots may be reused
            }
            slot_a0 = slot_next;
        }
        // the next item reads what this one wrote (other wavefronts' rows included)
        __threadfence_block();
        __syncthreads();
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

void joint_plan(int32_t max_c1, int32_t max_c2, int32_t max_items, int32_t max_batch, int32_t lds_per_wg_bytes,
                JointPlan *p)
{
    p->rows = max_c1 + 1;
    p->pitch = (max_c2 + 1 + 63) / 64 * 64;
    p->lds_pitch = (max_c2 + 1 + 3) / 4 * 4;  // rows stay 16-byte aligned for the 16-byte LDS-direct loads
    // as many LDS rows as fit, but no more than the table has (plus one block)
    int64_t ring = (int64_t)lds_per_wg_bytes / ((int64_t)p->lds_pitch * 4);
    if (ring > p->rows) ring = p->rows;
    if (ring < 2) ring = 2;
    p->ring_rows = (int32_t)ring;
    p->lds_bytes = (int32_t)(ring * p->lds_pitch * 4);
    p->max_items = max_items;
    p->max_batch = max_batch;
    p->scratch_bytes = (int64_t)(align256((size_t)max_batch * 2 * p->rows * p->pitch * 4) +
                                 align256((size_t)max_batch * max_items * p->rows * (p->pitch / 64) * 16) +
                                 align256((size_t)max_batch * sizeof(InstState)));
}

hipError_t joint_prepare(const JointPlan &p)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&jt_sweep_all),
                               hipFuncAttributeMaxDynamicSharedMemorySize, p.lds_bytes);
}

hipError_t joint_launch(const JointPlan &p, const BatchArgs &a, void *scratch, hipStream_t st, Profiler *prof)
{
    const Scratch s = carve(p, scratch);
    hipLaunchKernelGGL(jt_init, dim3(a.batch), dim3(kThreads), 0, st, a, s.state);
    if (prof) prof->sweep_begin(st);
    hipLaunchKernelGGL(jt_sweep_all, dim3((unsigned)a.batch), dim3(kSweepThreads), (size_t)p.lds_bytes, st, a, s.state,
                       s.tab, s.choice, p.rows, p.pitch, p.max_items, p.ring_rows, p.lds_pitch);
    if (prof) prof->sweep_end(st);
    hipLaunchKernelGGL(jt_traceback, dim3((a.batch + 63) / 64), dim3(64), 0, st, a, s.state, s.tab, s.choice,
                       p.rows, p.pitch, p.max_items);
    return hipGetLastError();
}

}  // namespace deft
