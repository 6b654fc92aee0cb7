// Sequential multiple-knapsack solve with the capacity row resident in LDS.
//
// One launch solves every stage of every instance (Sec. III.B: Problem 1 per
// window, windows filled one after the other).  An instance is owned by T
// lanes.  Cell c of the row lives in lane (c mod T), register slot (c div T),
// and a copy lives in LDS so that the shifted operand row[c - w] can be read
// by whichever lane needs it.  Per offered item:
//   phase A  every lane reads row[c - w] for its cells (LDS, 4 B/cell) and, as
//            the values arrive, computes cand = row[c - w] + v, take = cand >
//            row[c], row[c] = max(row[c], cand) in registers; the reads run a
//            fixed number of slots ahead of the arithmetic
//   barrier  (every lane has read the old row)
//   phase B  the new cells are written back (LDS, 4 B/cell); the take bits, one
//            32-bit word per 32 register slots, go to the keep table (HBM,
//            1/8 B/cell)
//   barrier  (the new row is visible)
// The textbook reverse sweep (c from C down to w) exists to read old values
// only; reading everything before the first barrier gives the same result.
// Cells below w must not change.  A guard zone of 128 or 256 cells holding
// INT_MIN (which can never win) sits below the row: for w <= guard size every
// lane simply reads row[c - w], landing in the guard when c < w.  Heavier items
// clamp each read index into the guard.
// The write-back uses ds_write_addtid_b32 (address = M0 + immediate + 4 * lane),
// which ships no address and runs at twice the rate of ds_write_b32 (rows longer
// than 64 KB through a second M0 base); the reads are ordinary loads, so the
// compiler tracks their completion itself.
//
// After the last item of a stage one wavefront traces the selection back from
// (last swept item, C) through the keep words just written and marks the chosen
// items, which the next stage then leaves out.
//
// Not every stage is swept: the first wavefront settles stages that are offered
// nothing, whose offered items all fit together, or that are offered at most
// six items, and where every value equals its weight a sweep ends as soon as
// every sum up to C can be reached.
//
// This header holds the kernel and its launcher as templates; seq_lds.hip instantiates
// them for the sequential mode and seq_lds_rec.hip for Algorithm 1 (REC = true), so the
// two sets of kernels compile side by side.
#pragma once

#include <limits.h>
#include <stdlib.h>

#include <type_traits>

#include "kernels.h"

namespace deft {

namespace {


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

// Makes what the lanes of the instance wrote to global memory (keep words, item
// lists) visible to its other lanes.  All of them run on one compute unit and share its
// vector L1, so workgroup scope is enough, for the fence and for the reads that follow it.
// A wider scope would write back and invalidate L2 at every call.
template <int T>
__device__ __forceinline__ void global_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if constexpr (T == 64) {
        __builtin_amdgcn_wave_barrier();
    } else {
        __builtin_amdgcn_s_barrier();
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Sum / maximum over the 64 lanes of a wavefront whose lanes are all active, the result in
// every lane.  Data-parallel primitives only (two exchanges inside each group of four
// lanes, two rotations inside each row of sixteen, then the four row results are read out):
// no LDS access, whose latency under the sweeps of the neighbouring workgroups is what the
// serial wavefront would otherwise wait for, several times per stage.
template <class Op>
__device__ __forceinline__ int wave_reduce(int x, Op op)
{
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0x124, 0xf, 0xf, false));  // row_ror:4
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0x128, 0xf, 0xf, false));  // row_ror:8
    return op(op(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
              op(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}
// Suffix sums over the wavefront (all lanes active): lane l gets x[l] + x[l+1] + ... + x[63].
// Shifts inside each row of sixteen lanes (zeros come in from beyond the row), then the totals
// of the rows above are added in.
__device__ __forceinline__ int wave_suffix_sum(int x, int lane)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x101, 0xf, 0xf, true);  // row_shl:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x102, 0xf, 0xf, true);  // row_shl:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x104, 0xf, 0xf, true);  // row_shl:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x108, 0xf, 0xf, true);  // row_shl:8
    const int t1 = __builtin_amdgcn_readlane(x, 16), t2 = __builtin_amdgcn_readlane(x, 32),
              t3 = __builtin_amdgcn_readlane(x, 48);
    return x + (lane < 16 ? t1 : 0) + (lane < 32 ? t2 : 0) + (lane < 48 ? t3 : 0);
}
__device__ __forceinline__ int wave_sum(int x) { return wave_reduce(x, [](int a, int b) { return a + b; }); }
__device__ __forceinline__ int wave_max(int x) { return wave_reduce(x, [](int a, int b) { return max(a, b); }); }

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

typedef __attribute__((address_space(3))) int32_t lds_i32;
// One offered item as the sweep and the traceback see it.
struct __attribute__((aligned(16))) OfferedItem {
    int32_t w, v, index, pad;
};
// Reads the first or second half of a list entry.  The lists (and the keep words) are
// written and read inside one launch by wavefronts of one workgroup, which share a compute
// unit and its vector L1: workgroup scope is all the ordering these reads need (after
// global_sync's release, barrier and acquire at the same scope).  A wider scope makes every
// such read go past the L2 of its chip to the memory side, which the walk's chain of
// dependent reads pays for round by round.  The scalar cache is not a way to read them: it
// can still hold a line from an earlier launch.
__device__ __forceinline__ int2 load_item_wv(const OfferedItem *e)
{
    const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(e), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_WORKGROUP);
    return make_int2((int)(uint32_t)u, (int)(uint32_t)(u >> 32));
}
__device__ __forceinline__ int load_item_index(const OfferedItem *e)
{
    return __hip_atomic_load(&e->index, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ int load_item_pad(const OfferedItem *e)
{
    return __hip_atomic_load(&e->pad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// Algorithm 1 (REC kernels): the best level seen so far.  A level is a prefix of the
// list (its length) solved with the remaining time that is left once the items behind
// the prefix have been taken off the list.
struct BestLevel {
    int value, length, remain;
};
// The same pointer in every lane of the wavefront: says so to the compiler, which then
// keeps it in scalar registers and addresses memory as scalar base + lane offset.
template <class P>
__device__ __forceinline__ P *uniform_ptr(P *p)
{
    const uintptr_t v = (uintptr_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    // rebuilt as a global-memory pointer, so that accesses stay global_* instructions
    typedef P __attribute__((address_space(1))) GlobalP;
    return (P *)(GlobalP *)(((uintptr_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_offset(int32_t *p)
{
    return (uint32_t)(uintptr_t)(lds_i32 *)p;
}

// LDS write addressed as M0 + OFF + 4 * lane.  M0 is an operand the compiler
// materialises and keeps across consecutive statements that use the same value.
// The hardware needs one wait state between a scalar write of M0 and an add-TID
// access, which the compiler's hazard pass does not know to apply to inline asm:
// m0_settle() supplies it and must precede the first add-TID access of a run.
// The compiler does not track these accesses either, so a run ends with an
// explicit s_waitcnt lgkmcnt(0) before the barrier that publishes it.
template <int OFF>
__device__ __forceinline__ void write_addtid(int m0, int d)
{
    asm volatile("ds_write_addtid_b32 %0 offset:%2" ::"v"(d), "{m0}"(m0), "n"(OFF) : "memory");
}
__device__ __forceinline__ void m0_settle(int m0) { asm volatile("s_nop 0" ::"{m0}"(m0) : "memory"); }
// Calls f(integral_constant<int, k>) for k = K0 down to 0 (compile-time indices for
// the immediate offsets of the add-TID writes).
template <int K0>
struct SlotsDown {
    template <class F>
    static __device__ __forceinline__ void all(F &&f)
    {
        f(std::integral_constant<int, K0>{});
        if constexpr (K0 > 0) SlotsDown<K0 - 1>::all(f);
    }
};
// Calls f(integral_constant<int, k>) for k = HI down to LO.
template <int HI, int LO>
struct SlotsDownTo {
    template <class F>
    static __device__ __forceinline__ void all(F &&f)
    {
        f(std::integral_constant<int, HI>{});
        if constexpr (HI > LO) SlotsDownTo<HI - 1, LO>::all(f);
    }
};
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// acc |= 1 << bit on the scalar unit (acc is the same in every lane; written this way the
// compiler keeps it in a scalar register instead of spending vector instructions on it).
__device__ __forceinline__ void scalar_set_bit(uint32_t &acc, int bit)
{
    uint32_t a = (uint32_t)__builtin_amdgcn_readfirstlane((int)acc);
    asm("s_bitset1_b32 %0, %1" : "+s"(a) : "s"(__builtin_amdgcn_readfirstlane(bit)));
    acc = a;
}

// LDS of one instance: [8 ints of scratch][guard_cells - 8 ints of INT_MIN][row_cells].
// The scratch words are the lowest cells of the guard zone; an item counts as light
// only if it cannot reach them (w <= guard_cells - 8).
struct LdsLayout {
    int32_t guard_cells, row_cells, ints_per_inst;
};
constexpr int kMiscInts = 8;
// Stages that are offered at most this many items are settled by enumeration of their subsets.
constexpr int kEnumItems = 6;
// Second M0 base of the add-TID write-back, in bytes above the first.
constexpr int kSecondBase = 60416;

// All offered items of one stage, for a row of NB register slots per lane (NB is a
// compile-time multiple of the chunk size, so the code is straight-line per item).
// Slots 0 .. NB-1 cover cells 0 .. NB*T - 1 >= C; the cells above C are swept along and
// never read back.
//
// REC (Algorithm 1): entry q of the list also carries, in `pad`, the remaining time P_q of
// the level made of the items before q (-1 if that is negative).  The row after items
// 0 .. q-1 is the DP row of exactly that level, so its answer is row[P_q]: one more LDS
// read per item, taken while item q reads the row.  Levels are met deepest first and a
// shallower one replaces the incumbent only when strictly greater, as the recursion does
// on its way back up.
//
// VEQW, sequential mode: once cell C holds its own index (the capacity itself can be
// reached: the kept value row[C] - C is 0) the stage's value is final, and no later item is
// taken at C (a take needs a strict improvement), so the walk back from C passes every later
// item and only ever reads keep rows up to here: the sweep ends there.  Checked after every
// eighth item (every second one of a list of at most 64), between two items: the wavefront
// that owns cell C stores the check's tag in `unfinished` while the cell is short of C, and
// after a barrier everyone looks at it.  Algorithm 1 (`levels`) ends its sweep the same way
// and settles the levels it has not met (settle_levels below); the capacity sweep, which
// reads the row at other cells as well, goes through the whole list.
// Returns the number of items swept (the keep rows beyond were never written).
template <int T, int NB, int G, int NW, bool ADDTID, bool VEQW, bool REC, bool SKIP_UNCHANGED>
__device__ __forceinline__ int sweep_stage(int32_t *row, uint32_t row_off, int light_max, int tid, int nact,
                                            const OfferedItem *list, uint32_t *kp, unsigned long long &nzm,
                                            BestLevel &best, int C, int32_t *unfinished, bool levels)
{
    constexpr bool STOP_WHEN_FULL = VEQW;  // (REC: Algorithm 1 only, see settle_levels)
    // short lists: after every second item, else every eighth; never for the capacity sweep,
    // which reads the row below C as well
    const int check_mask = REC && !levels ? INT_MAX : nact <= 64 ? 1 : 7;
    // What follows from the lane index alone (a slot's initial value and LDS address, for every
    // slot count instantiated) is cheap to compute here; left visible to the compiler it is all
    // computed at kernel entry instead, parked in scratch memory and fetched back per stage.
    asm volatile("" : "+v"(tid));
    constexpr int D = NB < 12 ? NB : 12;  // slots the reads run ahead of the arithmetic (<= 15 LDS ops in flight)
    const int wave_first = tid & ~63;     // first lane of this wavefront within the instance
    // VEQW (every value equals its weight, the paper's Problem 1): the row is kept as
    // row[c] - c, which turns row[c-w] + w into a plain copy of the shifted operand and
    // saves the add; comparisons and hence take bits are unchanged.
    // Each wavefront holds 64 list entries in two registers (lane l: entry 64 c + l) and
    // fetches the next 64 while it works through these, so an item's weight and value are
    // two lane reads and the sweep waits on vector memory once per 64 items.
    const int lane = tid & 63;
    auto load_chunk = [&](int first) {
        return first + lane < nact ? load_item_wv(list + first + lane) : make_int2(0, 0);
    };
    auto load_probe_chunk = [&](int first) {
        return REC && first + lane < nact ? load_item_pad(list + first + lane) : -1;
    };
    int2 cur = load_chunk(0);
    int cur_p = load_probe_chunk(0);
    int own[NB];
#pragma unroll
    for (int k = 0; k < NB; ++k) {
        own[k] = VEQW ? -(k * T + tid) : 0;
        row[k * T + tid] = own[k];
    }
    lds_sync<T>();  // initial row visible to every lane

    const int m0w = uniform((int)row_off + wave_first * 4);
    const int m0w2 = m0w + kSecondBase;
    uint32_t nz_acc = 0;  // flags of the items since the last multiple of 32 (the same in every lane)
    auto hand_over = [&](int q) {  // q: the last item whose flag nz_acc holds
        if ((tid & 63) == (q >> 6)) nzm |= (unsigned long long)nz_acc << (q & 32);
        nz_acc = 0;
    };
    // One item.  HEAVY is a compile-time flag and the two kinds run in separate loops
    // below, so that the loop over the (common) light items has a single body and the
    // compiler keeps every cell in one register across iterations.
    auto item = [&](auto heavy_tag, int q, int w, int v) {
        constexpr bool HEAVY = decltype(heavy_tag)::value;
        uint32_t bits[NW];
#pragma unroll
        for (int x = 0; x < NW; ++x) bits[x] = 0;
        int rd[NB];
        auto update = [&](int k) {
            const int cand = VEQW ? rd[k] : rd[k] + v;
            bits[k >> 5] = shift_in_take(bits[k >> 5], cand, own[k]);  // slot k ends at bit k % 32
            own[k] = max(own[k], cand);
        };
        int probe_at = -1, probe = 0;
        if constexpr (REC) {
            probe_at = __builtin_amdgcn_readlane(cur_p, q & 63);
            probe = row[max(probe_at, 0)];
        }
        const int idx = tid - w;
        const int32_t *src = row + idx;
        // light item: every lane reads row[c - w]; c < w lands in the guard.  Heavy item
        // (rare): each lane clamps its read index into the guard, so cells below w read
        // INT_MIN wherever they are.
        auto read = [&](int k) { return HEAVY ? row[max(idx + k * T, -1)] : src[k * T]; };
        // The order of phase A is pinned: D slots of reads up front, then two slots of
        // arithmetic for every two further reads.
#pragma unroll
        for (int k = NB - 1; k >= NB - D; --k) rd[k] = read(k);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = NB - 1; k >= 0; k -= 2) {
            update(k);
            if (k >= 1) update(k - 1);
            if (k - D >= 0) rd[k - D] = read(k - D);
            if (k - D - 1 >= 0) rd[k - D - 1] = read(k - D - 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (REC) {
            const int level_value = uniform(probe) + (VEQW ? probe_at : 0);
            if (probe_at >= 0 && level_value > best.value) best = BestLevel{level_value, q, probe_at};
        }
        // which groups of slots changed anywhere in this wavefront: one ballot per group over
        // the group's bits of the take word
        constexpr int kGroup = T == 768 ? 20 : 16;
        constexpr int kGroups = (NB - 1) / kGroup + 1;
        bool group_changed[kGroups];
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int lo = g * kGroup, hi = lo + kGroup - 1 < NB - 1 ? lo + kGroup - 1 : NB - 1;
            const uint32_t mask = (uint32_t)(((1ull << (hi - lo + 1)) - 1ull) << (lo & 31));
            group_changed[g] = !SKIP_UNCHANGED || __builtin_amdgcn_ballot_w64((bits[lo >> 5] & mask) != 0) != 0ull;
        }
        lds_sync<T>();  // every lane has read the old row

        if constexpr (ADDTID) {
            // The instruction's offset and M0's base are 16 bits each: slots whose byte
            // offset within the row is above 65535 go through a second base, kSecondBase
            // further up (both bases stay below 65536: the row starts within 5 KB of the
            // start of LDS); slots beyond the reach of that one are written with addresses.
            // A slot in which none of this wavefront's 64 cells took the item holds what LDS
            // already has.  Slots are written back in groups of sixteen, and a group only if one
            // of its slots changed (measured on the ResNet shape: 2.73 ms per step with groups of
            // sixteen, 2.76 with eight, 2.82 with four, 2.96 with a branch per slot, 2.88 when
            // everything is written).
            // (Twenty for 768 lanes, so that a group's slots all lie on one side of kSecondBase.)
            SlotsDown<(NB - 1) / kGroup>::all([&](auto gc) {
                constexpr int lo = gc.value * kGroup;
                constexpr int hi = lo + kGroup - 1 < NB - 1 ? lo + kGroup - 1 : NB - 1;
                static_assert((lo >> 5) == (hi >> 5), "a group's take bits sit in one word");
                static_assert(hi * T * 4 <= 65535 || lo * T * 4 >= kSecondBase, "a group does not straddle the M0 bases");
                if (group_changed[gc.value]) {
                    if constexpr (hi * T * 4 <= 65535) {
                        m0_settle(m0w);
                        SlotsDownTo<hi, lo>::all([&](auto kc) { write_addtid<kc.value * T * 4>(m0w, own[kc.value]); });
                    } else if constexpr (hi * T * 4 - kSecondBase <= 65535) {
                        m0_settle(m0w2);
                        SlotsDownTo<hi, lo>::all(
                            [&](auto kc) { write_addtid<kc.value * T * 4 - kSecondBase>(m0w2, own[kc.value]); });
                    } else {
                        SlotsDownTo<hi, lo>::all([&](auto kc) { row[kc.value * T + tid] = own[kc.value]; });
                    }
                }
            });
        } else {
#pragma unroll
            for (int k = NB - 1; k >= 0; --k) row[k * T + tid] = own[k];
        }
        // Row q of the keep table belongs to the q-th offered item.  A wavefront whose 64
        // lanes took nothing writes nothing and notes that in nzm: bit (q % 64) of lane
        // (q / 64) says whether this wavefront's part of row q exists.  The flags of 32
        // items are collected in a scalar first.
        bool nz;
        if constexpr (SKIP_UNCHANGED) {
            nz = false;
#pragma unroll
            for (int g = 0; g < kGroups; ++g) nz = nz || group_changed[g];
        } else {
            uint32_t any_bits = bits[0];
#pragma unroll
            for (int x = 1; x < NW; ++x) any_bits |= bits[x];
            nz = __builtin_amdgcn_ballot_w64(any_bits != 0) != 0ull;
        }
        if (nz) {
            uint32_t *kq = kp + (size_t)q * (NW * T);  // scalar base, lane offsets that never change
#pragma unroll
            for (int x = 0; x < NW; ++x) kq[x * T + tid] = bits[x];
            scalar_set_bit(nz_acc, q & 31);
        }
        if ((q & 31) == 31) hand_over(q);
        if constexpr (ADDTID) wait_lds();
        lds_sync<T>();  // the new row is visible
    };
    // After item q: can the capacity itself be reached?  (The same answer in every lane of the instance.)
    auto capacity_reached = [&](int q) -> bool {
        if constexpr (!STOP_WHEN_FULL) {
            return false;
        } else {
            if ((q & check_mask) != check_mask) return false;
            int any = 0;
#pragma unroll
            for (int k = NB - G; k < NB; ++k)  // cell C sits in one of the last G slots
                any |= k * T + tid == C ? own[k] : 0;
            const bool wave_full = __builtin_amdgcn_ballot_w64(any != 0) == 0ull;
            if constexpr (T == 64) {
                return wave_full;
            } else {
                if (!wave_full && (tid & 63) == 0) *unfinished = q + 1;
                lds_sync<T>();
                return uniform(*unfinished) != q + 1;
            }
        }
    };

    // Algorithm 1, once the whole remaining time C is reachable (after item q): no level is worth
    // more; the levels met so far are worth less (their rows did not reach C); a later level is
    // worth C exactly when its own remaining time is C (nothing is dropped after it).  The first
    // such entry among those not met yet, else the whole list, is the answer: the deepest level
    // among equals.
    auto settle_levels = [&](int q) {
        if constexpr (REC) {
            int found = nact;
            for (int c0 = (q + 1) & ~63; c0 < nact; c0 += 64) {
                const int e = c0 + lane;
                const unsigned long long hit =
                    __builtin_amdgcn_ballot_w64(e > q && e < nact && load_item_pad(list + e) == C);
                if (hit != 0ull) {
                    found = c0 + __builtin_ctzll(hit);
                    break;
                }
            }
            // (the check runs every few items: a level met since C was reached may hold it already)
            if (best.value < C) best = BestLevel{C, found, C};
        }
    };

    for (int q0 = 0; q0 < nact; q0 += 64) {
        const int2 nxt = load_chunk(q0 + 64);
        const int nxt_p = load_probe_chunk(q0 + 64);
        const int q1 = min(q0 + 64, nact);
        int q = q0;
        while (q < q1) {
            int w = __builtin_amdgcn_readlane(cur.x, q & 63);
            while (w <= light_max) {  // run of light items
                item(std::false_type{}, q, w, VEQW ? w : __builtin_amdgcn_readlane(cur.y, q & 63));
                if (capacity_reached(q)) { settle_levels(q); hand_over(q); return q + 1; }
                if (++q >= q1) break;
                w = __builtin_amdgcn_readlane(cur.x, q & 63);
            }
            if (q < q1) {  // one heavy item
                item(std::true_type{}, q, w, VEQW ? w : __builtin_amdgcn_readlane(cur.y, q & 63));
                if (capacity_reached(q)) { settle_levels(q); hand_over(q); return q + 1; }
                ++q;
            }
        }
        cur = nxt;
        cur_p = nxt_p;
    }
    if (nact > 0) hand_over(nact - 1);
    return nact;
}

// Picks the sweep_stage instance for the stage's chunk count (1 .. N).
template <int T, int G, int NW, bool ADDTID, bool VEQW, bool REC, bool SKIP_UNCHANGED, int N>
__device__ __forceinline__ int sweep_dispatch(int nchunk, int32_t *row, uint32_t row_off, int light_max, int tid,
                                               int nact, const OfferedItem *list, uint32_t *kp,
                                               unsigned long long &nzm, BestLevel &best, int C, int32_t *unfinished, bool levels)
{
    if (nchunk == N) {
        return sweep_stage<T, N * G, G, NW, ADDTID, VEQW, REC, SKIP_UNCHANGED>(row, row_off, light_max, tid, nact, list, kp, nzm,
                                                            best, C, unfinished, levels);
    } else if constexpr (N > 1) {
        return sweep_dispatch<T, G, NW, ADDTID, VEQW, REC, SKIP_UNCHANGED, N - 1>(nchunk, row, row_off, light_max, tid, nact, list, kp,
                                                                  nzm, best, C, unfinished, levels);
    }
    return 0;
}

// ---- rows of 16-bit cells (P16 kernels) -----------------------------------------------
// Where every value equals its weight (the paper's Problem 1) the row is kept as
// row[c] - c, which lies in [-c, 0]: with capacities up to 32766 it fits 16 bits.  The P16
// kernels store two cells per 32-bit word, in registers and in LDS: word (j * T + t) holds
// cell (2j * T + t) in its low half and cell ((2j + 1) * T + t) in its high half, so lane t
// owns "pair j" = register slots 2j and 2j + 1.  Half the LDS per instance (more workgroups
// per compute unit), half the LDS instructions per cell, and packed 16-bit arithmetic:
//   cand pair = row pair shifted by w cells; diff = own - cand (negative where the item is
//   taken: both lie in [-32767, 0], so the difference cannot overflow); own = max(own, cand);
//   the two sign bits of diff are shifted into the keep word.
// Every LDS access stays an aligned 32-bit one.  With s = t - w = -a * T + r (0 <= r < T) slot
// k of lane t needs logical slot k - a of column r.  For even a that is a whole stored pair;
// for odd a it is the high half of one stored word and the low half of the next, which one
// byte permute assembles.  A light item (w <= T) has a in {0, 1}; every lane then reads words
// j * T + r for j = -1 .. NP-1 (the word at j = -1 lies in the guard zone, T words holding
// -32767 in both halves, which no cell can fall below), and a wavefront whose lanes all have
// a = 0 (its first lane is at or above w: most wavefronts, for the usual light items) skips
// the permutes and the guard read.  Heavy items compute a per lane and clamp each word index
// into the guard.
// The keep word of (item, lane) holds the take bit of slot k at bit 8 (k mod 4) + 7 - (k div 4)
// (at most 32 slots per lane): the sign bytes of two pairs' differences are gathered by one
// byte permute and their top bits dropped into bit 7 of the four bytes of the word, which
// moves down by one bit per two pairs (pairs 2i and 2i + 1 make step i, taken from the top).
constexpr int kGuard16 = (int)0x80018001;  // -32767 in both halves

__device__ __forceinline__ uint32_t pk_sub_i16(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_sub_i16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_max_i16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
// One step of the keep word: the word moves down by one bit and the sign bits of the four
// halves of (diff_hi, diff_lo) - the differences of pairs 2i + 1 and 2i - land in bit 7 of
// bytes 3, 2 (pair 2i + 1: high half, low half) and 1, 0 (pair 2i).  Three instructions for two
// pairs; the bit-field insert is pinned (the compiler would otherwise split it).
__device__ __forceinline__ uint32_t shift_in_signs(uint32_t acc, uint32_t diff_hi, uint32_t diff_lo, uint32_t top_bits)
{
    const uint32_t sign_bytes = __builtin_amdgcn_perm(diff_hi, diff_lo, 0x07050301u);
    uint32_t out;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(out) : "s"(top_bits), "v"(sign_bytes), "v"(acc >> 1));
    return out;
}
// Bit of slot k in a keep word of the packed kernels.
__device__ __forceinline__ int keep_bit16(int k) { return (k & 3) * 8 + 7 - (k >> 2); }
// Cell c of a packed row (sign-extended).
template <int T>
__device__ __forceinline__ int row16_cell(const int32_t *row, int c)
{
    const int k = c / T, t = c - k * T;
    const int word = row[(k >> 1) * T + t];
    return (int)(int16_t)((uint32_t)word >> ((k & 1) * 16));
}

// All offered items of one stage on a packed row of NP pairs per lane (cells 0 .. 2 NP T - 1
// >= C).  Same contract as sweep_stage (VEQW only): returns the number of items swept.
template <int T, int NP, bool REC, bool SKIP_UNCHANGED>
__device__ __forceinline__ int sweep_stage_p16(int32_t *row, uint32_t row_off, int tid, int nact, const OfferedItem *list,
                                                uint32_t *kp, unsigned long long &nzm, BestLevel &best, int C,
                                                int32_t *unfinished, bool levels)
{
    constexpr bool STOP_WHEN_FULL = true;  // (REC: Algorithm 1 only, see settle_levels)
    // short lists: after every second item, else every eighth; never for the capacity sweep,
    // which reads the row below C as well
    const int check_mask = REC && !levels ? INT_MAX : nact <= 64 ? 1 : 7;
    static_assert(NP >= 1 && NP <= 16, "the take bits of a lane fit one keep word");
    asm volatile("" : "+v"(tid));  // (as in sweep_stage: keeps the per-lane constants out of kernel entry)
    const int wave_first = uniform(tid & ~63);
    const int lane = tid & 63;
    auto load_chunk = [&](int first) {
        return first + lane < nact ? load_item_wv(list + first + lane) : make_int2(0, 0);
    };
    auto load_probe_chunk = [&](int first) {
        return REC && first + lane < nact ? load_item_pad(list + first + lane) : -1;
    };
    int2 cur = load_chunk(0);
    int cur_p = load_probe_chunk(0);
    uint32_t own[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        own[j] = ((uint32_t)(-(2 * j * T + tid)) & 0xffffu) | ((uint32_t)(-((2 * j + 1) * T + tid)) << 16);
        row[j * T + tid] = (int32_t)own[j];
    }
    lds_sync<T>();  // initial row visible to every lane

    const int m0w = uniform((int)row_off + wave_first * 4);
    uint32_t nz_acc = 0;
    auto hand_over = [&](int q) {
        if ((tid & 63) == (q >> 6)) nzm |= (unsigned long long)nz_acc << (q & 32);
        nz_acc = 0;
    };
    constexpr uint32_t kSelSame = 0x07060504u;   // the stored pair itself
    constexpr uint32_t kSelCross = 0x05040302u;  // high half of the word below, low half of this one
    // KIND 0: whole wavefront at or above w (no permutes); 1: light item, mixed lanes; 2: heavy item
    auto item = [&](auto kind_tag, int q, int w) {
        constexpr int KIND = decltype(kind_tag)::value;
        uint32_t acc = 0;
        uint32_t cand[NP];
        int probe_at = -1, probe = 0;
        if constexpr (REC) {
            probe_at = __builtin_amdgcn_readlane(cur_p, q & 63);
            probe = row16_cell<T>(row, max(probe_at, 0));
        }
        if constexpr (KIND == 0) {
            const int32_t *src = row + (tid - w);
#pragma unroll
            for (int j = NP - 1; j >= 0; --j) cand[j] = (uint32_t)src[j * T];
        } else if constexpr (KIND == 1) {
            const int below = tid < w ? 1 : 0;
            const int32_t *src = row + (tid - w + below * T);
            const uint32_t sel = below ? kSelCross : kSelSame;
            uint32_t d[NP + 1];
#pragma unroll
            for (int j = NP; j >= 0; --j) d[j] = (uint32_t)src[(j - 1) * T];  // d[j] = word j - 1
#pragma unroll
            for (int j = NP - 1; j >= 0; --j) cand[j] = __builtin_amdgcn_perm(d[j + 1], d[j], sel);
        } else {
            const int a = tid < w ? (w - tid + T - 1) / T : 0;
            const int r = tid - w + a * T, e = a >> 1;
            const uint32_t sel = (a & 1) ? kSelCross : kSelSame;
#pragma unroll
            for (int j = NP - 1; j >= 0; --j) {
                const uint32_t hi = (uint32_t)row[max(j - e, -1) * T + r];
                const uint32_t lo = (uint32_t)row[max(j - e - 1, -1) * T + r];
                cand[j] = __builtin_amdgcn_perm(hi, lo, sel);
            }
        }
        const uint32_t top_bits = (uint32_t)uniform((int)0x80808080u);  // (a scalar operand of the insert)
#pragma unroll
        for (int i = (NP - 1) / 2; i >= 0; --i) {  // step i: pairs 2i + 1 (if there is one) and 2i
            uint32_t diff_hi = 0;
            if (2 * i + 1 < NP) {
                diff_hi = pk_sub_i16(own[2 * i + 1], cand[2 * i + 1]);
                own[2 * i + 1] = pk_max_i16(own[2 * i + 1], cand[2 * i + 1]);
            }
            const uint32_t diff_lo = pk_sub_i16(own[2 * i], cand[2 * i]);
            own[2 * i] = pk_max_i16(own[2 * i], cand[2 * i]);
            acc = shift_in_signs(acc, diff_hi, diff_lo, top_bits);  // step i ends at bit 7 - i of each byte
        }
        if constexpr (REC) {
            const int level_value = uniform(probe) + probe_at;
            if (probe_at >= 0 && level_value > best.value) best = BestLevel{level_value, q, probe_at};
        }
        constexpr int kGroup = 8;  // pairs per write-back group
        constexpr int kGroups = (NP - 1) / kGroup + 1;
        bool group_changed[kGroups];
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            // pairs 8g .. 8g + 7 are steps 4g .. 4g + 3: bits 7 - 4g .. 4 - 4g of every byte
            const uint32_t m = (0xF0u >> (4 * g)) * 0x01010101u;
            group_changed[g] = !SKIP_UNCHANGED || __builtin_amdgcn_ballot_w64((acc & m) != 0) != 0ull;
        }
        lds_sync<T>();  // every lane has read the old row

        SlotsDown<(NP - 1) / kGroup>::all([&](auto gc) {
            constexpr int lo = gc.value * kGroup;
            constexpr int hi = lo + kGroup - 1 < NP - 1 ? lo + kGroup - 1 : NP - 1;
            static_assert(hi * T * 4 <= 65535, "the add-TID offset reaches every pair");
            if (group_changed[gc.value]) {
                m0_settle(m0w);
                SlotsDownTo<hi, lo>::all([&](auto jc) { write_addtid<jc.value * T * 4>(m0w, (int)own[jc.value]); });
            }
        });
        bool nz;
        if constexpr (SKIP_UNCHANGED) {
            nz = false;
#pragma unroll
            for (int g = 0; g < kGroups; ++g) nz = nz || group_changed[g];
        } else {
            nz = __builtin_amdgcn_ballot_w64(acc != 0) != 0ull;
        }
        if (nz) {
            uint32_t *kq = kp + (size_t)q * T;  // scalar base, a lane offset that never changes
            kq[tid] = acc;
            scalar_set_bit(nz_acc, q & 31);
        }
        if ((q & 31) == 31) hand_over(q);
        wait_lds();
        lds_sync<T>();  // the new row is visible
    };
    auto capacity_reached = [&](int q) -> bool {
        if constexpr (!STOP_WHEN_FULL) {
            return false;
        } else {
            if ((q & check_mask) != check_mask) return false;
            // cell C sits in the top pair
            constexpr int j = NP - 1;
            const uint32_t any = own[j] & ((2 * j * T + tid == C ? 0xffffu : 0u) | ((2 * j + 1) * T + tid == C ? 0xffff0000u : 0u));
            const bool wave_full = __builtin_amdgcn_ballot_w64(any != 0) == 0ull;
            if constexpr (T == 64) {
                return wave_full;
            } else {
                if (!wave_full && (tid & 63) == 0) *unfinished = q + 1;
                lds_sync<T>();
                return uniform(*unfinished) != q + 1;
            }
        }
    };

    // Algorithm 1, once the whole remaining time C is reachable (after item q): no level is worth
    // more; the levels met so far are worth less (their rows did not reach C); a later level is
    // worth C exactly when its own remaining time is C (nothing is dropped after it).  The first
    // such entry among those not met yet, else the whole list, is the answer: the deepest level
    // among equals.
    auto settle_levels = [&](int q) {
        if constexpr (REC) {
            int found = nact;
            for (int c0 = (q + 1) & ~63; c0 < nact; c0 += 64) {
                const int e = c0 + lane;
                const unsigned long long hit =
                    __builtin_amdgcn_ballot_w64(e > q && e < nact && load_item_pad(list + e) == C);
                if (hit != 0ull) {
                    found = c0 + __builtin_ctzll(hit);
                    break;
                }
            }
            // (the check runs every few items: a level met since C was reached may hold it already)
            if (best.value < C) best = BestLevel{C, found, C};
        }
    };

    for (int q0 = 0; q0 < nact; q0 += 64) {
        const int2 nxt = load_chunk(q0 + 64);
        const int nxt_p = load_probe_chunk(q0 + 64);
        const int q1 = min(q0 + 64, nact);
        for (int q = q0; q < q1; ++q) {
            const int w = __builtin_amdgcn_readlane(cur.x, q & 63);
            if (w <= wave_first) item(std::integral_constant<int, 0>{}, q, w);
            else if (w <= T) item(std::integral_constant<int, 1>{}, q, w);
            else item(std::integral_constant<int, 2>{}, q, w);
            if (capacity_reached(q)) { settle_levels(q); hand_over(q); return q + 1; }
        }
        cur = nxt;
        cur_p = nxt_p;
    }
    if (nact > 0) hand_over(nact - 1);
    return nact;
}

// Picks the sweep_stage_p16 instance for the stage's pair count (1 .. N).
template <int T, bool REC, bool SKIP_UNCHANGED, int N>
__device__ __forceinline__ int sweep_dispatch_p16(int npair, int32_t *row, uint32_t row_off, int tid, int nact,
                                                   const OfferedItem *list, uint32_t *kp, unsigned long long &nzm,
                                                   BestLevel &best, int C, int32_t *unfinished, bool levels)
{
    if (npair == N) {
        return sweep_stage_p16<T, N, REC, SKIP_UNCHANGED>(row, row_off, tid, nact, list, kp, nzm, best, C, unfinished, levels);
    } else if constexpr (N > 1) {
        return sweep_dispatch_p16<T, REC, SKIP_UNCHANGED, N - 1>(npair, row, row_off, tid, nact, list, kp, nzm, best, C,
                                                                 unfinished, levels);
    }
    return 0;
}

// WPE = wavefronts per SIMD the register budget is held to (LDS allows that many).
// REC = false: the sequential mode.  REC = true: the modes that read more than row[C] off
// one sweep, chosen by a.mode at run time:
//   Algorithm 1 on one knapsack (every item offered, the best level tracked during the
//   sweep, the walk started at that level);
//   the capacity sweep (Sec. IV.C feedback): one sweep at the largest of the instance's
//   capacities, then the value at each capacity is a cell of the final row and each
//   capacity gets a walk of its own, the wavefronts of the instance sharing the walks.
// P16: rows of 16-bit cells (see sweep_stage_p16); every instance must have values equal to
// its weights, which the handle's creator promised, and one that has not is refused.
template <int T, int K, int G, int WPE, bool REC, bool P16>
__global__ void __launch_bounds__(T == 64 ? 256 : T, WPE)
seq_lds_kernel(BatchArgs a, LdsLayout lay, uint32_t *keep, int64_t keep_words_per_inst, OfferedItem *lists,
               int list_stride, unsigned long long *swept_cells)
{
    static_assert(!P16 || (K % 2 == 0 && K <= 32 && K * T <= 32767), "packed rows: whole pairs, one keep word, 16-bit cells");
    extern __shared__ __align__(16) int32_t lds_raw[];
    static_assert(K <= 64, "at most 64 segments per wavefront");
    constexpr int NW = (K + 31) / 32;
    static_assert(K % G == 0, "whole chunks");
    // add-TID write-back wherever M0 stays below 65536 (one instance per workgroup: the row
    // starts at most 1 KB into LDS and a wavefront's first lane at most 4 KB further; the
    // four-instances-per-workgroup variant keeps its rows within 64 KB altogether)
    constexpr bool ADDTID = true;
    static_assert(T != 64 || 4 * (256 + K * T) * 4 <= 65536, "rows of the packed variant stay below 64 KB");
    constexpr int NCH = (K + G - 1) / G;
    // Long rows: a group of slots in which the wavefront changed nothing is not written back
    // (measured: 5 % on the ResNet shape with 26 slots, 1 % on the VGG shape with 20; with 16
    // slots, on the same shapes scaled down, the test costs 1-3 % more than it saves).
    constexpr bool kSkipUnchanged = K >= 20;
    static_assert(T % 64 == 0 && T <= 1024, "whole wavefronts");

    const int sub = (T == 64) ? (int)(threadIdx.x >> 6) : 0;
    const int tid = (T == 64) ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
    const int inst = (T == 64) ? (int)blockIdx.x * 4 + sub : (int)blockIdx.x;
    if (inst >= a.batch) return;  // whole wavefront (T == 64) or never (grid == batch)
    // One wavefront of the instance does everything that is serial: the stage set-up, the
    // stages settled without a sweep, the walk.  Its instructions all issue on the one SIMD
    // it lives on, next to that SIMD's share of the sweeps; which wavefront it is rotates
    // with the instance, so that the workgroups sharing a compute unit spread this work over
    // its SIMDs instead of piling it onto the first.
    constexpr int kSerialChoices = T / 64 < 4 ? T / 64 : 4;
    const int serial_wave = (T == 64) ? 0 : (int)(blockIdx.x % kSerialChoices);
    const bool serial = (tid >> 6) == serial_wave;
    const int sl = tid & 63;  // lane within the wavefront

    int32_t *misc = lds_raw + (size_t)sub * lay.ints_per_inst;
    int32_t *row = misc + lay.guard_cells;
    const uint32_t row_off = lds_offset(row);
    // misc: [0] fault flags (bit 2: some value differs from its weight), [1] offered-item count,
    //       [2..3] value sum, [4..5] fill-order seen mask, [6] the stage being swept, [7] tag of the
    //       last row-is-full check that found an unfinished cell

    const int n = a.n_items[inst];
    const int m = a.n_knapsacks[inst];
    const int32_t *__restrict__ W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *__restrict__ V = a.values + (size_t)inst * a.item_stride;
    const int32_t *__restrict__ cap = a.capacities + (size_t)inst * a.knap_stride;
    const int32_t *__restrict__ ord =
        !REC && a.fill_order ? a.fill_order + (size_t)inst * a.knap_stride : nullptr;
    const bool levels = REC && a.mode == DEFT_MODE_RECURSIVE;      // Algorithm 1
    const bool caps_sweep = REC && a.mode == DEFT_MODE_CAPACITY_SWEEP;
    const int32_t *__restrict__ drop = levels ? a.drop_time + (size_t)inst * a.item_stride : nullptr;
    int32_t *out_asg = a.assignment + (size_t)inst * a.item_stride;
    int32_t *out_kv = a.knap_value + (size_t)inst * a.knap_stride;
    int32_t *out_kl = a.knap_load + (size_t)inst * a.knap_stride;
    uint32_t *kp = uniform_ptr(keep + (size_t)inst * keep_words_per_inst);
    // one item list per stage
    OfferedItem *inst_lists = uniform_ptr(lists + (size_t)inst * a.knap_stride * list_stride);

    // ---- per-instance validation -------------------------------------------
    // The first T items and the capacities are fetched here, before n and m have arrived
    // and been checked (the arrays are item_stride / knap_stride long whatever the counts
    // say), so that one memory round trip serves both.
    const bool pre_item = tid < a.item_stride, pre_knap = (tid & 63) < a.knap_stride;
    const int w_pre = pre_item ? W[tid] : 0, v_pre = pre_item ? V[tid] : 0;
    const int d_pre = REC && levels && pre_item ? drop[tid] : 0;
    const int cap_pre = pre_knap ? cap[tid & 63] : 0;
    const int ord_pre = ord && pre_knap ? ord[tid & 63] : (tid & 63);
    if (tid < kMiscInts) misc[tid] = 0;
    for (int i = kMiscInts + tid; i < lay.guard_cells; i += T) misc[i] = P16 ? kGuard16 : INT_MIN;
    lds_sync<T>();
    // Kept in registers for the whole kernel, so that the stage loop below never waits on
    // memory for them: lane j of every wavefront holds capacity j and the j-th entry of the
    // fill order (at most 64 knapsacks), and lane i of the serial wavefront holds weight and
    // value of item i (the first 64 items; longer lists reload the rest from the cache).
    int cap_l = 0, ord_l = tid & 63, w_first = 0, v_first = 0;
    {
        uint32_t flags = 0;
        unsigned long long vs = 0;
        const bool counts_ok = n >= 0 && n <= a.item_stride && m >= 0 && m <= a.knap_stride &&
                               (!levels || m == 1) && (!caps_sweep || m <= 31);
        if (!counts_ok) {
            flags = 1;
        } else {
            if ((tid & 63) < m) {
                cap_l = cap_pre;
                ord_l = ord_pre;
            }
            for (int i = tid; i < n; i += T) {
                const bool pre = i == tid;  // the first round: fetched above
                const int w = pre ? w_pre : W[i], v = pre ? v_pre : V[i];
                if (w < 1 || v < 0) flags |= 1; else vs += (unsigned)v;
                if (v != w) flags |= P16 ? 5 : 4;
                if constexpr (REC) {
                    if (levels && (pre ? d_pre : drop[i]) < 0) flags |= 1;
                }
            }
            for (int j = tid; j < m; j += T) {
                const int c = cap_l;
                if (c < 0) flags |= 1; else if (c > a.max_capacity) flags |= 2;
                if (ord) {
                    const int o = ord_l;
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
        // one LDS atomic per wavefront (every lane is here: the branches above are uniform or
        // closed); a lane's value sum is below 2^35, summed in three 16-bit-wide parts
        const uint32_t wave_flags = (__ballot(flags & 1) ? 1u : 0u) | (__ballot(flags & 2) ? 2u : 0u) |
                                    (__ballot(flags & 4) ? 4u : 0u);
        const unsigned long long wave_vs = (unsigned long long)(unsigned)wave_sum((int)(vs & 0xffffu)) +
                                           ((unsigned long long)(unsigned)wave_sum((int)((vs >> 16) & 0xffffu)) << 16) +
                                           ((unsigned long long)(unsigned)wave_sum((int)(vs >> 32)) << 32);
        if ((tid & 63) == 0) {
            if (wave_flags) atomicOr(reinterpret_cast<uint32_t *>(&misc[0]), wave_flags);
            if (wave_vs) atomicAdd(reinterpret_cast<unsigned long long *>(&misc[2]), wave_vs);
        }
    }
    lds_sync<T>();
    int status = DEFT_OK;
    const bool veqw = uniform(misc[0] & 4) == 0;
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
    // knapsack ids start at "none"; the capacity sweep's masks start empty
    for (int i = tid; i < a.item_stride; i += T) out_asg[i] = caps_sweep ? 0 : -1;
    if (status != DEFT_OK) {
        if (tid == 0) a.total_value[inst] = 0;
        return;
    }

    // ---- stages ----------------------------------------------------------------
    if (serial && sl < n) { w_first = W[sl]; v_first = V[sl]; }
    // Items already placed: bit (i / 64) of lane (i % 64) of the serial wavefront.
    unsigned long long placed = 0;
    long long total = 0;
    const int stages = caps_sweep ? min(m, 1) : m;
    // (an out-of-range order entry was rejected above, so s and j are below 64 here)
    auto stage_knapsack = [&](int s) { return __builtin_amdgcn_readlane(ord_l, s); };
    int cap_max = 0;  // capacity sweep: one sweep at the largest capacity serves them all
    if constexpr (REC) {
        if (caps_sweep) {
            cap_max = (tid & 63) < m ? cap_l : 0;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) cap_max = max(cap_max, __shfl_xor(cap_max, off));
            cap_max = uniform(cap_max);
        }
    }
    auto stage_capacity = [&](int j) {
        if constexpr (REC) {
            if (caps_sweep) return cap_max;
        }
        return __builtin_amdgcn_readlane(cap_l, j);
    };
    // weight and value of item i0 + lane, as the serial wavefront's stage loop reads them
    auto item_w = [&](int i0, int i) { return i >= n ? 0 : i0 == 0 ? w_first : W[i]; };
    auto item_v = [&](int i0, int i) { return i >= n ? 0 : i0 == 0 ? v_first : V[i]; };
    int s = 0;
    while (true) {
        // The serial wavefront prepares stages one after the other, settling those that need
        // no sweep on its own, until it reaches one that does; only then do the other
        // wavefronts of the instance join in.  misc[1] = that stage's offered-item count
        // (negative: every stage is done), misc[6] = the stage.
        if (serial) {
            const int tid = sl;  // (the lane: this block addresses items as i0 + lane)
            int cnt = -1;
            for (; s < stages; ++s) {
                const int j = stage_knapsack(s);
                const int C = stage_capacity(j);
                OfferedItem *list = inst_lists + (size_t)s * list_stride;
                if (levels) {
                    // Algorithm 1: the whole list is offered in generation order (an item heavier
                    // than the remaining time changes nothing, but the levels are counted in list
                    // positions).  Entry i gets P_i = R - sum of drop[t] over t >= i, the remaining
                    // time of the level that ends before item i, from a suffix sum taken 64 items
                    // at a time from the end of the list.
                    // Only "how far below C" matters, and C is at most 2^24: a drop time is
                    // clamped just above that and so is the running sum, which keeps everything
                    // in 32 bits and exact wherever the remaining time is not negative.
                    constexpr int kOver = (1 << 24) + 1;
                    int behind = 0;  // sum of drop over the chunks already done (uniform)
                    for (int i0 = (n - 1) & ~63; i0 >= 0 && n > 0; i0 -= 64) {
                        const int i = i0 + tid;
                        const int x = wave_suffix_sum(i < n ? min(drop[i], kOver) : 0, tid);
                        if (i < n) {
                            const int left = C - min(x + behind, kOver);
                            OfferedItem e;
                            e.w = W[i]; e.v = V[i]; e.index = i; e.pad = left < 0 ? -1 : left;
                            list[i] = e;
                        }
                        behind = min(behind + __builtin_amdgcn_readlane(x, 0), kOver);
                    }
                    cnt = n;
                    break;
                }
                // offered items: not yet placed and able to fit at all, ascending index
                cnt = 0;
                int unplaced = 0;
                int offered_weight = 0;  // per lane at most 64 items of at most 2^24 each
                for (int i0 = 0; i0 < n; i0 += 64) {
                    const int i = i0 + tid;
                    const int w = item_w(i0, i);
                    const int v = item_v(i0, i);
                    const bool open = i < n && ((placed >> (i0 >> 6)) & 1ull) == 0;
                    const bool f = open && w <= C;
                    unplaced += __popcll(__ballot(open));
                    const unsigned long long mask = __ballot(f);
                    if (f) {
                        OfferedItem e;
                        e.w = w; e.v = v; e.index = i; e.pad = -1;  // no level ends here
                        list[cnt + __popcll(mask & ((1ull << tid) - 1ull))] = e;
                        offered_weight += w;
                    }
                    cnt += __popcll(mask);
                }
                if (unplaced == 0) {  // every item is placed: the remaining stages stay empty
                    s = stages;
                    break;
                }
                // Nothing is offered, or everything offered fits together: the DP has nothing to
                // decide.  Its answer is known: at every step of the walk the capacity left
                // still holds all earlier items, so an item is taken exactly when its value is
                // positive (a zero-value item never strictly improves a cell).  The stage is
                // settled here, without a sweep.  (Not for the capacity sweep: its other
                // capacities are smaller.)
                if (!caps_sweep) {
                    // (a lane's share is clamped just above the largest capacity, so that the
                    // wavefront's sum stays in range and still exceeds C whenever the true sum does)
                    offered_weight = wave_sum(min(offered_weight, (1 << 24) + 1));
                    if (offered_weight <= C) {
                        int vsum = 0, lsum = 0;  // values sum to less than 2^31, weights to at most C
                        for (int i0 = 0; i0 < n; i0 += 64) {
                            const int i = i0 + tid;
                            const int w = item_w(i0, i);
                            const int v = item_v(i0, i);
                            if (i < n && ((placed >> (i0 >> 6)) & 1ull) == 0 && w <= C && v > 0) {
                                placed |= 1ull << (i0 >> 6);
                                out_asg[i] = j;
                                vsum += v;
                                lsum += w;
                            }
                        }
                        vsum = wave_sum(vsum);
                        lsum = wave_sum(lsum);
                        if (tid == 0) {
                            out_kv[j] = vsum;
                            out_kl[j] = lsum;
                            total += vsum;
                        }
                        cnt = -1;  // tells every wavefront that the stage is done
                    } else if (cnt <= kEnumItems) {
                        // A handful of offered items: lane L weighs the subset whose members are the
                        // set bits of L (bit t = the t-th offered item).  The DP with its walk returns
                        // the feasible subset of greatest value and, among equals, the one with the
                        // smallest such number; that is picked here directly.
                        int wq[kEnumItems], vq[kEnumItems], iq[kEnumItems];
#pragma unroll
                        for (int t = 0; t < kEnumItems; ++t) { wq[t] = 0; vq[t] = 0; iq[t] = 0; }
                        int got = 0;
                        for (int i0 = 0; i0 < n; i0 += 64) {
                            const int i = i0 + tid;
                            const int w = item_w(i0, i);
                            const int v = item_v(i0, i);
                            unsigned long long mask =
                                __ballot(i < n && ((placed >> (i0 >> 6)) & 1ull) == 0 && w <= C);
                            while (mask) {
                                const int l = __builtin_ctzll(mask);
                                mask &= mask - 1;
                                const int wl = __builtin_amdgcn_readlane(w, l), vl = __builtin_amdgcn_readlane(v, l);
#pragma unroll
                                for (int t = 0; t < kEnumItems; ++t)
                                    if (t == got) { wq[t] = wl; vq[t] = vl; iq[t] = i0 + l; }
                                ++got;
                            }
                        }
                        int ws = 0, vs = 0;  // six weights of at most 2^24; values sum to less than 2^31
#pragma unroll
                        for (int t = 0; t < kEnumItems; ++t)
                            if ((tid >> t) & 1) { ws += wq[t]; vs += vq[t]; }
                        const bool feasible = tid < (1 << cnt) && ws <= C;
                        const int best_value = wave_max(feasible ? vs : -1);
                        // (the empty subset is always feasible, so the ballot is never empty)
                        const int pick = __builtin_ctzll(__ballot(feasible && vs == best_value));
                        const int load = __builtin_amdgcn_readlane(ws, pick);
#pragma unroll
                        for (int t = 0; t < kEnumItems; ++t) {
                            if ((pick >> t) & 1) {
                                if (tid == (iq[t] & 63)) placed |= 1ull << (iq[t] >> 6);
                                if (tid == 0) out_asg[iq[t]] = j;
                            }
                        }
                        if (tid == 0) {
                            out_kv[j] = best_value;
                            out_kl[j] = load;
                            total += best_value;
                        }
                        cnt = -1;
                    }
                }
                if (cnt >= 0) break;  // this stage needs its sweep
            }
            if (tid == 0) {
                misc[1] = s < stages ? cnt : -1;
                misc[6] = s;
                misc[7] = 0;  // no check of this stage has run yet
            }
        }
        global_sync<T>();  // the list (global memory), the count and the stage (LDS) are visible
        if (uniform(misc[1]) < 0) break;
        s = uniform(misc[6]);
        const int j = stage_knapsack(s);
        const int C = stage_capacity(j);
        OfferedItem *list = inst_lists + (size_t)s * list_stride;

        const int nchunk = uniform((C / T + G) / G);  // G-slot chunks covering cells 0 .. C
        const int nact = min(uniform(misc[1]), list_stride);
        unsigned long long nzm = 0;
        BestLevel best{0, 0, 0};
        const int light_max = lay.guard_cells - kMiscInts;
        int swept;
        if constexpr (P16)
            swept = sweep_dispatch_p16<T, REC, kSkipUnchanged, K / 2>(uniform((C / T + 2) / 2), row, row_off, tid, nact, list, kp,
                                                                      nzm, best, C, &misc[7], levels);
        else if (veqw)
            swept = sweep_dispatch<T, G, NW, ADDTID, true, REC, kSkipUnchanged, NCH>(nchunk, row, row_off, light_max, tid, nact, list,
                                                                     kp, nzm, best, C, &misc[7], levels);
        else
            swept = sweep_dispatch<T, G, NW, ADDTID, false, REC, kSkipUnchanged, NCH>(nchunk, row, row_off, light_max, tid, nact, list,
                                                                      kp, nzm, best, C, &misc[7], levels);

        // the value at capacity c as the final row holds it
        auto row_value = [&](int c) {
            if constexpr (P16) return row16_cell<T>(row, c) + c;
            else return row[c] + (veqw ? c : 0);
        };
        int value = uniform(row_value(C));
        // where the walk starts: the last offered item at the full capacity, or (Algorithm 1)
        // the last item of the best level at that level's remaining time
        int walk_from = swept - 1, walk_cap = C;  // items that were not swept were not taken
        int sweep_cap = 0, sweep_value = 0;  // capacity sweep: lane x holds capacity x and the value there
        if constexpr (REC) {
            if (levels) {
                if (value > best.value) best = BestLevel{value, nact, C};  // level 0: the whole list
                value = best.value;
                walk_from = min(best.length, swept) - 1;  // what was not swept was not taken
                walk_cap = best.remain;
            }
            if (caps_sweep && (tid & 63) < m) {
                sweep_cap = cap_l;
                sweep_value = row_value(sweep_cap);
            }
        }

        // ---- traceback ------------------------------------------------------------
        // The row is dead now; its LDS holds what the walk needs: weight and index of
        // every offered item and, per wavefront, which keep-row parts exist.
        lds_sync<T>();  // every lane has read its cells of the final row
        int32_t *tb_w = row, *tb_index = row + list_stride;
        unsigned long long *tb_nz = reinterpret_cast<unsigned long long *>(row + 2 * list_stride);
        for (int i = tid; i < swept; i += T) {
            tb_w[i] = load_item_wv(list + i).x;
            tb_index[i] = load_item_index(list + i);
        }
        tb_nz[tid] = nzm;  // wavefront x, lane l: rows 64 l .. 64 l + 63
        if (swept_cells && tid < 64) {
            // measurement only: the cell-updates this stage's sweep evaluated, as the metric
            // counts them (C - w + 1 per swept item)
            unsigned long long cells = 0;
            for (int i = tid; i < swept; i += 64) cells += (unsigned)max(C - load_item_wv(list + i).x + 1, 0);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) cells += __shfl_down(cells, off);
            if (tid == 0) atomicAdd(swept_cells, cells);
        }
        global_sync<T>();  // keep words (global memory) and the staged data (LDS) are visible

        // One wavefront walks the keep words back from (last offered item, C).  The
        // walk is a chain of dependent loads, so six steps are taken per memory round
        // trip: lane L in [2^d, 2^(d+1)) assumes the decisions spelled by the bits of
        // L below its leading one for the items q .. q-d+1 (most significant first)
        // and fetches the keep bit of item q-d at the capacity those decisions leave;
        // a ballot then gives all 63 answers and the true path is read off it.  A lane
        // whose keep-row part was never written knows its answer (not taken) without a
        // load, so rounds through all-zero rows cost no memory round trip.
        // Returns the capacity left at the end; `chosen` gets the items taken, laid out
        // like `placed`.
        auto walk = [&](int L, int from, int at, unsigned long long &chosen) {
            // Every index is range-checked before it is used; a violation (never expected)
            // marks the instance DEFT_ERR_DEVICE instead of touching memory.
            bool broken = false;
            int c = at;
            int q = from;
            chosen = 0;
            const int d = 31 - __clz(L | 1);
            const int p = L - (1 << d);
            while (q >= 0) {
                int wv[6], tv[6];
                {
                    const bool have = L < 6 && q - L >= 0;
                    int w_l = 0, t_l = 0;
                    if (have) {
                        w_l = tb_w[q - L];
                        t_l = tb_index[q - L];
                        if (t_l < 0 || t_l >= n) { broken = true; t_l = 0; }
                    }
#pragma unroll
                    for (int i = 0; i < 6; ++i) {
                        tv[i] = __builtin_amdgcn_readlane(t_l, i);
                        wv[i] = __builtin_amdgcn_readlane(w_l, i);
                    }
                }
                int cl = c, wd = wv[0];
#pragma unroll
                for (int i = 0; i < 5; ++i) {
                    if (i < d && ((p >> (d - 1 - i)) & 1)) cl -= wv[i];
                    if (d == i + 1) wd = wv[i + 1];
                }
                uint32_t bit = 0;
                // lane L tests offered item q-d; items past the head of the list (q-d < 0) carry
                // w = 0 and are excluded here, so cl never leaves [-5*C, C]
                if (L >= 1 && q - d >= 0 && cl >= 0 && wd <= cl) {
                    const int k = cl / T, lane = cl % T, qd = q - d;  // cl >= 0 here
                    if (k < K && cl <= C) {
                        const unsigned long long nzw = tb_nz[(lane >> 6) * 64 + (qd >> 6)];
                        if ((nzw >> (qd & 63)) & 1ull) {
                            const uint32_t word = __hip_atomic_load(&kp[((size_t)qd * NW + (k >> 5)) * T + lane],
                                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            bit = (word >> (P16 ? keep_bit16(k) : (k & 31))) & 1u;
                        }
                    } else {
                        broken = true;
                    }
                }
                const unsigned long long takes = __ballot(bit != 0);
                int node = 1;
#pragma unroll
                for (int i = 0; i < 6; ++i) {
                    const int b = (int)((takes >> node) & 1ull);
                    if (b) {
                        const int t = tv[i];  // uniform
                        if (L == (t & 63)) chosen |= 1ull << (t >> 6);
                        c -= wv[i];
                    }
                    node = 2 * node + b;
                }
                q -= 6;
            }
            if (__ballot(broken) != 0ull && L == 0) a.status[inst] = DEFT_ERR_DEVICE;
            return c;
        };
        if (!caps_sweep) {
            if (serial) {
                    const int L = sl;
                unsigned long long chosen;
                const int c = walk(L, walk_from, walk_cap, chosen);
                placed |= chosen;
                while (chosen) {  // outside the walk: no store sits in its chain of loads
                    const int b = __builtin_ctzll(chosen);
                    chosen &= chosen - 1;
                    out_asg[b * 64 + L] = j;
                }
                if (L == 0) {
                    out_kv[j] = value;
                    out_kl[j] = walk_cap - c;
                    if constexpr (REC) {  // slot 1 reports the level: items left off the list, its remaining time
                        out_kv[1] = n - best.length;
                        out_kl[1] = value > 0 ? walk_cap : 0;
                    }
                }
            }
        } else if constexpr (REC) {
            // one walk per capacity, dealt out to the wavefronts of the instance; an item's
            // mask collects the capacities at which it is taken
            const int L = tid & 63;
            for (int x = tid >> 6; x < m; x += T / 64) {
                const int at = __builtin_amdgcn_readlane(sweep_cap, x);
                unsigned long long chosen;
                const int c = walk(L, swept - 1, at, chosen);
                while (chosen) {
                    const int b = __builtin_ctzll(chosen);
                    chosen &= chosen - 1;
                    atomicOr(reinterpret_cast<unsigned int *>(&out_asg[b * 64 + L]), 1u << x);
                }
                if (L == 0) {
                    out_kv[x] = __builtin_amdgcn_readlane(sweep_value, x);
                    out_kl[x] = at - c;
                }
            }
        }
        total += value;
        lds_sync<T>();
        ++s;
    }

    if (serial && sl == 0) a.total_value[inst] = total;
}

struct Variant {
    int threads, cells, chunk;
    int guard;  // cells below the row (8 scratch words + INT_MIN); items up to guard - 8 take the light path
    const void *fn;
};

#define DEFT_VARIANT(T, K, G, WPE, GUARD) \
    { T, K, G, GUARD, reinterpret_cast<const void *>(&seq_lds_kernel<T, K, G, WPE, REC, false>) }
template <bool REC>
const Variant *variant_table()
{
    static const Variant table[] = {
    DEFT_VARIANT(64, 16, 4, 5, 256),    // capacity <= 1023: one wavefront per instance, four per workgroup
    DEFT_VARIANT(256, 16, 4, 7, 256),   // <= 4095
    DEFT_VARIANT(256, 32, 4, 4, 256),   // <= 8191
    DEFT_VARIANT(512, 20, 1, 8, 128),   // <= 10239: four workgroups per CU when the row stays under 40 KB
    DEFT_VARIANT(512, 26, 1, 6, 128),   // <= 13311: with the 128-cell guard three workgroups share a CU's LDS
    DEFT_VARIANT(768, 26, 1, 6, 128),   // <= 19967: two workgroups of twelve wavefronts share a CU when the row stays under 80 KB
    DEFT_VARIANT(1024, 26, 1, 4, 256),  // <= 26623: sixteen wavefronts on a 104 KB row
    DEFT_VARIANT(1024, 38, 2, 4, 256),  // <= 38911: 153 KB of row, the most that 160 KB of LDS holds with the guard
    };
    return table;
}
#undef DEFT_VARIANT
constexpr int kNumVariants = 8;

// Rows of 16-bit cells: the same lane and slot counts (the 38-slot one is out of the 16-bit
// range); the guard zone is one pair row (T words) above 64 words that hold the scratch ints,
// and the register budget always allows the 8 wavefronts per SIMD that the smaller rows leave
// room for (two workgroups of 12 or 16 wavefronts for the two largest).
#define DEFT_VARIANT16(T, K, WPE) \
    { T, K, 2, T + 64, reinterpret_cast<const void *>(&seq_lds_kernel<T, K, 2, WPE, REC, true>) }
template <bool REC>
const Variant *variant_table16()
{
    static const Variant table[] = {
    DEFT_VARIANT16(64, 16, 8),     // capacity <= 1023
    DEFT_VARIANT16(256, 16, 8),    // <= 4095
    DEFT_VARIANT16(256, 32, 8),    // <= 8191
    DEFT_VARIANT16(320, 30, 8),    // <= 9599: 21 KB per workgroup, six workgroups of five wavefronts per CU
    DEFT_VARIANT16(512, 20, 8),    // <= 10239
    DEFT_VARIANT16(512, 26, 8),    // <= 13311: 29 KB per workgroup, four workgroups of eight wavefronts per CU
    DEFT_VARIANT16(768, 26, 6),    // <= 19967: two workgroups of twelve wavefronts
    DEFT_VARIANT16(1024, 26, 8),   // <= 26623: two workgroups of sixteen wavefronts
    };
    return table;
}
#undef DEFT_VARIANT16
constexpr int kNumVariants16 = 8;

template <int T, int K, int G, int WPE, bool REC, bool P16>
hipError_t launch_one(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                      unsigned long long *swept_cells)
{
    const LdsLayout lay{p.guard_cells, p.row_cells, p.lds_bytes / p.inst_per_wg / 4};
    const unsigned grid = (unsigned)((a.batch + p.inst_per_wg - 1) / p.inst_per_wg);
    uint32_t *keep = static_cast<uint32_t *>(scratch);
    OfferedItem *lists = reinterpret_cast<OfferedItem *>(static_cast<char *>(scratch) + p.keep_bytes);
    hipLaunchKernelGGL((seq_lds_kernel<T, K, G, WPE, REC, P16>), dim3(grid), dim3(p.wg_threads), (size_t)p.lds_bytes, st,
                       a, lay, keep, p.keep_words_per_inst, lists, p.n_pad, swept_cells);
    return hipGetLastError();
}

template <bool REC>
hipError_t launch_variant(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                          unsigned long long *swept_cells)
{
    switch (p.variant) {
    case 0: return launch_one<64, 16, 4, 5, REC, false>(p, a, scratch, st, swept_cells);
    case 1: return launch_one<256, 16, 4, 7, REC, false>(p, a, scratch, st, swept_cells);
    case 2: return launch_one<256, 32, 4, 4, REC, false>(p, a, scratch, st, swept_cells);
    case 3: return launch_one<512, 20, 1, 8, REC, false>(p, a, scratch, st, swept_cells);
    case 4: return launch_one<512, 26, 1, 6, REC, false>(p, a, scratch, st, swept_cells);
    case 5: return launch_one<768, 26, 1, 6, REC, false>(p, a, scratch, st, swept_cells);
    case 6: return launch_one<1024, 26, 1, 4, REC, false>(p, a, scratch, st, swept_cells);
    case 7: return launch_one<1024, 38, 2, 4, REC, false>(p, a, scratch, st, swept_cells);
    default: return hipErrorInvalidValue;
    }
}

template <bool REC>
hipError_t launch_variant16(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                            unsigned long long *swept_cells)
{
    switch (p.variant) {
    case 0: return launch_one<64, 16, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    case 1: return launch_one<256, 16, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    case 2: return launch_one<256, 32, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    case 3: return launch_one<320, 30, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    case 4: return launch_one<512, 20, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    case 5: return launch_one<512, 26, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    case 6: return launch_one<768, 26, 2, 6, REC, true>(p, a, scratch, st, swept_cells);
    case 7: return launch_one<1024, 26, 2, 8, REC, true>(p, a, scratch, st, swept_cells);
    default: return hipErrorInvalidValue;
    }
}

// Sets the dynamic-LDS attribute of the plan's kernel and returns how many of its
// workgroups the runtime would place on a compute unit.  The attribute belongs to the
// kernel, not to the handle, so it is set to the most any handle on this variant can ask
// for (the variant's full row): a later, smaller handle never lowers it under an earlier one.
template <bool REC, bool P16>
hipError_t prepare_variant(const SeqLdsPlan &plan, int *wg_per_cu)
{
    const Variant *table;
    if constexpr (P16) table = variant_table16<REC>(); else table = variant_table<REC>();
    const Variant &v = table[plan.variant];
    const void *fn = v.fn;
    const int full_row = (v.guard + (P16 ? v.cells / 2 : v.cells) * v.threads) * 4 * plan.inst_per_wg;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, full_row);
    if (e != hipSuccess) return e;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(wg_per_cu, fn, plan.wg_threads, (size_t)plan.lds_bytes);
}

}  // namespace

}  // namespace deft
