// Sequential multiple-knapsack solve for instances whose values equal their weights (the
// paper's Problem 1: a bucket's profit is its communication time), one bit per capacity cell.
//
// With v == w the DP value row[c] is the largest reachable sum not above c, so the row is
// described by the set of reachable sums: one bit per cell, and an item is a shift-and-or of
// the whole set, reach |= reach << w, 32 cells per instruction.  The selection the exact DP
// walks back (take an item at a cell only when it strictly improves the value, walk from
// the last item: among optimal subsets the one with the smallest mask) comes out of one
// more array, first[t] = the first offered item that made the sum t reachable:
//   the DP keeps item q at cell c exactly when the best sum up to c rises with item q, i.e.
//   when the target t = row_q[c] was not reachable before q; if q is not kept the target
//   stays, if it is the target becomes t - w_q.  So the walk is t = row[C]; while t > 0:
//   q = first[t], take q, t -= w_q - a chain of LDS lookups, one per item taken, with no keep
//   table and no memory round trips.
// One wavefront owns an instance (one 64-thread workgroup; no barriers).  Word i of the set
// (cells 32 i .. 32 i + 31) lives in lane i % 64, register slot i / 64, with a copy in LDS
// that the shifted operand is read from; first[] (8 or 16 bits per cell, by the handle's
// longest list) and the stage's offered items (weight, index) live in LDS too, so the kernel
// needs no scratch memory at all.  A sweep ends as soon as the capacity itself is reachable.
// Below the set a guard zone of zero words serves the reads of light items; heavier items
// clamp their word index into it.
#pragma once

#include "instance_check.h"

namespace deft {

namespace {

constexpr int kBitsGuardWords = 128;  // zero words below the set: items up to 32 * 126 cells read without clamping

__device__ __forceinline__ void wave_lds_sync()
{
    // one wavefront: LDS executes its instructions in order; only the compiler has to be
    // kept from reordering
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

template <class Op>
__device__ __forceinline__ int bits_wave_reduce(int x, Op op)
{
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0x124, 0xf, 0xf, false));  // row_ror:4
    x = op(x, __builtin_amdgcn_update_dpp(x, x, 0x128, 0xf, 0xf, false));  // row_ror:8
    return op(op(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
              op(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}
// Sum over the lanes at and above `lane`: shifts inside each row of sixteen lanes (zeros come
// in from beyond the row), then the totals of the rows above are added in.
__device__ __forceinline__ int bits_wave_suffix_sum(int x, int lane)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x101, 0xf, 0xf, true);  // row_shl:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x102, 0xf, 0xf, true);  // row_shl:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x104, 0xf, 0xf, true);  // row_shl:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x108, 0xf, 0xf, true);  // row_shl:8
    const int t1 = __builtin_amdgcn_readlane(x, 16), t2 = __builtin_amdgcn_readlane(x, 32),
              t3 = __builtin_amdgcn_readlane(x, 48);
    return x + (lane < 16 ? t1 : 0) + (lane < 32 ? t2 : 0) + (lane < 48 ? t3 : 0);
}
__device__ __forceinline__ int bits_wave_sum(int x) { return bits_wave_reduce(x, [](int a, int b) { return a + b; }); }
__device__ __forceinline__ int bits_wave_max(int x) { return bits_wave_reduce(x, [](int a, int b) { return max(a, b); }); }

// One stage's sweep over `nact` offered items (weights in lw[], LDS) at capacity C, NB words
// per lane.  Returns the stage's value (largest reachable sum <= C); first[t] is set for
// every reachable t in 1 .. C (when the sweep ends early: for every t reached so far).
// The sweep ends as soon as C itself is reachable: the value is final, and the walk from C
// only follows sums that were reached by earlier items.
// SNAP (8-bit cells, lists of 256 .. 511 items): a cell keeps the low eight bits of the
// position, and `snap` keeps the set as it stood after the item at position 255: a sum in it
// was first reached by a position below 256, any other by 256 + the cell.
// REC (Algorithm 1): lp[q] is the remaining time P_q of the level made of the items before q
// (-1 if that is negative).  The set before item q is exactly that level's, so its answer is
// the largest reachable sum <= P_q: the word that holds P_q read from LDS and, where that one
// has nothing at or below P_q, a search of the words below.  Levels are met deepest first and
// a shallower one replaces the incumbent only when strictly greater, as the recursion does
// on its way back up.  With `levels` the sweep ends, as in the sequential mode, once C (the
// whole remaining time) is reachable: no level is worth more, the levels so far are worth
// less (their sets did not hold C), and a later level is worth C exactly when its remaining
// time is C (nothing is dropped after it) - the first such entry, else the whole list, is
// the answer.  Without `levels` (the capacity sweep) it goes through the whole list.
struct BitsLevel {
    int value, length, remain;
};
template <int NB>
__device__ __forceinline__ int largest_sum_up_to(const uint32_t *set, const uint32_t (&own)[NB], int lane, int limit)
{
    const int wi = limit >> 5;
    const uint32_t x = set[wi] & (0xffffffffu >> (31 - (limit & 31)));  // every lane reads the same word
    if (x != 0) return wi * 32 + 31 - __builtin_clz(x);               // (the same in every lane)
    int best = 0;
#pragma unroll
    for (int k = 0; k < NB; ++k)
        if (own[k] != 0 && k * 64 + lane < wi) best = max(best, (k * 64 + lane) * 32 + 31 - __builtin_clz(own[k]));
    return bits_wave_max(best);
}
template <int NB, class FirstT, bool SNAP, bool REC>
__device__ __forceinline__ int sweep_bits(uint32_t *set, FirstT *first, uint32_t *snap, const int32_t *lw, const int32_t *lp,
                                          int lane, int nact, int C, BitsLevel &best, bool levels)
{
    uint32_t own[NB], need[NB];  // need: the cells of the word that are <= C
#pragma unroll
    for (int k = 0; k < NB; ++k) {
        const int cell0 = (k * 64 + lane) * 32;
        need[k] = cell0 + 31 <= C ? 0xffffffffu : cell0 > C ? 0u : (1u << (C - cell0 + 1)) - 1u;
        own[k] = (k == 0 && lane == 0) ? 1u : 0u;  // the empty sum
        set[k * 64 + lane] = own[k];
        if constexpr (SNAP) snap[k * 64 + lane] = 0xffffffffu;  // until position 255 has been swept: everything
    }
    wave_lds_sync();
    const int c_lane = (C >> 5) & 63;
    const uint32_t c_bit = 1u << (C & 31);
    for (int q0 = 0; q0 < nact; q0 += 64) {
        const int wchunk = q0 + lane < nact ? lw[q0 + lane] : 0;  // 64 weights in a register
        const int pchunk = REC && q0 + lane < nact ? lp[q0 + lane] : -1;
        const int q1 = min(q0 + 64, nact);
        for (int q = q0; q < q1; ++q) {
            const int w = __builtin_amdgcn_readlane(wchunk, q & 63);
            if constexpr (REC) {
                const int probe_at = __builtin_amdgcn_readlane(pchunk, q & 63);
                if (probe_at >= 0) {
                    const int level_value = largest_sum_up_to<NB>(set, own, lane, probe_at);
                    if (level_value > best.value) best = BitsLevel{level_value, q, probe_at};
                }
            }
            // new word i = old cells 32 i - w .. 32 i - w + 31: two neighbouring old words, funnel-shifted
            const int ws = w >> 5, bs = w & 31;
            const int sh = (32 - bs) & 31;
            const int base = lane - ws - (bs ? 1 : 0);  // old word below the pair of slot 0
            uint32_t fresh[NB];
            uint32_t any = 0;
            if (ws + 2 <= kBitsGuardWords) {
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    const uint32_t lo = set[base + k * 64], hi = set[base + k * 64 + 1];
                    const uint32_t nw = own[k] | __builtin_amdgcn_alignbit(hi, lo, sh);
                    fresh[k] = nw & ~own[k] & need[k];
                    own[k] = nw;
                    any |= fresh[k];
                }
            } else {
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    const uint32_t lo = set[max(base + k * 64, -kBitsGuardWords)];
                    const uint32_t hi = set[max(base + k * 64 + 1, -kBitsGuardWords)];
                    const uint32_t nw = own[k] | __builtin_amdgcn_alignbit(hi, lo, sh);
                    fresh[k] = nw & ~own[k] & need[k];
                    own[k] = nw;
                    any |= fresh[k];
                }
            }
            wave_lds_sync();  // the old set has been read
            if (__builtin_amdgcn_ballot_w64(any != 0) != 0ull) {
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    unsigned long long who = __builtin_amdgcn_ballot_w64(fresh[k] != 0);
                    if (who == 0ull) continue;  // nobody reached anything in this slot
                    set[k * 64 + lane] = own[k];
                    // Item q is the first to reach these sums.  Few words hold fresh bits (an item
                    // mostly extends the set by a run of sums at its top), so the words are taken
                    // one pair at a time and their bits are spread over the lanes: lane b of
                    // either half of the wavefront marks cell b of its half's word.
                    do {
                        const int l0 = __builtin_ctzll(who);
                        who &= who - 1;
                        int l1 = l0;  // (an odd count: both halves mark the same word)
                        if (who != 0ull) {
                            l1 = __builtin_ctzll(who);
                            who &= who - 1;
                        }
                        const uint32_t bits0 = __builtin_amdgcn_readlane(fresh[k], l0);
                        const uint32_t bits1 = __builtin_amdgcn_readlane(fresh[k], l1);
                        const int l = lane < 32 ? l0 : l1;
                        const uint32_t bits = lane < 32 ? bits0 : bits1;
                        if ((bits >> (lane & 31)) & 1u) first[(k * 64 + l) * 32 + (lane & 31)] = (FirstT)q;
                    } while (who != 0ull);
                }
                // (C's word is in the last slot: NB is the smallest count that covers it)
                const bool reached = lane == c_lane && (fresh[NB - 1] & c_bit) != 0;
                wave_lds_sync();  // the new set is visible
                if (__builtin_amdgcn_ballot_w64(reached) != 0ull) {
                    if constexpr (!REC) {
                        return C;
                    } else if (levels) {
                        int found = nact;  // the whole list
                        for (int c0 = (q + 1) & ~63; c0 < nact; c0 += 64) {
                            const int e = c0 + lane;
                            const unsigned long long hit =
                                __builtin_amdgcn_ballot_w64(e > q && e < nact && lp[e] == C);
                            if (hit != 0ull) {
                                found = c0 + __builtin_ctzll(hit);
                                break;
                            }
                        }
                        best = BitsLevel{C, found, C};
                        return C;
                    }
                }
            }
            if constexpr (SNAP) {
                if (q == 255) {
#pragma unroll
                    for (int k = 0; k < NB; ++k) snap[k * 64 + lane] = own[k];
                }
            }
        }
    }
    int top = 0;
#pragma unroll
    for (int k = 0; k < NB; ++k) {
        const uint32_t x = own[k] & need[k];
        if (x) top = max(top, (k * 64 + lane) * 32 + 31 - __builtin_clz(x));
    }
    return bits_wave_max(top);
}

template <int N, class FirstT, bool SNAP, bool REC>
__device__ __forceinline__ int sweep_bits_dispatch(int nb, uint32_t *set, FirstT *first, uint32_t *snap, const int32_t *lw,
                                                   const int32_t *lp, int lane, int nact, int C, BitsLevel &best, bool levels)
{
    if (nb == N) {
        return sweep_bits<N, FirstT, SNAP, REC>(set, first, snap, lw, lp, lane, nact, C, best, levels);
    } else if constexpr (N > 1) {
        return sweep_bits_dispatch<N - 1, FirstT, SNAP, REC>(nb, set, first, snap, lw, lp, lane, nact, C, best, levels);
    }
    return 0;
}

// K: words per lane the variant is compiled for (capacities up to 2048 K - 1).
// LDS: [guard zeros][set: row_words][first: first_ints ints][lw: n_pad][li: n_pad]
//      [lp: n_pad, if REC][snap: row_words, if SNAP]
// FirstT: the cell type of first[].  An 8-bit cell serves lists of at most 255 items, with
// SNAP (one snapshot of the set) of at most 511, and halves the instance's LDS, so that
// about twice as many instances share a compute unit.
// REC = false: DEFT_MODE_SEQUENTIAL.  REC = true, chosen by a.mode at run time:
// DEFT_MODE_RECURSIVE (Algorithm 1 on one window: every item offered in generation order, the
// best level tracked during the sweep, the walk started at that level's value) and
// DEFT_MODE_CAPACITY_SWEEP (one sweep at the largest capacity, one walk per capacity).
template <int K, class FirstT, bool SNAP, bool REC>
__global__ void __launch_bounds__(64) seq_bits_kernel(BatchArgs a, int row_words, int first_ints, int n_pad)
{
    extern __shared__ __align__(16) int32_t lds_bits[];
    const int inst = blockIdx.x, lane = threadIdx.x;
    uint32_t *set = reinterpret_cast<uint32_t *>(lds_bits) + kBitsGuardWords;
    FirstT *first = reinterpret_cast<FirstT *>(set + row_words);
    int32_t *lw = reinterpret_cast<int32_t *>(set + row_words) + first_ints;
    int32_t *li = lw + n_pad;
    int32_t *lp = li + n_pad;
    uint32_t *snap = reinterpret_cast<uint32_t *>(lp + (REC ? n_pad : 0));

    // Everything whose address follows from the instance number alone is fetched at once: the
    // kernel's entry is one memory round trip (two for lists of more than 64 items).
    const int32_t *__restrict__ W = a.weights + (size_t)inst * a.item_stride;
    const int32_t *__restrict__ V = a.values + (size_t)inst * a.item_stride;
    const int32_t *cap = a.capacities + (size_t)inst * a.knap_stride;
    const int32_t *ord = a.fill_order ? a.fill_order + (size_t)inst * a.knap_stride : nullptr;
    const int w_first = lane < a.item_stride ? W[lane] : 0;
    const int v_first = lane < a.item_stride ? V[lane] : 0;
    const int cap_raw = lane < a.knap_stride ? cap[lane] : 0;
    const int ord_raw = ord && lane < a.knap_stride ? ord[lane] : lane;
    const int n = a.n_items[inst], m = a.n_knapsacks[inst];
    const bool caps_sweep = REC && a.mode == DEFT_MODE_CAPACITY_SWEEP;  // (the REC kernels serve both modes)

    // Input checks, in the order every kernel of the library reports them: invalid data, the
    // handle's limits, overflow of the value sum; then the handle's promise that every value
    // equals its weight.
    int status = DEFT_OK;
    {
        uint32_t flags = 0;
        unsigned long long vs = 0;
        bool differs = false;
        if (n < 0 || n > a.item_stride || m < 0 || m > a.knap_stride || (REC && (caps_sweep ? m > 31 : m != 1))) {
            flags = 1;
        } else {
            for (int i0 = 0; i0 < n; i0 += 64) {
                const int i = i0 + lane;
                if (i < n) {
                    const int w = i0 == 0 ? w_first : W[i], v = i0 == 0 ? v_first : V[i];
                    bool bad = w < 1 || v < 0;
                    if constexpr (REC) bad = bad || (!caps_sweep && a.drop_time[(size_t)inst * a.item_stride + i] < 0);
                    if (bad) flags |= 1; else vs += (unsigned)v;
                    differs = differs || v != w;
                }
            }
            unsigned long long seen = 0;
            if (lane < m) {
                if (cap_raw < 0) flags |= 1; else if (cap_raw > a.max_capacity) flags |= 2;
                if (ord_raw < 0 || ord_raw >= m) flags |= 1; else seen = 1ull << ord_raw;
            }
            // a fill order names every knapsack once: m entries in range with m distinct values
            auto bit_or = [](int x, int y) { return x | y; };
            const int seen_lo = bits_wave_reduce((int)(uint32_t)seen, bit_or);
            const int seen_hi = bits_wave_reduce((int)(uint32_t)(seen >> 32), bit_or);
            if ((int)(__popc((uint32_t)seen_lo) + __popc((uint32_t)seen_hi)) != m) flags |= 1;
        }
        // (a lane adds at most 64 values below 2^31: three 16-bit pieces keep the sums in range)
        const unsigned long long total_v = (unsigned long long)(unsigned)bits_wave_sum((int)(vs & 0xffffu)) +
                                           ((unsigned long long)(unsigned)bits_wave_sum((int)((vs >> 16) & 0xffffu)) << 16) +
                                           ((unsigned long long)(unsigned)bits_wave_sum((int)(vs >> 32)) << 32);
        if (__builtin_amdgcn_ballot_w64((flags & 1) != 0) != 0ull) status = DEFT_ERR_INVALID_ARG;
        else if (__builtin_amdgcn_ballot_w64((flags & 2) != 0) != 0ull) status = DEFT_ERR_LIMIT;
        else if (total_v >= (1ull << 31)) status = DEFT_ERR_OVERFLOW;
        else if (__builtin_amdgcn_ballot_w64(differs) != 0ull) status = DEFT_ERR_INVALID_ARG;
    }
    clear_outputs(a, inst, status);
    if (status != DEFT_OK) return;

    for (int i = lane; i < kBitsGuardWords; i += 64) lds_bits[i] = 0;
    const int cap_l = lane < m ? cap_raw : 0;
    const int ord_l = lane < m ? ord_raw : lane;
    int32_t *out_asg = a.assignment + (size_t)inst * a.item_stride;
    int32_t *out_kv = a.knap_value + (size_t)inst * a.knap_stride;
    int32_t *out_kl = a.knap_load + (size_t)inst * a.knap_stride;
    wave_lds_sync();

    if constexpr (REC) {
        if (caps_sweep) {
            // The capacity sweep: one sweep over the whole list at the largest capacity; the
            // final set answers every capacity (the largest reachable sum not above it), and the
            // chain through first[] from that sum is the selection the DP would walk back at that
            // capacity.  Lane x takes capacity x: all the walks run side by side, each lane
            // following its own chain through LDS, and an item's mask collects the capacities
            // at which it is taken.
            const int cap_max = bits_wave_max(cap_l);
            if (n == 0 || m == 0) return;  // (every output is already zero)
            for (int i = lane; i < n; i += 64) {
                lw[i] = i < 64 ? w_first : W[i];
                lp[i] = -1;  // no level ends anywhere
            }
            wave_lds_sync();
            BitsLevel unused{0, 0, 0};
            const int nb = (cap_max / 32 + 64) / 64;
            (void)sweep_bits_dispatch<K, FirstT, SNAP, true>(nb, set, first, snap, lw, lp, lane, n, cap_max, unused, false);
            int t = 0;
            if (lane < m) {
                int wi = cap_l >> 5;
                uint32_t x = set[wi] & (0xffffffffu >> (31 - (cap_l & 31)));
                while (x == 0) x = set[--wi];  // (word 0 holds the empty sum)
                t = wi * 32 + 31 - __builtin_clz(x);
            }
            const int value = t;
            __threadfence_block();  // the cleared masks are in place before bits are set in them
            int guard = n;          // (a chain is never longer than the list)
            while (__builtin_amdgcn_ballot_w64(t > 0) != 0ull && guard-- > 0) {
                if (t > 0) {
                    int q = first[t];
                    if constexpr (SNAP) q += ((snap[t >> 5] >> (t & 31)) & 1u) ? 0 : 256;
                    q = min(q, n - 1);
                    atomicOr(reinterpret_cast<unsigned int *>(&out_asg[q]), 1u << lane);
                    t -= lw[q];
                }
            }
            if (lane < m) {
                out_kv[lane] = value;
                out_kl[lane] = value;
            }
            const int at_largest = bits_wave_max(value);
            const bool broken = __builtin_amdgcn_ballot_w64(t != 0) != 0ull;  // (never expected)
            if (lane == 0) {
                a.total_value[inst] = at_largest;
                if (broken) a.status[inst] = DEFT_ERR_DEVICE;
            }
            return;
        }
        // Algorithm 1: the whole list is offered in generation order (an item heavier than the
        // remaining time changes nothing, but the levels are counted in list positions).
        // Entry i gets P_i = R - sum of drop[t] over t >= i, from a suffix sum taken 64 items at
        // a time from the end of the list.  Only "how far below R" matters and R is at most
        // 2^16: a drop time is clamped just above 2^24 and so is the running sum, which keeps
        // everything in 32 bits and exact wherever the remaining time is not negative.
        constexpr int kOver = (1 << 24) + 1;
        const int C = __builtin_amdgcn_readlane(cap_l, 0);
        const int32_t *drop = a.drop_time + (size_t)inst * a.item_stride;
        int behind = 0;  // sum of drop over the chunks already done (uniform)
        for (int i0 = (n - 1) & ~63; i0 >= 0 && n > 0; i0 -= 64) {
            const int i = i0 + lane;
            const int x = bits_wave_suffix_sum(i < n ? min(drop[i], kOver) : 0, lane);
            if (i < n) {
                const int left = C - min(x + behind, kOver);
                lw[i] = i0 == 0 ? w_first : W[i];
                li[i] = i;
                lp[i] = left < 0 ? -1 : left;
            }
            behind = min(behind + __builtin_amdgcn_readlane(x, 0), kOver);
        }
        wave_lds_sync();
        BitsLevel best{0, 0, 0};
        int value = 0;
        if (n > 0) {
            const int nb = (C / 32 + 64) / 64;
            value = sweep_bits_dispatch<K, FirstT, SNAP, true>(nb, set, first, snap, lw, lp, lane, n, C, best, true);
        }
        if (value > best.value) best = BitsLevel{value, n, C};  // level 0: the whole list
        // the walk from the best level's value: its chain only meets sums first reached by
        // items of that level (a sum reachable with the first q items was first reached by one of them)
        int t = best.value;
        int guard = n;
        while (t > 0 && guard-- > 0) {
            int q = first[t];
            if constexpr (SNAP) q += ((snap[t >> 5] >> (t & 31)) & 1u) ? 0 : 256;
            q = min(q, n - 1);
            if (lane == 0) out_asg[q] = 0;
            t -= lw[q];
        }
        if (lane == 0) {
            if (t != 0) a.status[inst] = DEFT_ERR_DEVICE;  // (never expected)
            out_kv[0] = best.value;
            out_kl[0] = best.value;
            out_kv[1] = n - best.length;  // the level: items left off the list, its remaining time
            out_kl[1] = best.value > 0 ? best.remain : 0;
            a.total_value[inst] = best.value;
        }
        return;
    }

    // items already placed: bit (i / 64) of lane (i % 64)
    unsigned long long placed = 0;
    long long total = 0;
    for (int s = 0; s < m; ++s) {
        const int j = __builtin_amdgcn_readlane(ord_l, s);
        const int C = __builtin_amdgcn_readlane(cap_l, j);
        // offered items: not yet placed and able to fit at all, ascending index
        int cnt = 0, unplaced = 0, offered_weight = 0;
        for (int i0 = 0; i0 < n; i0 += 64) {
            const int i = i0 + lane;
            const int w = i >= n ? 0 : i0 == 0 ? w_first : W[i];
            const bool open = i < n && ((placed >> (i0 >> 6)) & 1ull) == 0;
            const bool f = open && w <= C;
            unplaced += __popcll(__builtin_amdgcn_ballot_w64(open));
            const unsigned long long mask = __builtin_amdgcn_ballot_w64(f);
            if (f) {
                const int pos = cnt + __popcll(mask & ((1ull << lane) - 1ull));
                lw[pos] = w;
                li[pos] = i;
                offered_weight += w;
            }
            cnt += __popcll(mask);
        }
        if (unplaced == 0) break;  // every item is placed: the remaining stages stay empty
        if (cnt == 0) continue;
        wave_lds_sync();
        // (a lane's share is clamped just above the largest capacity, so that the sum stays in
        // range and still exceeds C whenever the true sum does)
        offered_weight = bits_wave_sum(min(offered_weight, (1 << 24) + 1));
        int value;
        if (offered_weight <= C) {
            // everything offered fits together: the DP takes it all (every value is positive)
            for (int p = lane; p < cnt; p += 64) {
                const int i = li[p];
                out_asg[i] = j;
            }
            for (int i0 = 0; i0 < n; i0 += 64) {
                const int i = i0 + lane;
                const int w = i >= n ? 0 : i0 == 0 ? w_first : W[i];
                if (i < n && ((placed >> (i0 >> 6)) & 1ull) == 0 && w <= C) placed |= 1ull << (i0 >> 6);
            }
            value = offered_weight;
        } else {
            const int nb = (C / 32 + 64) / 64;  // words per lane covering cells 0 .. C
            BitsLevel unused{0, 0, 0};
            value = sweep_bits_dispatch<K, FirstT, SNAP, false>(nb, set, first, snap, lw, lp, lane, cnt, C, unused, false);
            // the walk: every lane follows the same chain; the lane that owns an item's bit marks it
            int t = value;
            int guard = cnt;  // (a chain is never longer than the list)
            while (t > 0 && guard-- > 0) {
                int q = first[t];
                if constexpr (SNAP) q += ((snap[t >> 5] >> (t & 31)) & 1u) ? 0 : 256;
                const int w = lw[min(q, cnt - 1)], i = li[min(q, cnt - 1)];
                if (lane == (i & 63)) placed |= 1ull << (i >> 6);
                if (lane == 0) out_asg[i] = j;
                t -= w;
            }
            if (t != 0 && lane == 0) a.status[inst] = DEFT_ERR_DEVICE;  // (never expected)
        }
        if (lane == 0) {
            out_kv[j] = value;
            out_kl[j] = value;
        }
        total += value;
        wave_lds_sync();
    }
    if (lane == 0) a.total_value[inst] = total;
}

// Compiled words-per-lane counts (capacities up to 2048 K - 1), each with the three layouts of first[].
constexpr int kBitsWords[] = {2, 5, 7, 10, 13, 19, 32};
constexpr int kNumBitsWords = 7;

// mode: 0 = 16-bit cells, 1 = 8-bit cells, 2 = 8-bit cells and the snapshot
template <int K, bool REC, class F>
auto with_bits_mode(int mode, F &&f)
{
    switch (mode) {
    case 0: return f(&seq_bits_kernel<K, uint16_t, false, REC>);
    case 1: return f(&seq_bits_kernel<K, uint8_t, false, REC>);
    default: return f(&seq_bits_kernel<K, uint8_t, true, REC>);
    }
}
template <bool REC, class F>
auto with_bits_kernel(int variant, F &&f)
{
    switch (variant / 3) {
    case 0: return with_bits_mode<2, REC>(variant % 3, f);
    case 1: return with_bits_mode<5, REC>(variant % 3, f);
    case 2: return with_bits_mode<7, REC>(variant % 3, f);
    case 3: return with_bits_mode<10, REC>(variant % 3, f);
    case 4: return with_bits_mode<13, REC>(variant % 3, f);
    case 5: return with_bits_mode<19, REC>(variant % 3, f);
    case 6: return with_bits_mode<32, REC>(variant % 3, f);
    default: return f(static_cast<void (*)(BatchArgs, int, int, int)>(nullptr));
    }
}

template <bool REC>
hipError_t bits_prepare(int variant)
{
    // the attribute belongs to the kernel, not to the handle: the most any handle may ask for
    // (a compute unit's LDS less a small allowance)
    return with_bits_kernel<REC>(variant, [](auto fn) {
        if (!fn) return hipErrorInvalidValue;
        return hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   160 * 1024 - 256);
    });
}

template <bool REC>
hipError_t bits_launch(const SeqBitsPlan &p, const BatchArgs &a, hipStream_t st)
{
    return with_bits_kernel<REC>(p.variant, [&](auto fn) {
        if (!fn) return hipErrorInvalidValue;
        hipLaunchKernelGGL(fn, dim3((unsigned)a.batch), dim3(64), (size_t)(REC ? p.lds_bytes_rec : p.lds_bytes), st, a,
                           p.row_words, p.first_ints, p.n_pad);
        return hipGetLastError();
    });
}

}  // namespace

}  // namespace deft
