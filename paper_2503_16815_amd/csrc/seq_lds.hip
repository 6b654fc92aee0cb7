// Sequential mode with the capacity row resident in LDS: variant choice for the
// create-time limits, and the launch of the kernels in seq_lds_kernel.h.
#include "seq_lds_kernel.h"

namespace deft {

// LDS is handed out in granules of 1280 bytes, 128 of them per compute unit (measured:
// three 53760-byte workgroups run together on a CU, three 54016-byte ones do not, whatever
// the occupancy query says).
constexpr int kLdsGranule = 1280, kLdsGranulesPerCu = 128;

bool seq_lds_plan(int32_t max_capacity, int32_t max_items, int32_t max_knapsacks, int32_t max_batch,
                  int32_t lds_per_wg_bytes, bool packed16, SeqLdsPlan *plan)
{
    const int32_t n_pad = (max_items + 7) & ~7;  // list entries per stage (whole 64-byte lines)
    const int count = packed16 ? kNumVariants16 : kNumVariants;
    for (int i = 0; i < count; ++i) {
        const Variant &v = packed16 ? variant_table16<false>()[i] : variant_table<false>()[i];
        const int guard = v.guard;
        // register slots needed by lane 0, rounded up to whole chunks
        int64_t slots = ((int64_t)max_capacity / v.threads + v.chunk) / v.chunk * v.chunk;
        if (slots > v.cells) continue;
        const int cells_per_word = packed16 ? 2 : 1;  // LDS words hold one cell, or a pair of 16-bit cells
        slots /= cells_per_word;
        // after a stage's sweep the row's LDS stages the walk's data: two ints per list
        // entry and one 64-bit word per lane; a long item list on a short row gets the LDS
        // it needs for that, up to the variant's full row
        int64_t row_cells = slots * v.threads;
        const int64_t staging = 2 * (int64_t)n_pad + 2 * v.threads;
        if (row_cells < staging) row_cells = (staging + v.threads - 1) / v.threads * v.threads;
        if (row_cells > (int64_t)v.cells / cells_per_word * v.threads) continue;
        const int64_t per_inst = (guard + row_cells) * 4;
        const int inst_per_wg = v.threads == 64 ? 4 : 1;
        const int64_t lds = per_inst * inst_per_wg;
        if (lds > lds_per_wg_bytes) continue;
        plan->packed16 = packed16 ? 1 : 0;
        plan->variant = i;
        plan->threads = v.threads;
        plan->cells_per_thread = v.cells;
        plan->keep_words = (v.cells + 31) / 32;
        plan->guard_cells = guard;
        plan->row_cells = (int32_t)row_cells;
        plan->n_pad = n_pad;
        plan->lds_bytes = (int32_t)lds;
        plan->wg_threads = v.threads == 64 ? 256 : v.threads;
        plan->inst_per_wg = inst_per_wg;
        plan->wg_per_cu = 0;
        plan->keep_words_per_inst = (int64_t)max_items * plan->keep_words * v.threads;
        plan->keep_bytes = plan->keep_words_per_inst * 4 * max_batch;
        plan->scratch_bytes = plan->keep_bytes + (int64_t)max_batch * max_knapsacks * n_pad * (int64_t)sizeof(OfferedItem);
        return true;
    }
    return false;
}

hipError_t seq_lds_prepare(SeqLdsPlan *plan)
{
    int nb = 0;
    const hipError_t e = plan->packed16 ? seq_lds_p16_prepare(*plan, &nb) : prepare_variant<false, false>(*plan, &nb);
    if (e != hipSuccess) return e;
    const int by_lds = kLdsGranulesPerCu / ((plan->lds_bytes + kLdsGranule - 1) / kLdsGranule);
    plan->wg_per_cu = nb < by_lds ? nb : by_lds;
    return plan->wg_per_cu > 0 ? hipSuccess : hipErrorInvalidConfiguration;
}

hipError_t seq_lds_launch(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                          unsigned long long *swept_cells)
{
    if (p.packed16) return seq_lds_p16_launch(p, a, scratch, st, swept_cells);
    return launch_variant<false>(p, a, scratch, st, swept_cells);
}

}  // namespace deft
