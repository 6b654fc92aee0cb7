// The bit-set kernels of the sequential mode (DEFT_FLAG_SUBSET_SUM handles) and the plan both
// sets of bit-set kernels share.
#include "seq_bits_kernel.h"

namespace deft {

bool seq_bits_plan(int32_t max_capacity, int32_t max_items, int32_t lds_per_wg_bytes, SeqBitsPlan *plan)
{
    const int32_t n_pad = (max_items + 7) & ~7;
    // a cell holds a position in the stage's list
    const int mode = max_items <= 255 ? 1 : max_items <= 511 ? 2 : 0;
    const int cell_bytes = mode == 0 ? 2 : 1;
    for (int i = 0; i < kNumBitsWords; ++i) {
        const int K = kBitsWords[i];
        if ((int64_t)max_capacity > (int64_t)K * 2048 - 1) continue;
        const int64_t row_words = (int64_t)K * 64;
        const int64_t first_ints = (((int64_t)max_capacity + 1) * cell_bytes + 3) / 4;  // cells 0 .. max_capacity
        const int64_t lds = (kBitsGuardWords + row_words + first_ints + 2 * (int64_t)n_pad + (mode == 2 ? row_words : 0)) * 4;
        if (lds > lds_per_wg_bytes - 256) return false;
        plan->variant = 3 * i + mode;
        plan->words_per_lane = K;
        plan->row_words = (int32_t)row_words;
        plan->first_ints = (int32_t)first_ints;
        plan->n_pad = n_pad;
        plan->lds_bytes = (int32_t)lds;
        // Algorithm 1 keeps one more list (the levels' remaining times); where that does not
        // fit any more, the mode stays on the LDS-row kernels
        const int64_t lds_rec = lds + (int64_t)n_pad * 4;
        plan->lds_bytes_rec = lds_rec > lds_per_wg_bytes - 256 ? 0 : (int32_t)lds_rec;
        return true;
    }
    return false;
}

hipError_t seq_bits_prepare(const SeqBitsPlan &plan) { return bits_prepare<false>(plan.variant); }

hipError_t seq_bits_launch(const SeqBitsPlan &p, const BatchArgs &a, hipStream_t st) { return bits_launch<false>(p, a, st); }

}  // namespace deft
