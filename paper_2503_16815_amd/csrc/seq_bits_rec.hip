// The bit-set kernels of Algorithm 1 (DEFT_MODE_RECURSIVE on DEFT_FLAG_SUBSET_SUM handles): a
// translation unit of their own, compiled beside the sequential-mode ones.
#include "seq_bits_kernel.h"

namespace deft {

hipError_t seq_bits_rec_prepare(const SeqBitsPlan &plan) { return bits_prepare<true>(plan.variant); }

hipError_t seq_bits_rec_launch(const SeqBitsPlan &p, const BatchArgs &a, hipStream_t st) { return bits_launch<true>(p, a, st); }

}  // namespace deft
