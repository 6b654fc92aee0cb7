// The sequential mode on rows of 16-bit cells (values equal to weights, capacities up to
// 26623): the kernels of seq_lds_kernel.h instantiated with P16 = true, in a translation unit
// of their own so that they compile beside the 32-bit ones.
#include "seq_lds_kernel.h"

namespace deft {

hipError_t seq_lds_p16_prepare(const SeqLdsPlan &plan, int *wg_per_cu)
{
    return prepare_variant<false, true>(plan, wg_per_cu);
}

hipError_t seq_lds_p16_launch(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                              unsigned long long *swept_cells)
{
    return launch_variant16<false>(p, a, scratch, st, swept_cells);
}

}  // namespace deft
