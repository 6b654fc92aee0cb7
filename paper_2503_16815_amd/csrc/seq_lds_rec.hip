// Algorithm 1 (RecursiveKnapsack) on the LDS-resident row: the kernels of
// seq_lds_kernel.h instantiated with REC = true, under the plan made for the
// sequential mode (same variants, same scratch).
#include "seq_lds_kernel.h"

namespace deft {

hipError_t seq_lds_rec_prepare(const SeqLdsPlan &plan)
{
    if (plan.packed16) return seq_lds_p16_rec_prepare(plan);
    int nb = 0;
    const hipError_t e = prepare_variant<true, false>(plan, &nb);
    if (e != hipSuccess) return e;
    return nb > 0 ? hipSuccess : hipErrorInvalidConfiguration;
}

hipError_t seq_lds_rec_launch(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                              unsigned long long *swept_cells)
{
    if (p.packed16) return seq_lds_p16_rec_launch(p, a, scratch, st, swept_cells);
    return launch_variant<true>(p, a, scratch, st, swept_cells);
}

}  // namespace deft
