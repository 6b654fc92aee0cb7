// Algorithm 1 and the capacity sweep on rows of 16-bit cells: the kernels of
// seq_lds_kernel.h with REC = true and P16 = true (own translation unit).
#include "seq_lds_kernel.h"

namespace deft {

hipError_t seq_lds_p16_rec_prepare(const SeqLdsPlan &plan)
{
    int nb = 0;
    const hipError_t e = prepare_variant<true, true>(plan, &nb);
    if (e != hipSuccess) return e;
    return nb > 0 ? hipSuccess : hipErrorInvalidConfiguration;
}

hipError_t seq_lds_p16_rec_launch(const SeqLdsPlan &p, const BatchArgs &a, void *scratch, hipStream_t st,
                                  unsigned long long *swept_cells)
{
    return launch_variant16<true>(p, a, scratch, st, swept_cells);
}

}  // namespace deft
