// The draft kernel for one method.
#include "draft_kernel.h"

namespace mdsd {

void launch_draft_rrsw(int dtype, bool logits, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                       const Params& P)
{
    launch_draft_method<kRRSw>(dtype, logits, nit, masked, grid, block, st, P);
}

}  // namespace mdsd
