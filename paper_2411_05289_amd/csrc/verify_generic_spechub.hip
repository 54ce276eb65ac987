// The generic verify kernel for one method.
#include "verify_generic.h"

namespace mdsd {

void launch_verify_generic_spechub(int dtype, bool logits, int nit, bool path, dim3 grid, dim3 block, hipStream_t st,
                                   const Params& P)
{
    launch_verify_generic<kSpecHub>(dtype, logits, nit, path, grid, block, st, P);
}

}  // namespace mdsd
