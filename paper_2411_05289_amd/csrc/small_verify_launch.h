// The generic verify kernel built for short rows: included once by a translation unit that has set
// MDSD_WG (threads per node), MDSD_NS (the build's namespace), MDSD_MAX_SLABS and
// MDSD_NODES_PER_WG (1).  Every method, logits or probabilities, fp32 or bf16, full and path-only;
// rows of up to four chunks per lane, held in registers.
#include "verify_generic.h"

#include "launch_small.h"

namespace MDSD_NS {

template <int DT, bool LG, int METHOD>
static void launch_one(bool path, dim3 grid, hipStream_t st, const Params& P)
{
    if (path)
        hipLaunchKernelGGL((verify_path_kernel<DT, LG, METHOD, 4>), grid, dim3(kWG * kNodesPerWG), 0, st, P);
    else
        hipLaunchKernelGGL((verify_kernel<DT, LG, METHOD, 4>), grid, dim3(kWG * kNodesPerWG), 0, st, P);
}

template <int METHOD>
static void launch_method(int dtype, bool logits, bool path, dim3 grid, hipStream_t st, const Params& P)
{
    if (dtype == MDSD_FP32) {
        if (logits)
            launch_one<0, true, METHOD>(path, grid, st, P);
        else
            launch_one<0, false, METHOD>(path, grid, st, P);
    } else {
        if (logits)
            launch_one<1, true, METHOD>(path, grid, st, P);
        else
            launch_one<1, false, METHOD>(path, grid, st, P);
    }
}

void launch_verify(int method, int dtype, bool logits, bool path, dim3 grid, hipStream_t st, const Params& P)
{
    static_assert(kNodesPerWG == 1, "the caller's grid has one workgroup per node (path: per tree)");
    static_assert(kMaxChunks == 4 * kWG && kMaxSlabs * 64 >= kMaxChunks, "four chunks per lane");
    if (method == kSpecHub)
        launch_method<kSpecHub>(dtype, logits, path, grid, st, P);
    else if (method == kRRS)
        launch_method<kRRS>(dtype, logits, path, grid, st, P);
    else
        launch_method<kRRSw>(dtype, logits, path, grid, st, P);
}

}  // namespace MDSD_NS
