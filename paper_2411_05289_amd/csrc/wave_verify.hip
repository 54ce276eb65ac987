// The generic verify kernel built for one wavefront per node (64-thread workgroups): every method,
// logits or probabilities, rows of up to four chunks per lane held in registers.
#define MDSD_WG 64
#define MDSD_NS mdsd_wave
#define MDSD_MAX_SLABS 4
#define MDSD_NODES_PER_WG 1
#include "verify_generic.h"

#include "launch_wave.h"

namespace mdsd_wave {

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
    if (method == kSpecHub)
        launch_method<kSpecHub>(dtype, logits, path, grid, st, P);
    else if (method == kRRS)
        launch_method<kRRS>(dtype, logits, path, grid, st, P);
    else
        launch_method<kRRSw>(dtype, logits, path, grid, st, P);
}

}  // namespace mdsd_wave
