// The draft kernel built for one wavefront per node (64-thread workgroups): every method, logits
// or probabilities, rows of up to four chunks per lane held in registers.
#define MDSD_WG 64
#define MDSD_NS mdsd_wave
#define MDSD_MAX_SLABS 4
#define MDSD_NODES_PER_WG 4
#include "draft_kernel.h"

#include "launch_wave.h"

namespace mdsd_wave {

template <int METHOD>
static void launch_method(int dtype, bool logits, dim3 grid, hipStream_t st, const Params& P)
{
    if (dtype == MDSD_FP32) {
        if (logits)
            hipLaunchKernelGGL((draft_kernel<0, true, METHOD, 4>), grid, dim3(kWG * kNodesPerWG), 0, st, P);
        else
            hipLaunchKernelGGL((draft_kernel<0, false, METHOD, 4>), grid, dim3(kWG * kNodesPerWG), 0, st, P);
    } else {
        if (logits)
            hipLaunchKernelGGL((draft_kernel<1, true, METHOD, 4>), grid, dim3(kWG * kNodesPerWG), 0, st, P);
        else
            hipLaunchKernelGGL((draft_kernel<1, false, METHOD, 4>), grid, dim3(kWG * kNodesPerWG), 0, st, P);
    }
}

void launch_draft(int method, int dtype, bool logits, hipStream_t st, const Params& P)
{
    const int64_t items = (int64_t)P.B * P.N;  // one wavefront per node, numbered in one dimension
    const dim3 grid((unsigned)((items + kNodesPerWG - 1) / kNodesPerWG));
    if (method == kSpecHub)
        launch_method<kSpecHub>(dtype, logits, grid, st, P);
    else if (method == kRRS)
        launch_method<kRRS>(dtype, logits, grid, st, P);
    else
        launch_method<kRRSw>(dtype, logits, grid, st, P);
}

}  // namespace mdsd_wave
