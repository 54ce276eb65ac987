// The draft kernel built for short rows: included once by a translation unit that has set MDSD_WG
// (threads per node), MDSD_NS (the build's namespace), MDSD_MAX_SLABS and MDSD_NODES_PER_WG.
// Every method, logits or probabilities, fp32 or bf16; rows of up to four chunks per lane, held in
// registers.
#include "draft_kernel.h"

#include "launch_small.h"

namespace MDSD_NS {

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
    static_assert(kMaxChunks == 4 * kWG && kMaxSlabs * 64 >= kMaxChunks, "four chunks per lane");
    const int64_t items = (int64_t)P.B * P.N;  // nodes, numbered in one dimension
    const dim3 grid((unsigned)((items + kNodesPerWG - 1) / kNodesPerWG));
    if (method == kSpecHub)
        launch_method<kSpecHub>(dtype, logits, grid, st, P);
    else if (method == kRRS)
        launch_method<kRRS>(dtype, logits, grid, st, P);
    else
        launch_method<kRRSw>(dtype, logits, grid, st, P);
}

}  // namespace MDSD_NS
