// The verify kernels for rows in registers, 256 threads per node (see launch_half.h).
#define MDSD_WG 256
#define MDSD_NS mdsd_half
#define MDSD_MAX_SLABS 64
#include "spechub_resident_kernels.h"
#include "rrs_resident_kernels.h"

#include "launch_half.h"

namespace mdsd_half {

static_assert(kMaxChunks == 16 * kWG && kMaxSlabs * 64 >= kMaxChunks, "sixteen chunks per lane");

void launch_spechub(int dtype, bool masked, dim3 grid, hipStream_t st, const Params& P)
{
    const dim3 block(kWG);
    if (dtype == MDSD_FP32) {
        if (masked)
            hipLaunchKernelGGL((spechub_verify_resident<0, 16, true, true>), grid, block, 0, st, P);
        else
            hipLaunchKernelGGL((spechub_verify_resident<0, 16, false, true>), grid, block, 0, st, P);
    } else {
        if (masked)
            hipLaunchKernelGGL((spechub_verify_resident<1, 16, true, true>), grid, block, 0, st, P);
        else
            hipLaunchKernelGGL((spechub_verify_resident<1, 16, false, true>), grid, block, 0, st, P);
    }
}

// fp32 rows masked or not, bf16 rows that need no masking (as in the main build)
bool rrs_covers(int dtype, bool masked) { return dtype == MDSD_FP32 || !masked; }

template <bool WO>
static void launch_rrs_of(int dtype, bool masked, dim3 grid, hipStream_t st, const Params& P)
{
    const dim3 block(kWG);
    if (dtype == MDSD_FP32) {
        if (masked)
            hipLaunchKernelGGL((rrs_verify_resident<0, 16, true, WO>), grid, block, 0, st, P);
        else
            hipLaunchKernelGGL((rrs_verify_resident<0, 16, false, WO>), grid, block, 0, st, P);
    } else {
        hipLaunchKernelGGL((rrs_verify_resident<1, 16, false, WO>), grid, block, 0, st, P);
    }
}

void launch_rrs(bool without_replacement, int dtype, bool masked, dim3 grid, hipStream_t st, const Params& P)
{
    if (without_replacement)
        launch_rrs_of<true>(dtype, masked, grid, st, P);
    else
        launch_rrs_of<false>(dtype, masked, grid, st, P);
}

}  // namespace mdsd_half
