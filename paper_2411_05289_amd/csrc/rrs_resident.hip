// Launchers of the RRS / RRSw kernels for rows in registers, main build (512 threads per node).
#include "rrs_resident_kernels.h"

namespace mdsd {

// which shapes the RRS kernel for rows in registers is built for (the others would spill; they
// take the generic kernel): fp32 in every size, bf16 only for rows that need no masking
bool rrs_resident_covers(int dtype, int nit, bool masked)
{
    return nit > 0 && (dtype == MDSD_FP32 || !masked);
}
template <bool WO>
static void launch_rrs_resident_of(int dtype, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                                const Params& P)
{
#define MDSD_LAUNCH_RRS(DT, N, M) hipLaunchKernelGGL((rrs_verify_resident<DT, N, M, WO>), grid, block, 0, st, P)
    if (dtype == MDSD_FP32) {
        if (nit == 4) {
            if (masked) MDSD_LAUNCH_RRS(0, 4, true); else MDSD_LAUNCH_RRS(0, 4, false);
        } else if (nit == 8) {
            if (masked) MDSD_LAUNCH_RRS(0, 8, true); else MDSD_LAUNCH_RRS(0, 8, false);
        } else {
            if (masked) MDSD_LAUNCH_RRS(0, 16, true); else MDSD_LAUNCH_RRS(0, 16, false);
        }
    } else {
        if (nit == 4)
            MDSD_LAUNCH_RRS(1, 4, false);
        else if (nit == 8)
            MDSD_LAUNCH_RRS(1, 8, false);
        else
            MDSD_LAUNCH_RRS(1, 16, false);
    }
#undef MDSD_LAUNCH_RRS
}

void launch_rrs_resident(bool without_replacement, int dtype, int nit, bool masked, dim3 grid, dim3 block,
                         hipStream_t st, const Params& P)
{
    if (without_replacement)
        launch_rrs_resident_of<true>(dtype, nit, masked, grid, block, st, P);
    else
        launch_rrs_resident_of<false>(dtype, nit, masked, grid, block, st, P);
}

}  // namespace mdsd
