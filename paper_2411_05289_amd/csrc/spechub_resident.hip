// Launchers of the SpecHub kernels for rows in registers, main build (512 threads per node).
#include "spechub_resident_kernels.h"

namespace mdsd {

template <int DT>
static void launch_spechub_resident_of(int nit, bool masked, bool path, dim3 grid, dim3 block, hipStream_t st,
                                    const Params& P)
{
#define MDSD_LAUNCH_RES3(KERNEL, N, M)                                                              \
    if (P.stats_in)                                                                                 \
        hipLaunchKernelGGL((KERNEL<DT, N, M, true>), grid, block, 0, st, P);                        \
    else                                                                                            \
        hipLaunchKernelGGL((KERNEL<DT, N, M, false>), grid, block, 0, st, P)
#define MDSD_LAUNCH_RES2(N, M)                                                                      \
    if (path) {                                                                                     \
        MDSD_LAUNCH_RES3(spechub_path_resident, N, M);                                              \
    } else {                                                                                        \
        MDSD_LAUNCH_RES3(spechub_verify_resident, N, M);                                            \
    }
#define MDSD_LAUNCH_RES(N)                                                                          \
    if (masked) {                                                                                   \
        MDSD_LAUNCH_RES2(N, true);                                                                  \
    } else {                                                                                        \
        MDSD_LAUNCH_RES2(N, false);                                                                 \
    }
    if (nit == 4) {
        MDSD_LAUNCH_RES(4);
    } else if (nit == 8) {
        MDSD_LAUNCH_RES(8);
    } else {
        MDSD_LAUNCH_RES(16);
    }
#undef MDSD_LAUNCH_RES
#undef MDSD_LAUNCH_RES2
#undef MDSD_LAUNCH_RES3
}

void launch_spechub_resident(int dtype, int nit, bool masked, bool path, dim3 grid, dim3 block, hipStream_t st,
                             const Params& P)
{
    if (dtype == MDSD_FP32)
        launch_spechub_resident_of<0>(nit, masked, path, grid, block, st, P);
    else
        launch_spechub_resident_of<1>(nit, masked, path, grid, block, st, P);
}

}  // namespace mdsd
