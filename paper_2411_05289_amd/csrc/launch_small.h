// Launchers of the builds of the generic kernels for short rows (wave_*.hip, pair_*.hip,
// quad_*.hip): a node is handled by 64, 128 or 256 threads instead of 512, four 16-byte chunks of
// the row per lane, so that no wavefront of a node is without a part of the row.  Same arguments
// as the launchers of the main build.  verify: the caller's grid has one workgroup per node (path:
// per tree); draft: the launcher sizes the grid itself (the 64-thread build puts several nodes in a
// workgroup).
#pragma once
#include <hip/hip_runtime.h>

#include "params.h"

#define MDSD_DECLARE_SMALL_BUILD(ns, threads)                                                                      \
    namespace ns {                                                                                                 \
    /* the longest row of this build, in 16-byte chunks (head of an unaligned row included) */                     \
    constexpr int kMaxChunks = 4 * (threads);                                                                      \
    void launch_verify(int method, int dtype, bool logits, bool path, dim3 grid, hipStream_t st,                   \
                       const mdsd::Params& P);                                                                     \
    void launch_draft(int method, int dtype, bool logits, hipStream_t st, const mdsd::Params& P);                  \
    }

MDSD_DECLARE_SMALL_BUILD(mdsd_wave, 64)   // one wavefront per node: up to 2040 bf16 / 1020 fp32 elements
MDSD_DECLARE_SMALL_BUILD(mdsd_pair, 128)  // two: up to 4088 / 2044
MDSD_DECLARE_SMALL_BUILD(mdsd_quad, 256)  // four: up to 8184 / 4092

#undef MDSD_DECLARE_SMALL_BUILD
