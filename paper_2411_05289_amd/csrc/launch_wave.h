// Launchers of the one-wavefront-per-node build of the generic kernels (wave_*.hip): for rows of at
// most kWaveBuildMaxChunks 16-byte chunks.  Same arguments as the launchers of the main build;
// workgroups are 64 threads, one per node (path: one per tree).
#pragma once
#include <hip/hip_runtime.h>

#include "params.h"

namespace mdsd_wave {

// four chunks per lane: 2048 bf16 or 1024 fp32 elements, less the masked head of an unaligned row
constexpr int kWaveBuildMaxChunks = 4 * 64;

void launch_verify(int method, int dtype, bool logits, bool path, dim3 grid, hipStream_t st, const mdsd::Params& P);
void launch_draft(int method, int dtype, bool logits, dim3 grid, hipStream_t st, const mdsd::Params& P);

}  // namespace mdsd_wave
