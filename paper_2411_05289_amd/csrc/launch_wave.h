// Launchers of the one-wavefront-per-node build of the generic kernels (wave_*.hip): for rows of at
// most kWaveBuildMaxChunks 16-byte chunks.  A workgroup is one or several wavefronts, each with a
// node of its own (path: a tree of its own); the launchers size the grid from the problem.
#pragma once
#include <hip/hip_runtime.h>

#include "params.h"

namespace mdsd_wave {

// four chunks per lane: 2048 bf16 or 1024 fp32 elements, less the masked head of an unaligned row
constexpr int kWaveBuildMaxChunks = 4 * 64;

void launch_verify(int method, int dtype, bool logits, bool path, dim3 grid, hipStream_t st, const mdsd::Params& P);
void launch_draft(int method, int dtype, bool logits, hipStream_t st, const mdsd::Params& P);

}  // namespace mdsd_wave
