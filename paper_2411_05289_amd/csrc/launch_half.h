// Launchers of the verify kernels for rows in registers built for 256 threads per node (sixteen
// chunks per lane, the draft call's records at hand): four nodes share a CU instead of three, which
// is worth 4-6 % on batches that fill the chip several times over and costs as much on those that do
// not (half_verify.hip; the caller chooses by batch size).  Rows of at most kMaxChunks 16-byte
// chunks; the caller's grid has one workgroup per node.
#pragma once
#include <hip/hip_runtime.h>

#include "params.h"

namespace mdsd_half {

constexpr int kMaxChunks = 16 * 256;

// SpecHub with P.stats_in set
void launch_spechub(int dtype, bool masked, dim3 grid, hipStream_t st, const mdsd::Params& P);
// RRS / RRSw with P.stats_in set; covers(): the shapes built (the others take the 512-thread path)
bool rrs_covers(int dtype, bool masked);
void launch_rrs(bool without_replacement, int dtype, bool masked, dim3 grid, hipStream_t st, const mdsd::Params& P);

}  // namespace mdsd_half
