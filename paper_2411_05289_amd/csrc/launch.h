// Host-side launchers of the kernel families; each is defined in the source file that holds
// its kernels, so that the families compile side by side.
#pragma once
#include "node_common.h"

namespace MDSD_NS {

// spechub_resident.hip: SpecHub on logit rows that fit in registers (nit = 4, 8 or 16 chunks
// per lane); path = one workgroup per tree
void launch_spechub_resident(int dtype, int nit, bool masked, bool path, dim3 grid, dim3 block, hipStream_t st,
                             const Params& P);

// rrs_resident.hip: RRS / RRSw on logit rows in registers with the draft call's records
bool rrs_resident_covers(int dtype, int nit, bool masked);
void launch_rrs_resident(bool without_replacement, int dtype, int nit, bool masked, dim3 grid, dim3 block,
                         hipStream_t st, const Params& P);

// verify_generic_*.hip: every other case (nit = 0: rows streamed in every pass)
void launch_verify_generic_spechub(int dtype, bool logits, int nit, bool path, dim3 grid, dim3 block,
                                   hipStream_t st, const Params& P);
void launch_verify_generic_rrs(int dtype, bool logits, int nit, bool path, dim3 grid, dim3 block, hipStream_t st,
                               const Params& P);
void launch_verify_generic_rrsw(int dtype, bool logits, int nit, bool path, dim3 grid, dim3 block, hipStream_t st,
                                const Params& P);

// draft_*.hip
void launch_draft_spechub(int dtype, bool logits, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                          const Params& P);
void launch_draft_rrs(int dtype, bool logits, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                      const Params& P);
void launch_draft_rrsw(int dtype, bool logits, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                       const Params& P);

}  // namespace MDSD_NS
