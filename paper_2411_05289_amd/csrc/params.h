// The parameter block every kernel of the library takes, filled by the host side of the C ABI.
// One type for every build of the kernels (see build_config.h), in the main namespace.
#pragma once
#include <stdint.h>

#include "mdsd.h"

namespace mdsd {

struct Params {
    const void* target;
    const void* draft;
    int64_t ld_t, ld_d;
    float temp_target, temp_draft;
    // log2(e) / temperature, formed once on the host: the correctly rounded quotient, which the
    // kernels would otherwise each compute again with a dozen instructions per wave
    float scale_t, scale_d;
    int B, N, V, k, depth, n_internal;
    const int32_t* first_child;
    const int32_t* tokens;
    const float* u;
    int32_t* outcome;
    int32_t* token;
    float* resid_mass;
    int32_t* flags;
    float* resid_prob;
    int32_t* accept_depth;  // path-only kernels, and the full kernels when they walk the trees themselves
    int32_t* emitted;
    // full verify kernels with the walk inside: one arrival counter per tree (all zero when the
    // kernel starts, all zero again when it ends); nullptr = the walk is a launch of its own
    int32_t* tree_count;
    // draft kernels
    int32_t* tokens_out;
    int32_t* hub_out;
    // draft-row statistics: written by the SpecHub draft kernel, read by the SpecHub verify kernel
    mdsd_row_stats* stats_out;
    const mdsd_row_stats* stats_in;
};

}  // namespace mdsd
