// Verify kernels for short rows, two wavefronts per node (see small_verify_launch.h).
#define MDSD_WG 128
#define MDSD_NS mdsd_pair
#define MDSD_MAX_SLABS 8
#define MDSD_NODES_PER_WG 1
#include "small_verify_launch.h"
