// Verify kernels for short rows, four wavefronts per node (see small_verify_launch.h).
#define MDSD_WG 256
#define MDSD_NS mdsd_quad
#define MDSD_MAX_SLABS 16
#define MDSD_NODES_PER_WG 1
#include "small_verify_launch.h"
