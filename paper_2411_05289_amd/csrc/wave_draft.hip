// Draft kernels for short rows, one wavefront per node (see small_draft_launch.h).
#define MDSD_WG 64
#define MDSD_NS mdsd_wave
#define MDSD_MAX_SLABS 4
#define MDSD_NODES_PER_WG 4
#include "small_draft_launch.h"
