// Which build of the kernels a translation unit holds.  The device code is written for a
// workgroup of MDSD_WG threads (kWaves = MDSD_WG / 64 wavefronts sharing one node) and lives in
// namespace MDSD_NS.  The library's main build is 512 threads in namespace mdsd; the files
// wave_*.hip build the generic kernels a second time for 64 threads in namespace mdsd_wave: one
// wavefront per node, for vocabularies of a few hundred tokens, where a 512-thread workgroup
// would have seven of its eight wavefronts hold no part of the row.
#pragma once

#ifndef MDSD_WG
#define MDSD_WG 512
#endif
#ifndef MDSD_NS
#define MDSD_NS mdsd
#endif
// nodes that share a workgroup (each with MDSD_WG threads of its own); more than one only with
// MDSD_WG == 64: the dispatcher starts about four times as many wavefronts per second in
// workgroups of four as in workgroups of one
#ifndef MDSD_NODES_PER_WG
#define MDSD_NODES_PER_WG 1
#endif
// slab sums a node keeps in LDS: bounds the vocabulary (64 chunks of 16 bytes per slab)
#ifndef MDSD_MAX_SLABS
#define MDSD_MAX_SLABS 2048
#endif
