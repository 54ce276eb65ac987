// Helpers for rows held in registers: picking a register chunk whose number is
// only known at run time without pushing the row out of registers.
#pragma once
#include <limits.h>

#include "scan_core.h"

namespace MDSD_NS {

// register chunk `it` of this lane, `it` known only at run time
template <int NIT>
__device__ __forceinline__ uint4 select_chunk(const uint4 (&d)[NIT], int it)
{
    // component by component: selecting whole uint4 objects makes the compiler pick an
    // address instead of a value, which would push the row out of registers
    uint32_t x = d[0].x, y = d[0].y, z = d[0].z, w = d[0].w;
#pragma unroll
    for (int i = 1; i < NIT; ++i) {
        const bool c = it == i;
        x = c ? d[i].x : x;
        y = c ? d[i].y : y;
        z = c ? d[i].z : z;
        w = c ? d[i].w : w;
    }
    return make_uint4(x, y, z, w);
}

// this lane's register chunk `it` (run-time value) as floats, boundary elements masked
template <int DT, int NIT, bool MASKED>
__device__ __forceinline__ void get_dyn(const RowSrc<DT, NIT, MASKED>& src, int it, float (&a)[Elem<DT>::kPerChunk])
{
    unpack<DT>(select_chunk<NIT>(src.d, it), a);
    src.mask((it * kWaves + wave_id()) * 64 + (int)(threadIdx.x & 63), a);
}

// the element of this lane's registers at virtual index v (the lane must own v)
template <int DT, int NIT, bool MASKED>
__device__ __forceinline__ float own_element(const RowSrc<DT, NIT, MASKED>& src, int v)
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int it = (v / (64 * E)) / kWaves;
    float a[E];
    get_dyn(src, it, a);
    float x = a[0];
#pragma unroll
    for (int e = 1; e < E; ++e)
        if ((v % E) == e) x = a[e];
    return x;
}

}  // namespace MDSD_NS
