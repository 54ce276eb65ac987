// Row access for the vocabulary scans: a row of V stored elements (fp32 or
// bf16) is read as 16-byte chunks, one chunk per lane, 64 consecutive chunks
// ("a slab") per wavefront instruction, so every load instruction covers
// 1 KiB of consecutive HBM.  A row whose start is not 16-byte aligned is
// read from the aligned address below it; the `head` elements in front of the
// row and the elements behind its end are masked, never used.
#pragma once
#include <hip/hip_runtime.h>

#include "build_config.h"
#include <stdint.h>

namespace MDSD_NS {

template <int DT> struct Elem;
template <> struct Elem<0> {  // fp32
    static constexpr int kBytes = 4;
    static constexpr int kPerChunk = 4;
};
template <> struct Elem<1> {  // bf16
    static constexpr int kBytes = 2;
    static constexpr int kPerChunk = 8;
};

// Row pointers are rebuilt from integer addresses, which would leave the compiler with generic
// ("flat") pointers; flat loads also count against the LDS counter, so every wait on an LDS
// operation would wait for the rows as well.  Naming the global address space keeps the row
// loads on the vector-memory counter alone.
#define MDSD_GLOBAL __attribute__((address_space(1)))
typedef uint32_t v4u32 __attribute__((ext_vector_type(4)));
typedef const MDSD_GLOBAL v4u32* GlobalChunks;

// chunk i >= 0 of a row (rows are far smaller than 4 GiB): an unsigned 32-bit byte offset on
// the row's address lets the load take the row pointer from scalar registers and keep one
// vector register per address instead of two
__device__ __forceinline__ uint4 load16(GlobalChunks p, int i)
{
    const MDSD_GLOBAL char* b = reinterpret_cast<const MDSD_GLOBAL char*>(p);
    const v4u32 v = *reinterpret_cast<GlobalChunks>(b + (uint32_t)i * 16u);
    return make_uint4(v.x, v.y, v.z, v.w);
}

struct RowView {
    GlobalChunks chunks;  // 16-byte aligned
    int head;             // masked elements in front of token 0
    int nvirt;            // head + V
    int nchunk;           // chunks that hold at least one real element
    int nslab;            // slabs of 64 chunks
};

template <int DT>
__device__ __forceinline__ RowView make_row(const void* base, int64_t ld, int64_t row, int V)
{
    const uintptr_t addr = reinterpret_cast<uintptr_t>(base) +
                           static_cast<uintptr_t>(row * ld) * Elem<DT>::kBytes;
    const int mis = static_cast<int>(addr & 15);
    RowView r;
    r.chunks = reinterpret_cast<GlobalChunks>(addr - mis);
    r.head = mis / Elem<DT>::kBytes;
    r.nvirt = r.head + V;
    r.nchunk = (r.nvirt + Elem<DT>::kPerChunk - 1) / Elem<DT>::kPerChunk;
    r.nslab = (r.nchunk + 63) / 64;
    return r;
}

// One stored element by token index (scalar lookup).
template <int DT>
__device__ __forceinline__ float load_elem(const RowView& r, int x)
{
    const int v = r.head + x;
    if constexpr (DT == 0) {
        return reinterpret_cast<const MDSD_GLOBAL float*>(r.chunks)[v];
    } else {
        const uint32_t h = reinterpret_cast<const MDSD_GLOBAL uint16_t*>(r.chunks)[v];
        return __builtin_bit_cast(float, h << 16);
    }
}

template <int DT>
__device__ __forceinline__ void unpack(const uint4& d, float (&v)[Elem<DT>::kPerChunk])
{
    if constexpr (DT == 0) {
        v[0] = __builtin_bit_cast(float, d.x);
        v[1] = __builtin_bit_cast(float, d.y);
        v[2] = __builtin_bit_cast(float, d.z);
        v[3] = __builtin_bit_cast(float, d.w);
    } else {
        const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            v[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
        }
    }
}

// Chunk `chunk` of the row as floats; chunks past the end read as `fill`,
// masked elements of the first and last chunk are replaced by `fill`.  In two steps, so that
// a loop can ask for its next chunk before it works on the current one:
// fetch_chunk queues the load, finish_chunk turns what arrived into floats.
// The load itself is unconditional (a chunk past the end reads the row's last chunk and is
// masked whole afterwards): a load inside a branch is waited for inside it, so two rows read
// side by side would cost two trips to memory instead of one, and the compiler could not
// count the loads in flight.
__device__ __forceinline__ uint4 fetch_chunk(const RowView& r, int chunk)
{
    return load16(r.chunks, chunk < r.nchunk ? chunk : r.nchunk - 1);
}

template <int DT>
__device__ __forceinline__ void finish_chunk(const RowView& r, int chunk, const uint4& d, float fill,
                                             float (&v)[Elem<DT>::kPerChunk])
{
    constexpr int E = Elem<DT>::kPerChunk;
    unpack<DT>(d, v);
    const int v0 = chunk * E;
    if (v0 < r.head || v0 + E > r.nvirt) {
#pragma unroll
        for (int e = 0; e < E; ++e)
            if (v0 + e < r.head || v0 + e >= r.nvirt) v[e] = fill;
    }
}

template <int DT>
__device__ __forceinline__ void load_chunk(const RowView& r, int chunk, float fill,
                                           float (&v)[Elem<DT>::kPerChunk])
{
    finish_chunk<DT>(r, chunk, fetch_chunk(r, chunk), fill, v);
}

}  // namespace MDSD_NS
