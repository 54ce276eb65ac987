// Wavefront (64 lanes) and workgroup reductions for gfx950, built on DPP
// row shifts and row broadcasts so that no LDS traffic is needed inside a
// wave.  Every reduction has a fixed association order: results are
// bit-reproducible from launch to launch.
#pragma once
#include <hip/hip_runtime.h>

#include "build_config.h"
#include <limits.h>

namespace MDSD_NS {

constexpr int kWave = 64;
// A node is handled by kWG threads = kWaves wavefronts.  A workgroup holds kNodesPerWG such groups:
// more than one only where a group is a single wavefront, so that the groups of a workgroup share
// nothing and never have to meet at a barrier.
constexpr int kWG = MDSD_WG;
constexpr int kWaves = kWG / kWave;
constexpr int kNodesPerWG = MDSD_NODES_PER_WG;
static_assert(kNodesPerWG == 1 || kWaves == 1, "several nodes per workgroup: one wavefront each");

// index of this wavefront among those of its node, as a scalar: the compiler cannot see that
// threadIdx.x / 64 is the same in all 64 lanes, and would otherwise guard every per-wave
// decision with an execution mask instead of a scalar branch
__device__ __forceinline__ int wave_id()
{
    if constexpr (kWaves == 1) {
        // 0, in a form the compiler cannot see through: with a constant here it unrolls and
        // hoists the passes of the one-wavefront build until they need a fifth more registers and run
        // a fifth slower (RRS on rows of 50 tokens: 240 against 202 us)
        int zero = 0;
        asm volatile("" : "+s"(zero));
        return zero;
    } else {
        return __builtin_amdgcn_readfirstlane((int)(threadIdx.x / 64u));
    }
}
// which of the workgroup's nodes this thread works on, and its number among that node's threads
__device__ __forceinline__ int node_slot()
{
    if constexpr (kNodesPerWG == 1)
        return 0;
    else
        return __builtin_amdgcn_readfirstlane((int)(threadIdx.x / 64u));
}
__device__ __forceinline__ int node_thread()
{
    if constexpr (kNodesPerWG == 1)
        return (int)threadIdx.x;
    else
        return (int)(threadIdx.x & 63u);
}
// every thread of the node has arrived and sees the others' writes to LDS.  A single wavefront
// runs its LDS instructions in order, so there only the compiler has to be kept from moving them.
__device__ __forceinline__ void node_barrier()
{
    if constexpr (kWaves == 1) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    } else {
        __syncthreads();
    }
}

__device__ __forceinline__ float as_f(int v) { return __builtin_bit_cast(float, v); }
__device__ __forceinline__ int as_i(float v) { return __builtin_bit_cast(int, v); }

// v_mov_b32 with a DPP control; lanes without a source (or masked rows) read `old`.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp(float old, float v)
{
    return as_f(__builtin_amdgcn_update_dpp(as_i(old), as_i(v), CTRL, ROW_MASK, 0xf, false));
}

constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143, kWaveShr1 = 0x138;
// lane i reads lane 7 - i of its group of 8; lane i ^ 1; lane i ^ 2; lane i ^ 8
constexpr int kRowHalfMirror = 0x141, kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowRor8 = 0x128;

// Inclusive prefix sum over the 64 lanes; lane 63 ends with the wave total.
__device__ __forceinline__ float wave_scan_add(float v)
{
    v += dpp<kRowShr1>(0.f, v);
    v += dpp<kRowShr2>(0.f, v);
    v += dpp<kRowShr4>(0.f, v);
    v += dpp<kRowShr8>(0.f, v);
    v += dpp<kRowBcast15, 0xa>(0.f, v);
    v += dpp<kRowBcast31, 0xc>(0.f, v);
    return v;
}

__device__ __forceinline__ float lane_bcast(float v, int lane)
{
    return as_f(__builtin_amdgcn_readlane(as_i(v), lane));
}

__device__ __forceinline__ float wave_sum(float v) { return lane_bcast(wave_scan_add(v), 63); }

// Largest value of the wave (NaN counts above +inf: callers that may hold NaN check the
// result).  Taken on the order-preserving integer image of the floats: an integer maximum
// needs no quieting of its inputs, so each step is one instruction with the lane shift folded
// into it, instead of four.
__device__ __forceinline__ float wave_max(float v)
{
    int k = as_i(v);
    k ^= (k >> 31) & 0x7fffffff;
    k = max(k, __builtin_amdgcn_update_dpp(INT_MIN, k, kRowShr1, 0xf, 0xf, false));
    k = max(k, __builtin_amdgcn_update_dpp(INT_MIN, k, kRowShr2, 0xf, 0xf, false));
    k = max(k, __builtin_amdgcn_update_dpp(INT_MIN, k, kRowShr4, 0xf, 0xf, false));
    k = max(k, __builtin_amdgcn_update_dpp(INT_MIN, k, kRowShr8, 0xf, 0xf, false));
    k = max(k, __builtin_amdgcn_update_dpp(INT_MIN, k, kRowBcast15, 0xa, 0xf, false));
    k = max(k, __builtin_amdgcn_update_dpp(INT_MIN, k, kRowBcast31, 0xc, 0xf, false));
    k = __builtin_amdgcn_readlane(k, 63);
    k ^= (k >> 31) & 0x7fffffff;
    return as_f(k);
}

// Eight wave-wide sums for the price of about two: every lane passes eight values; on return
// lane l holds the sum over all 64 lanes of value number (l & 7).  Three halving steps inside
// each group of 8 lanes (every lane keeps the half of the values that its own bit selects and
// hands the other half to its partner), then the 8 groups are added up.  Fixed order of
// additions: the result is the same from launch to launch.
__device__ __forceinline__ float wave_sums8(const float (&v)[8])
{
    const int lane = threadIdx.x & 63;
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
    float k[4], m[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float keep = b2 ? v[4 + j] : v[j], send = b2 ? v[j] : v[4 + j];
        k[j] = keep + dpp<kRowHalfMirror>(0.f, send);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float keep = b0 ? k[2 * j + 1] : k[2 * j], send = b0 ? k[2 * j] : k[2 * j + 1];
        m[j] = keep + dpp<kQuadXor1>(0.f, send);
    }
    const float keep = b1 ? m[1] : m[0], send = b1 ? m[0] : m[1];
    float r = keep + dpp<kQuadXor2>(0.f, send);
    r += dpp<kRowRor8>(0.f, r);
    r += __shfl_xor(r, 16, 64);
    r += __shfl_xor(r, 32, 64);
    return r;
}

// value of the lane below (lane 0 reads `fill`)
__device__ __forceinline__ float wave_shift_up(float v, float fill)
{
    return dpp<kWaveShr1>(fill, v);
}

// Workgroup reductions through a small double-buffered LDS area: one barrier
// per call; two consecutive calls never touch the same buffer.
template <int WAVES>
struct BlockScratch {
    float buf[2][WAVES][4];
    int ibuf[2][WAVES];
};

template <int WAVES, int NV>
__device__ __forceinline__ void block_sum(float (&v)[NV], BlockScratch<WAVES>& s, int& phase)
{
    static_assert(NV <= 4, "at most four values per reduction");
    const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float t = wave_scan_add(v[i]);
        if (lane == 63) s.buf[phase][wave][i] = t;
    }
    node_barrier();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) t += s.buf[phase][w][i];
        v[i] = t;
    }
    phase ^= 1;
}

template <int WAVES, int NV>
__device__ __forceinline__ void block_max(float (&v)[NV], BlockScratch<WAVES>& s, int& phase)
{
    static_assert(NV <= 4, "at most four values per reduction");
    const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const float t = wave_max(v[i]);
        if (lane == 63) s.buf[phase][wave][i] = t;
    }
    node_barrier();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float t = s.buf[phase][0][i];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) t = fmaxf(t, s.buf[phase][w][i]);
        v[i] = t;
    }
    phase ^= 1;
}

// Smallest index over the workgroup (INT_MAX where a thread has none).
template <int WAVES>
__device__ __forceinline__ int block_min_index(int idx, BlockScratch<WAVES>& s, int& phase)
{
    const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) idx = min(idx, __shfl_xor(idx, off, 64));
    if (lane == 0) s.ibuf[phase][wave] = idx;
    node_barrier();
    int r = s.ibuf[phase][0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) r = min(r, s.ibuf[phase][w]);
    phase ^= 1;
    return r;
}

}  // namespace MDSD_NS
