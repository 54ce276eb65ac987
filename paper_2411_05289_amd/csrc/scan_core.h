// Building blocks shared by the draft and verify kernels: the slab loop over
// one or two rows, per-slab partial sums kept in LDS, and the two-level
// inverse-CDF search that uses them.
//
// Layout of the work inside a workgroup of kWaves wavefronts: slab s (64
// chunks of 16 bytes) belongs to wave s % kWaves.  A pass that needs an
// index-ordered prefix later (an inverse-CDF draw) leaves one partial sum per
// slab in LDS; the search then scans those sums, picks the slab, and only
// that slab is recomputed element by element.
#pragma once
#include <hip/hip_runtime.h>

#include "row_io.h"
#include "wave_ops.h"

namespace MDSD_NS {

constexpr int kMaxSlabs = MDSD_MAX_SLABS;
constexpr float kLog2e = 1.44269504088896340736f;

// stored element -> unnormalised probability.  Logits: 2^(l*s - ms) with
// s = log2(e)/T and ms = max*s; probabilities pass through.
template <bool LOGITS>
struct ToWeight {
    float s, ms;
    __device__ __forceinline__ float operator()(float l) const
    {
        if constexpr (LOGITS)
            return __builtin_amdgcn_exp2f(fmaf(l, s, -ms));
        else
            return l;
    }
    static __device__ __forceinline__ float fill()
    {
        return LOGITS ? -__builtin_inff() : 0.f;
    }
};

// fixed-shape sum of one lane's chunk; every slab sum is built from it, so a
// recomputed slab reproduces the stored sum bit for bit
template <int E>
__device__ __forceinline__ float chunk_sum(const float (&w)[E])
{
    if constexpr (E == 8)
        return ((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]));
    else
        return (w[0] + w[1]) + (w[2] + w[3]);
}

// A row as the passes see it.  NIT == 0: every pass streams the row from memory
// (any V).  NIT > 0: the row is loaded once, NIT chunks per lane, and stays in
// registers for all passes (V up to NIT * kWaves * 64 chunks); chunk `it` of a
// lane belongs to slab it * kWaves + wave, so each load instruction of a wave
// still covers 1 KiB of consecutive memory.  Masked elements hold `fill`.
// MASKED = false: the caller has checked that every row starts on a 16-byte boundary and
// that V is a whole number of chunks, so no element ever needs masking.
template <int DT, int NIT, bool MASKED = true>
struct RowSrc {
    static constexpr int E = Elem<DT>::kPerChunk;
    static constexpr int kNit = NIT;
    RowView r;
    float fill;
    uint4 d[NIT];

    // queue the loads of the whole row; nothing waits here
    __device__ __forceinline__ void issue(const RowView& rv, float f)
    {
        r = rv;
        fill = f;
        const int lane = threadIdx.x & 63, wave = wave_id();
        const uint32_t fb = __builtin_bit_cast(uint32_t, f);
        const uint32_t fw = DT == 0 ? fb : ((fb >> 16) | (fb & 0xffff0000u));
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int chunk = (it * kWaves + wave) * 64 + lane;
            d[it] = chunk < r.nchunk ? load16(r.chunks, chunk) : make_uint4(fw, fw, fw, fw);
        }
    }
    __device__ __forceinline__ void init(const RowView& rv, float f) { issue(rv, f); }

    // the first and the last chunk of the row may hold elements that are not the row's:
    // those read as `fill`.  The registers themselves are left alone.
    __device__ __forceinline__ void mask(int chunk, float (&a)[E]) const
    {
        if constexpr (!MASKED) return;
        const int v0 = chunk * E;
        if (v0 < r.head || v0 + E > r.nvirt) {
#pragma unroll
            for (int e = 0; e < E; ++e)
                if (v0 + e < r.head || v0 + e >= r.nvirt) a[e] = fill;
        }
    }

    // this lane's register chunk `it` as floats (it: compile-time constant after unrolling)
    __device__ __forceinline__ void get(int it, float (&a)[E]) const
    {
        unpack<DT>(d[it], a);
        mask((it * kWaves + wave_id()) * 64 + (int)(threadIdx.x & 63), a);
    }

    // body(slab, chunk, a[E])
    template <class Body>
    __device__ __forceinline__ void for_each(Body body) const
    {
        const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int s = it * kWaves + wave;
            if (s < r.nslab) {
                float a[E];
                get(it, a);
                body(s, s * 64 + lane, a);
            }
        }
    }

    // body(it, slab, chunk, a[E]): as for_each, with the number of the register chunk
    template <class Body>
    __device__ __forceinline__ void for_each_it(Body body) const
    {
        const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int s = it * kWaves + wave;
            if (s < r.nslab) {
                float a[E];
                get(it, a);
                body(it, s, s * 64 + lane, a);
            }
        }
    }

    // A softmax shift for a quarter of the work of an exact maximum.  bf16 rows that need no
    // masking only: the largest 32-bit word of this lane's chunks read as a float, which is the
    // odd-indexed element with its neighbour's bits as extra mantissa (less than one bf16 ulp
    // away from it).  The even-indexed elements may lie above it: whoever shifts by this
    // value checks that the sum of the weights stayed finite and positive, and takes the
    // exact maximum if not.
    static constexpr bool kHasShiftEstimate = DT == 1 && !MASKED;
    __device__ __forceinline__ float lane_shift_estimate() const
    {
        const int lane = threadIdx.x & 63, wave = wave_id();
        float m = -__builtin_inff();
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            if ((it * kWaves + wave) * 64 + lane < r.nchunk) {
                m = fmaxf(fmaxf(m, __builtin_bit_cast(float, d[it].x)), __builtin_bit_cast(float, d[it].y));
                m = fmaxf(fmaxf(m, __builtin_bit_cast(float, d[it].z)), __builtin_bit_cast(float, d[it].w));
            }
        }
        return m;
    }
};

template <int DT, bool MASKED>
struct RowSrc<DT, 0, MASKED> {
    static constexpr int E = Elem<DT>::kPerChunk;
    static constexpr int kNit = 0;
    RowView r;
    float fill;

    __device__ __forceinline__ void init(const RowView& rv, float f)
    {
        r = rv;
        fill = f;
    }
    __device__ __forceinline__ void issue(const RowView& rv, float f) { init(rv, f); }

    template <int AHEAD = 1, class Body>
    __device__ __forceinline__ void for_each(Body body) const
    {
        // each chunk is asked for AHEAD steps before its use (the steps past the end read the
        // row's last chunk again and drop it)
        static_assert(AHEAD == 1 || AHEAD == 2, "one or two steps ahead");
        const int lane = threadIdx.x & 63, wave = wave_id();
        uint4 c[AHEAD];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) c[i] = fetch_chunk(r, (wave + i * kWaves) * 64 + lane);
        for (int s = wave; s < r.nslab; s += kWaves) {
            const uint4 nxt = fetch_chunk(r, (s + AHEAD * kWaves) * 64 + lane);
            float a[E];
            finish_chunk<DT>(r, s * 64 + lane, c[0], fill, a);
            body(s, s * 64 + lane, a);
#pragma unroll
            for (int i = 0; i + 1 < AHEAD; ++i) c[i] = c[i + 1];
            c[AHEAD - 1] = nxt;
        }
    }
};

// body(slab, chunk, a[E], b[E]) over two rows with the same head and length.  Streamed rows are
// asked for AHEAD (1 or 2) steps before their use; the steps past the end read the rows' last
// chunks again and drop them.
template <int AHEAD = 1, int DT, int NIT, bool MASKED, class Body>
__device__ __forceinline__ void for_each2(const RowSrc<DT, NIT, MASKED>& sa, const RowSrc<DT, NIT, MASKED>& sb,
                                          Body body)
{
    static_assert(AHEAD == 1 || AHEAD == 2, "one or two steps ahead");
    constexpr int E = Elem<DT>::kPerChunk;
    const int lane = threadIdx.x & 63, wave = wave_id();
    if constexpr (NIT == 0) {
        uint4 ca[AHEAD], cb[AHEAD];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            ca[i] = fetch_chunk(sa.r, (wave + i * kWaves) * 64 + lane);
            cb[i] = fetch_chunk(sb.r, (wave + i * kWaves) * 64 + lane);
        }
        for (int s = wave; s < sa.r.nslab; s += kWaves) {
            const uint4 na = fetch_chunk(sa.r, (s + AHEAD * kWaves) * 64 + lane);
            const uint4 nb = fetch_chunk(sb.r, (s + AHEAD * kWaves) * 64 + lane);
            float a[E], b[E];
            finish_chunk<DT>(sa.r, s * 64 + lane, ca[0], sa.fill, a);
            finish_chunk<DT>(sb.r, s * 64 + lane, cb[0], sb.fill, b);
            body(s, s * 64 + lane, a, b);
#pragma unroll
            for (int i = 0; i + 1 < AHEAD; ++i) {
                ca[i] = ca[i + 1];
                cb[i] = cb[i + 1];
            }
            ca[AHEAD - 1] = na;
            cb[AHEAD - 1] = nb;
        }
    } else {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int s = it * kWaves + wave;
            if (s < sa.r.nslab) {
                float a[E], b[E];
                sa.get(it, a);
                sb.get(it, b);
                body(s, s * 64 + lane, a, b);
            }
            __builtin_amdgcn_sched_barrier(0);  // one chunk pair at a time
        }
    }
}

// half H (0 or 1) of a 16-byte chunk as floats; `chunk` is its number in row r, whose masked
// elements read as `fill`
template <int DT, bool MASKED, int H>
__device__ __forceinline__ void unpack_half(const uint4& d, const RowView& r, float fill, int chunk,
                                            float (&v)[Elem<DT>::kPerChunk / 2])
{
    constexpr int E = Elem<DT>::kPerChunk, HE = E / 2;
    const uint32_t w0 = H == 0 ? d.x : d.z, w1 = H == 0 ? d.y : d.w;
    if constexpr (DT == 0) {
        v[0] = __builtin_bit_cast(float, w0);
        v[1] = __builtin_bit_cast(float, w1);
    } else {
        v[0] = __builtin_bit_cast(float, w0 << 16);
        v[1] = __builtin_bit_cast(float, w0 & 0xffff0000u);
        v[2] = __builtin_bit_cast(float, w1 << 16);
        v[3] = __builtin_bit_cast(float, w1 & 0xffff0000u);
    }
    if constexpr (MASKED) {
        const int v0 = chunk * E + H * HE;
        if (v0 < r.head || v0 + HE > r.nvirt) {
#pragma unroll
            for (int e = 0; e < HE; ++e)
                if (v0 + e < r.head || v0 + e >= r.nvirt) v[e] = fill;
        }
    }
}

// body(it, slab, chunk, a, b) with the packed chunks of row a (register chunk it) and of row b, which is
// read from memory as the loop goes, QW chunks ahead of their use: b is read exactly once and
// never held whole.  Chunks of b past the end of the row read as `fill_b`.
template <int QW, int DT, int NIT, bool MASKED, class Body>
__device__ __forceinline__ void for_each_streamed_at(int lane, int wave, const RowSrc<DT, NIT, MASKED>& sa,
                                                     const RowView& rb, float fill_b, Body body);

template <int QW, int DT, int NIT, bool MASKED, class Body>
__device__ __forceinline__ void for_each_streamed(const RowSrc<DT, NIT, MASKED>& sa, const RowView& rb,
                                                  float fill_b, Body body)
{
    for_each_streamed_at<QW>((int)(threadIdx.x & 63), wave_id(), sa, rb, fill_b, body);
}

// the same with the lane and wave numbers handed in (a caller that runs the pass inside a loop
// hands in copies the compiler cannot see through, so that it does not hoist the address and
// mask arithmetic of every chunk out of that loop and hold it in registers)
template <int QW, int DT, int NIT, bool MASKED, class Body>
__device__ __forceinline__ void for_each_streamed_at(int lane, int wave, const RowSrc<DT, NIT, MASKED>& sa,
                                                     const RowView& rb, float fill_b, Body body)
{
    static_assert(NIT > 0 && QW > 0, "row a must be resident");
    const uint32_t fb = __builtin_bit_cast(uint32_t, fill_b);
    const uint32_t fw = DT == 0 ? fb : ((fb >> 16) | (fb & 0xffff0000u));
    // Every lane issues every load (a lane past the row reads the row's last chunk again and
    // drops it below): with a load inside a branch the compiler could not count the loads in
    // flight and would wait for all of them, the one just issued included, before each use.
    auto fetch = [&](int it) {
        const int chunk = (it * kWaves + wave) * 64 + lane;
        return load16(rb.chunks, chunk < rb.nchunk ? chunk : rb.nchunk - 1);
    };
    uint4 win[QW];
#pragma unroll
    for (int i = 0; i < QW && i < NIT; ++i) win[i] = fetch(i);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int s = it * kWaves + wave;
        uint4 cur = win[it % QW];
        if (it + QW < NIT) win[it % QW] = fetch(it + QW);
        if (s < sa.r.nslab) {
            if ((s + 1) * 64 > rb.nchunk) {  // the row's last slab, not full
                if (s * 64 + lane >= rb.nchunk) cur = make_uint4(fw, fw, fw, fw);
            }
            body(it, s, s * 64 + lane, sa.d[it], cur);
        }
        __builtin_amdgcn_sched_barrier(0);  // one chunk pair at a time
    }
}

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>)
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

// The same pass with the first QC chunks of row b kept in LDS between passes: a pass with
// CACHED = false reads all of b from memory and leaves those chunks in `cache` (one 16-byte
// entry per thread and chunk, read and written by that thread only: no barrier), a pass with
// CACHED = true takes them from there and reads only the rest of b from memory.
template <int QW, int QC, bool CACHED, int DT, int NIT, bool MASKED, class Body>
__device__ __forceinline__ void for_each_streamed_cached(int lane, int wave, const RowSrc<DT, NIT, MASKED>& sa,
                                                         const RowView& rb, float fill_b, uint4 (*cache)[kWG],
                                                         Body body)
{
    static_assert(NIT > 0 && QW == 1 && QC <= NIT, "row a must be resident, one chunk ahead");
    const uint32_t fb = __builtin_bit_cast(uint32_t, fill_b);
    const uint32_t fw = DT == 0 ? fb : ((fb >> 16) | (fb & 0xffff0000u));
    const int tid = wave * 64 + lane;
    auto fetch = [&](auto IT) {
        constexpr int it = decltype(IT)::value;
        if constexpr (CACHED && it < QC) {
            return cache[it][tid];
        } else {
            const int chunk = (it * kWaves + wave) * 64 + lane;
            return load16(rb.chunks, chunk < rb.nchunk ? chunk : rb.nchunk - 1);
        }
    };
    uint4 nxt = fetch(std::integral_constant<int, 0>{});
    static_for<NIT>([&](auto IT) {
        constexpr int it = decltype(IT)::value;
        const int s = it * kWaves + wave;
        uint4 cur = nxt;
        if constexpr (it + 1 < NIT) nxt = fetch(std::integral_constant<int, it + 1>{});
        if (s < sa.r.nslab) {
            if ((s + 1) * 64 > rb.nchunk) {  // the row's last slab, not full
                if (s * 64 + lane >= rb.nchunk) cur = make_uint4(fw, fw, fw, fw);
            }
            if constexpr (!CACHED && it < QC) cache[it][tid] = cur;
            body(it, s, s * 64 + lane, sa.d[it], cur);
        }
        __builtin_amdgcn_sched_barrier(0);  // one chunk pair at a time
    });
}

// store one slab's sum: every lane passes its chunk sum, lane 63 writes
__device__ __forceinline__ void store_slab_sum(float* slab_w, int s, float lane_sum)
{
    const float t = wave_scan_add(lane_sum);
    if ((threadIdx.x & 63) == 63) slab_w[s] = t;
}

// The slab sums of a row held in registers, reduced eight at a time: put() takes this lane's sum
// of its register chunk `it` (slab it * kWaves + wave), store() leaves every slab's sum in LDS.
template <int NIT>
struct SlabSums {
    static constexpr int kSlots = (NIT + 7) / 8 * 8;
    float v[kSlots];
    __device__ __forceinline__ SlabSums()
    {
#pragma unroll
        for (int i = 0; i < kSlots; ++i) v[i] = 0.f;
    }
    __device__ __forceinline__ void put(int it, float lane_sum) { v[it] = lane_sum; }
    __device__ __forceinline__ void store(float* slab_w, int nslab) const
    {
        const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
        for (int b = 0; b < kSlots / 8; ++b) {
            const float g[8] = {v[8 * b], v[8 * b + 1], v[8 * b + 2], v[8 * b + 3],
                                v[8 * b + 4], v[8 * b + 5], v[8 * b + 6], v[8 * b + 7]};
            const float t = wave_sums8(g);
            const int s = (8 * b + lane) * kWaves + wave;
            if (lane < 8 && s < nslab) slab_w[s] = t;
        }
    }
};

// Sum of the slab sums, in slab order.  Every wave computes it on its own
// (identical arithmetic, so identical bits) -- no broadcast needed.
template <class SlabVal>
__device__ __forceinline__ float slab_total(int nslab, SlabVal slab_val)
{
    const int lane = threadIdx.x & 63;
    float W = 0.f;
    for (int base = 0; base < nslab; base += 64) {
        const float v = (base + lane < nslab) ? slab_val(base + lane) : 0.f;
        W += wave_sum(v);
    }
    return W;
}

// Inverse CDF in two stages.  Stage 1 (every wave, redundantly): scan the slab
// sums for the first slab whose running sum exceeds t = u * W.  Returns false
// when there is nothing to draw (W == 0).  If rounding leaves no crossing the
// last slab with positive sum is taken and t becomes +inf, so that stage 2
// falls through to its last positive element.
struct SlabHit {
    int slab;    // slab that holds the drawn element
    float excl;  // running sum in front of that slab
    float t;     // threshold
};

template <class SlabVal>
__device__ __forceinline__ bool icdf_find_slab(int nslab, float u, float W, SlabVal slab_val, SlabHit& h)
{
    const int lane = threadIdx.x & 63;
    if (!(W > 0.f)) return false;
    h.t = u * W;
    h.excl = 0.f;
    h.slab = -1;
    float carry = 0.f;
    int last_pos = -1;
    for (int base = 0; base < nslab; base += 64) {
        const float v = (base + lane < nslab) ? slab_val(base + lane) : 0.f;
        const float incl = wave_scan_add(v);
        const float excl = carry + wave_shift_up(incl, 0.f);
        const unsigned long long hit = __ballot(carry + incl > h.t);
        const unsigned long long pos = __ballot(v > 0.f);
        if (hit) {
            const int l = __ffsll(hit) - 1;
            h.slab = base + l;
            h.excl = __shfl(excl, l, 64);
            return true;
        }
        if (pos) last_pos = base + 63 - __clzll(pos);
        carry += lane_bcast(incl, 63);
    }
    if (last_pos < 0) return false;
    h.slab = last_pos;
    h.t = __builtin_inff();
    return true;
}

// Stage 2 (one wave): w = this lane's chunk of the slab found in stage 1.
// Returns the virtual index of the first element whose running sum exceeds t,
// else the last element with positive weight, else -1 (same value in every lane).
template <int E>
__device__ __forceinline__ int icdf_in_slab(const float (&w)[E], const SlabHit& h)
{
    const int lane = threadIdx.x & 63;
    float t = h.t;
    const float ls = chunk_sum<E>(w);
    const float incl = wave_scan_add(ls);
    const float lane_excl = wave_shift_up(incl, 0.f);
    const unsigned long long hit = __ballot(h.excl + incl > t);
    const unsigned long long pos = __ballot(ls > 0.f);
    int l;
    if (hit) {
        l = __ffsll(hit) - 1;
    } else {
        if (!pos) return -1;
        l = 63 - __clzll(pos);
        t = __builtin_inff();
    }
    float run = h.excl + lane_excl;
    int e_sel = -1, e_last = -1;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (w[e] > 0.f) e_last = e;
        run += w[e];
        if (e_sel < 0 && run > t) e_sel = e;
    }
    if (e_sel < 0) e_sel = e_last;
    const int vidx = (e_sel < 0) ? -1 : (h.slab * 64 + lane) * E + e_sel;
    return __shfl(vidx, l, 64);
}

// Both stages with the chunk recomputed by weights(s, w); every wave runs it redundantly.
template <int E, class SlabVal, class Weights>
__device__ __forceinline__ int icdf_slabs(int nslab, float u, float W, SlabVal slab_val, Weights weights)
{
    SlabHit h;
    if (!icdf_find_slab(nslab, u, W, slab_val, h)) return -1;
    float w[E];
    weights(h.slab, w);
    return icdf_in_slab<E>(w, h);
}

}  // namespace MDSD_NS
