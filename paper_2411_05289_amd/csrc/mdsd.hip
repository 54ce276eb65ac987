// HIP kernels and C ABI of the sampling-verification library (gfx950).
//
// One workgroup of 512 threads (8 wavefronts) owns one tree node -- or, in the path-only
// kernels, one tree, whose visited nodes it handles one after another.  A node's work is a few
// passes over its target row and, if it has children, its draft row, each pass a sequence of
// fully coalesced 16-byte loads or a sweep over registers that hold the row:
//   shift   a softmax shift for the stored logits: the row maximum, or a cheap estimate of it
//           (and the hub = argmax of the draft row, unless the draft call handed it on)
//   norm    softmax normalisers, sum of 2^((l - shift) * log2e / T)
//   test    scalar look-ups of p(x), q(x) at the draft tokens and the first acceptance test;
//           most nodes end here
//   resid   the vocabulary-wide residual sums of the method, one partial sum per slab in LDS
//   draw    inverse-CDF search over the slab sums, then inside one slab
// Kernel families, in the order of this file: helpers for the passes; the SpecHub kernel for
// logit rows in registers (spechub_*_resident); the RRS / RRSw kernel for the same (rrs_*_resident);
// the one-sweep statistics of streamed rows; the generic kernel for everything else
// (verify_node); the draft kernel; tree walk; Philox; host-side validation, dispatch and the
// C entry points.
#include <hip/hip_runtime.h>
#include <type_traits>
#include <limits.h>
#include <stdlib.h>
#include <stdint.h>

#include "mdsd.h"
#include "resident.h"
#include "scan_core.h"

namespace mdsd {

enum Method { kSpecHub = 0, kRRS = 1, kRRSw = 2 };

// SpecHub verify with draft statistics: chunks of the draft row requested ahead of their use in
// the residual pass (one is enough: a chunk pair is about 150 instructions of work for each of
// the 6 waves that share a SIMD), and the waves per SIMD the kernel is held to (6 = 80
// registers per lane = three workgroups per compute unit; 8 would spill).
constexpr int kStreamAhead = 1;
constexpr int kStatsWavesPerSimd = 6;

struct Params {
    const void* target;
    const void* draft;
    int64_t ld_t, ld_d;
    float temp_target, temp_draft;
    int B, N, V, k, depth, n_internal;
    const int32_t* first_child;
    const int32_t* tokens;
    const float* u;
    int32_t* outcome;
    int32_t* token;
    float* resid_mass;
    int32_t* flags;
    float* resid_prob;
    int32_t* accept_depth;  // path-only kernels
    int32_t* emitted;
    // draft kernels
    int32_t* tokens_out;
    int32_t* hub_out;
    // draft-row statistics: written by the SpecHub draft kernel, read by the SpecHub verify kernel
    mdsd_row_stats* stats_out;
    const mdsd_row_stats* stats_in;
};

struct Shared {
    BlockScratch<kWaves> red;
    float slab_w[kMaxSlabs];
    float bcast_f;  // one value handed from one lane to the workgroup
    int bcast_i;
    // RRS path for rows in registers: the node's draft tokens, the stored logits at them, the uniforms
    int node_x[MDSD_MAX_K];
    float node_lp[MDSD_MAX_K], node_lq[MDSD_MAX_K], node_u[MDSD_MAX_K + 1];
};

// Node of this workgroup.  Complete trees: nodes with children first (they
// scan two rows), leaves after, so the long workgroups start early.
struct NodeId {
    int b, n, c0;
    int64_t row;
};

__device__ __forceinline__ NodeId node_of_item(const Params& P, int w)
{
    NodeId id;
    if (P.first_child == nullptr) {
        const int total_int = P.B * P.n_internal;
        if (w < total_int) {
            id.b = w / P.n_internal;
            id.n = w - id.b * P.n_internal;
            id.c0 = P.k * id.n + 1;
        } else {
            w -= total_int;
            const int n_leaf = P.N - P.n_internal;
            id.b = w / n_leaf;
            id.n = P.n_internal + (w - id.b * n_leaf);
            id.c0 = -1;
        }
    } else {
        id.b = w / P.N;
        id.n = w - id.b * P.N;
        id.c0 = P.first_child[id.n];
        // an entry that leaves no room for k children is treated as a leaf
        if (id.c0 < 1 || id.c0 + P.k > P.N) id.c0 = -1;
    }
    id.row = (int64_t)id.b * P.N + id.n;
    return id;
}

__device__ __forceinline__ NodeId node_of_block(const Params& P) { return node_of_item(P, blockIdx.x); }

// ---------------------------------------------------------------- passes
// max of the stored values this lane holds
template <class Src>
__device__ __forceinline__ float lane_max(const Src& src)
{
    constexpr int E = Src::E;
    float m = -__builtin_inff();
    src.for_each([&](int, int, const float(&a)[E]) {
#pragma unroll
        for (int e = 0; e < E; ++e) m = fmaxf(m, a[e]);
    });
    return m;
}

// lowest virtual index at which this lane holds the value m (INT_MAX: nowhere)
template <class Src>
__device__ __forceinline__ int lane_first_index_of(const Src& src, float m)
{
    constexpr int E = Src::E;
    int idx = INT_MAX;
    src.for_each([&](int, int chunk, const float(&a)[E]) {
#pragma unroll
        for (int e = E - 1; e >= 0; --e)
            if (a[e] == m) idx = min(idx, chunk * E + e);
    });
    return idx;
}

// hub = lowest index among the maxima of the stored draft row (virtual index).
// Only lanes that hold the maximum look for its position.
template <class Src>
__device__ __forceinline__ int block_argmax(const Src& src, float m_lane, float m_block, Shared& sh,
                                            int& phase)
{
    int idx = INT_MAX;
    if (m_lane == m_block) idx = lane_first_index_of(src, m_block);
    const int a = block_min_index<kWaves>(idx, sh.red, phase);
    return a == INT_MAX ? src.r.head : a;  // a row of NaNs has no maximum: stay in bounds
}

// zero the entries of one chunk whose virtual index is listed in excl
template <int E>
__device__ __forceinline__ void zero_excluded(float (&w)[E], int chunk, const int* excl, int n_excl)
{
    for (int j = 0; j < n_excl; ++j) {
        const int off = excl[j] - chunk * E;
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = (e == off) ? 0.f : w[e];
    }
}

// slab holds one of the excluded elements?
template <int E>
__device__ __forceinline__ bool slab_has_excluded(int s, const int* excl, int n_excl)
{
    bool hit = false;
    for (int j = 0; j < n_excl; ++j) hit = hit || (excl[j] / (64 * E) == s);
    return hit;
}

// weights of one row, one slab sum per slab left in LDS; elements listed in
// excl count as 0
template <class CV, class Src>
__device__ __forceinline__ void pass_weights_to_slabs(const Src& src, CV cv, const int* excl, int n_excl,
                                                      float* slab_w)
{
    constexpr int E = Src::E;
    if constexpr (Src::kNit > 0) {
        SlabSums<Src::kNit> sums;
        src.for_each_it([&](int it, int s, int chunk, const float(&a)[E]) {
            float w[E];
#pragma unroll
            for (int e = 0; e < E; ++e) w[e] = cv(a[e]);
            if (slab_has_excluded<E>(s, excl, n_excl)) zero_excluded<E>(w, chunk, excl, n_excl);
            sums.put(it, chunk_sum<E>(w));
        });
        sums.store(slab_w, src.r.nslab);
    } else {
        src.for_each([&](int s, int chunk, const float(&a)[E]) {
            float w[E];
#pragma unroll
            for (int e = 0; e < E; ++e) w[e] = cv(a[e]);
            if (slab_has_excluded<E>(s, excl, n_excl)) zero_excluded<E>(w, chunk, excl, n_excl);
            store_slab_sum(slab_w, s, chunk_sum<E>(w));
        });
    }
}

// this lane's chunk of slab s of the same weights, read from memory (the draw
// inside one slab; the slab index is only known at run time)
template <int DT, class CV>
__device__ __forceinline__ void chunk_weights(const RowView& r, CV cv, const int* excl, int n_excl, int s,
                                              float (&w)[Elem<DT>::kPerChunk])
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int chunk = s * 64 + (threadIdx.x & 63);
    float a[E];
    load_chunk<DT>(r, chunk, CV::fill(), a);
#pragma unroll
    for (int e = 0; e < E; ++e) w[e] = cv(a[e]);
    zero_excluded<E>(w, chunk, excl, n_excl);
}

// Draw from the weights of one row (slab sums already in LDS and visible).
template <int DT, class CV>
__device__ __forceinline__ int draw_from_row(const RowView& r, CV cv, const int* excl, int n_excl,
                                             const float* slab_w, float u, float& W)
{
    constexpr int E = Elem<DT>::kPerChunk;
    auto sv = [&](int i) { return slab_w[i]; };
    W = slab_total(r.nslab, sv);
    return icdf_slabs<E>(r.nslab, u, W, sv,
                         [&](int s, float(&w)[E]) { chunk_weights<DT, CV>(r, cv, excl, n_excl, s, w); });
}

// ---------------------------------------------------------------- SpecHub element arithmetic
// App. B.2 for one token y != a, from unnormalised weights ep, eq:
//   P = ep/Zp, Q = eq/Zq, p' = max(P - Q, 0), Q'(y,a) = max(Q - P, 0),
//   t = c Q - p'  ->  Q'(a,y) = max(t, 0),  p''(y) = max(-t, 0).
struct HubScal {
    float iZp, iZq, c;
};

__device__ __forceinline__ float clamp01(float x) { return __builtin_amdgcn_fmed3f(x, 0.f, 1.f); }

// Every term is a probability (<= 1), so max(x, 0) is written as a clamp to [0, 1], which the
// hardware applies for free on the instruction that produces x.
__device__ __forceinline__ void spechub_terms(float ep, float eq, const HubScal& h, float& q_xa_res,
                                              float& q_ax_res, float& w)
{
    const float Pn = ep * h.iZp;
    const float Qn = eq * h.iZq;
    q_xa_res = clamp01(Qn - Pn);                // Q'(y,a) = max(Q - P, 0)
    const float pr = clamp01(Pn - Qn);          // p'(y)   = max(P - Q, 0)
    q_ax_res = clamp01(fmaf(h.c, Qn, -pr));     // Q'(a,y) = max(c Q - p', 0)
    w = clamp01(fmaf(-h.c, Qn, pr));            // p''(y)  = max(p' - c Q, 0)
}

template <int DT, class CV>
__device__ __forceinline__ void spechub_chunk_w(const RowView& rp, const RowView& rq, CV cp, CV cq,
                                                const HubScal& h, int a_virt, int s,
                                                float (&w)[Elem<DT>::kPerChunk])
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int chunk = s * 64 + (threadIdx.x & 63);
    float a[E], b[E];
    load_chunk<DT>(rp, chunk, CV::fill(), a);
    load_chunk<DT>(rq, chunk, CV::fill(), b);
#pragma unroll
    for (int e = 0; e < E; ++e) {
        float ep = cp(a[e]), eq = cq(b[e]);
        if (chunk * E + e == a_virt) ep = eq = 0.f;
        float s2, s1;
        spechub_terms(ep, eq, h, s2, s1, w[e]);
    }
}

// RRS residual weight for one token: max(p - c q, 0), c folded with 1/Zq
__device__ __forceinline__ float rrs_term(float ep, float eq, float iZp, float c_iZq)
{
    return fmaxf(fmaf(-c_iZq, eq, ep * iZp), 0.f);
}

template <int DT, class CV>
__device__ __forceinline__ void rrs_chunk_w(const RowView& rp, const RowView& rq, CV cp, CV cq, float iZp,
                                            float c_iZq, const int* excl, int n_excl, int s,
                                            float (&w)[Elem<DT>::kPerChunk])
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int chunk = s * 64 + (threadIdx.x & 63);
    float a[E], b[E];
    load_chunk<DT>(rp, chunk, CV::fill(), a);
    load_chunk<DT>(rq, chunk, CV::fill(), b);
#pragma unroll
    for (int e = 0; e < E; ++e) w[e] = rrs_term(cp(a[e]), cq(b[e]), iZp, c_iZq);
    zero_excluded<E>(w, chunk, excl, n_excl);
}

// write norm(w) of a whole row (diagnostic output)
template <int DT, class ChunkW>
__device__ __forceinline__ void write_resid_prob(float* out, const RowView& r, float W, ChunkW cw)
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int lane = threadIdx.x & 63, wave = wave_id();
    const float iW = W > 0.f ? 1.f / W : 0.f;
    for (int s = wave; s < r.nslab; s += kWaves) {
        float w[E];
        cw(s, w);
        const int v0 = (s * 64 + lane) * E;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int v = v0 + e;
            if (v >= r.head && v < r.nvirt) out[v - r.head] = w[e] * iW;
        }
    }
}

// ---------------------------------------------------------------- single-read paths (logits in registers)
struct NodeOut {
    int outcome, token, flags;
    float rmass;
};

using ExpW = ToWeight<true>;  // 2^(l*s - ms)

// Draw from weights held in registers: slab search by every wave, the search inside the slab by
// the wave that owns it; the result travels through LDS.  weights_of(it, w) gives this lane's
// weights of its register chunk `it` (run-time value).
template <int E, class SlabVal, class RegWeights>
__device__ __forceinline__ int draw_resident(int nslab, float u, float W, SlabVal sv, RegWeights weights_of,
                                             Shared& sh)
{
    SlabHit h;
    if (!icdf_find_slab(nslab, u, W, sv, h)) return -1;  // same decision in every wave
    if (wave_id() == h.slab % kWaves) {
        float w[E];
        weights_of(h.slab / kWaves, w);
        const int v = icdf_in_slab<E>(w, h);
        if ((threadIdx.x & 63) == 0) sh.bcast_i = v;
    }
    __syncthreads();
    return sh.bcast_i;
}

// leaf: bonus token ~ p (the k = 0 case of Alg. 1)
template <int DT, int NIT, bool MASKED>
__device__ __forceinline__ void leaf_resident(const Params& P, const RowView& rp,
                                              const RowSrc<DT, NIT, MASKED>& sp, float u, float* rprob,
                                              Shared& sh, int& phase, NodeOut& o)
{
    constexpr int E = Elem<DT>::kPerChunk;
    using Src = RowSrc<DT, NIT, MASKED>;
    ExpW cp;
    cp.s = kLog2e / P.temp_target;
    auto sv = [&](int i) { return sh.slab_w[i]; };
    float W;
    // the cheap estimate of the maximum as the shift where there is one; if the weights
    // overflowed or vanished with it, once more with the maximum itself
    auto slab_sums = [&](float lane_m) {
        float mm[1] = {lane_m};
        block_max<kWaves, 1>(mm, sh.red, phase);
        cp.ms = mm[0] * cp.s;
        pass_weights_to_slabs<ExpW>(sp, cp, nullptr, 0, sh.slab_w);
        __syncthreads();
        return slab_total(rp.nslab, sv);
    };
    if constexpr (Src::kHasShiftEstimate) {
        W = slab_sums(sp.lane_shift_estimate());
        if (__builtin_expect(!(W > 0.f && W < __builtin_inff()), 0)) {
            __syncthreads();  // every wave has read the slab sums that are about to be rewritten
            W = slab_sums(lane_max(sp));
        }
    } else {
        W = slab_sums(lane_max(sp));
    }
    const int v = draw_resident<E>(rp.nslab, u, W, sv, [&](int it, float(&w)[E]) {
        float a[E];
        get_dyn(sp, it, a);
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = cp(a[e]);
    }, sh);
    o.token = v < 0 ? -1 : v - rp.head;
    if (v < 0) o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
    o.rmass = 1.f;
    if (rprob)
        write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
            chunk_weights<DT, ExpW>(rp, cp, nullptr, 0, s, w);
        });
}

// the scalars of one node that come from memory: the pair, the stored logits at its tokens,
// the uniforms.  Asked for together with the rows, used after the first passes.
struct NodeIn {
    int x1, x2;
    bool tokens_ok;
    float lp1, lq1, lp2, lq2;
    float u0, u1, u2;
    // only with statistics handed on by the draft call
    int hub;          // token index, -1 = not usable
    float q_max, q_rest;
    float lpa;        // the target's stored logit at the hub
};

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform(float v) { return as_f(__builtin_amdgcn_readfirstlane(as_i(v))); }

// first the loads that depend on nothing but the node: uniforms, the pair, the record the
// draft call left
template <bool STATS>
__device__ __forceinline__ void fetch_node_scalars(const Params& P, const NodeId& id, NodeIn& in)
{
    const float* ur = P.u + id.row * 3;
    in.u0 = ur[0];
    in.u1 = ur[1];
    in.u2 = ur[2];
    in.x1 = in.x2 = -1;
    in.tokens_ok = false;
    in.lp1 = in.lq1 = in.lp2 = in.lq2 = 0.f;
    in.hub = -1;
    in.q_max = in.q_rest = in.lpa = 0.f;
    if (id.c0 >= 0) {
        const int32_t* xt = P.tokens + (int64_t)id.b * P.N + id.c0;
        in.x1 = xt[0];
        in.x2 = xt[1];
        in.tokens_ok = in.x1 >= 0 && in.x1 < P.V && in.x2 >= 0 && in.x2 < P.V;
        if constexpr (STATS) {
            const mdsd_row_stats st = P.stats_in[id.row];
            in.q_max = st.max_stored;
            in.q_rest = st.rest_mass;
            in.hub = (st.hub >= 0 && st.hub < P.V) ? st.hub : -1;
        }
    }
}

// then the stored logits at the tokens those loads named
template <int DT, bool STATS>
__device__ __forceinline__ void fetch_node_lookups(const NodeId& id, const RowView& rp, const RowView& rq,
                                                   NodeIn& in)
{
    if (id.c0 >= 0) {
        if (in.tokens_ok) {
            in.lp1 = load_elem<DT>(rp, in.x1);
            in.lq1 = load_elem<DT>(rq, in.x1);
            in.lp2 = load_elem<DT>(rp, in.x2);
            in.lq2 = load_elem<DT>(rq, in.x2);
        }
        if constexpr (STATS) {
            if (in.hub >= 0) in.lpa = load_elem<DT>(rp, in.hub);
        }
    }
}

template <int DT, bool STATS>
__device__ __forceinline__ void fetch_node_inputs(const Params& P, const NodeId& id, const RowView& rp,
                                                  const RowView& rq, NodeIn& in)
{
    fetch_node_scalars<STATS>(P, id, in);
    fetch_node_lookups<DT, STATS>(id, rp, rq, in);
}

// internal node, SpecHub (Alg. 3)
// STATS: the hub and the draft row's normalisers come with the node (the draft call left
// them); the draft row is then only needed for the residual sums, and is asked for only once
// the first test has failed.
template <int DT, int NIT, bool MASKED, bool STATS>
__device__ __forceinline__ void spechub_resident(const Params& P, const NodeIn& in, const RowView& rp,
                                                 const RowView& rq, const RowSrc<DT, NIT, MASKED>& sp,
                                                 RowSrc<DT, NIT, MASKED>& sq, bool need_full,
                                                 float* rprob, Shared& sh, int& phase, NodeOut& o)
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int x1 = in.x1, x2 = in.x2;
    const bool tokens_ok = in.tokens_ok;
    const float u0 = in.u0, u1 = in.u1, u2 = in.u2;

    float mm[2], z[2] = {0.f, 0.f};
    int a_virt;
    ExpW cp, cq;
    cp.s = kLog2e / P.temp_target;
    cq.s = kLog2e / P.temp_draft;
    float lp_hub;
    if constexpr (STATS) {
        if (in.hub < 0) {  // no usable record for this node
            o.flags |= MDSD_FLAG_BAD_PAIR;
            o.outcome = MDSD_BAD_PAIR;
            return;
        }
        // ---- target row alone: shift (the cheap estimate of the maximum first, the maximum
        // itself if the weights overflowed or vanished with it), then Zp
        using Src = RowSrc<DT, NIT, MASKED>;
        mm[1] = in.q_max;
        a_virt = rq.head + in.hub;
        cq.ms = mm[1] * cq.s;
        float z1[1];
        auto normaliser = [&](float lane_m) {
            float m1[1] = {lane_m};
            block_max<kWaves, 1>(m1, sh.red, phase);
            mm[0] = m1[0];
            cp.ms = mm[0] * cp.s;
            z1[0] = 0.f;
            sp.for_each([&](int, int, const float(&pa_)[E]) {
                float wp[E];
#pragma unroll
                for (int e = 0; e < E; ++e) wp[e] = cp(pa_[e]);
                z1[0] += chunk_sum<E>(wp);
            });
            block_sum<kWaves, 1>(z1, sh.red, phase);
        };
        if constexpr (Src::kHasShiftEstimate) {
            normaliser(sp.lane_shift_estimate());
            if (__builtin_expect(!(z1[0] > 0.f && z1[0] < __builtin_inff()), 0)) normaliser(lane_max(sp));
        } else {
            normaliser(lane_max(sp));
        }
        z[0] = z1[0];
        z[1] = in.q_rest;
        lp_hub = in.lpa;
    } else {
        // ---- maxima of the stored logits; hub = lowest index among the maxima of the draft row
        const float mq_lane = lane_max(sq);
        mm[0] = lane_max(sp);
        mm[1] = mq_lane;
        block_max<kWaves, 2>(mm, sh.red, phase);
        int my_idx = INT_MAX;
        if (mq_lane == mm[1]) my_idx = lane_first_index_of(sq, mm[1]);
        a_virt = block_min_index<kWaves>(my_idx, sh.red, phase);
        const bool owner = my_idx == a_virt && a_virt != INT_MAX;
        if (a_virt == INT_MAX) a_virt = rq.head;  // a row of NaNs has no maximum: stay in bounds
        a_virt = __builtin_amdgcn_readfirstlane(a_virt);
        if (owner) sh.bcast_f = own_element(sp, a_virt);  // the target's logit at the hub
        cp.ms = mm[0] * cp.s;
        cq.ms = mm[1] * cq.s;

        // ---- normalisers: Zp and the draft mass outside the hub, Zq' = sum_{y != a} eq (summed
        // without the hub, never formed as a difference)
        const int hub_slab = a_virt / (64 * E);
        for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
            float wp[E], wq[E];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                wp[e] = cp(pa_[e]);
                wq[e] = cq(qa_[e]);
            }
            if (__builtin_expect(s == hub_slab, 0)) {  // one slab of the row: a real (scalar) branch
                asm volatile("" ::: "memory");
                zero_excluded<E>(wq, chunk, &a_virt, 1);
            }
            z[0] += chunk_sum<E>(wp);
            z[1] += chunk_sum<E>(wq);
        });
        block_sum<kWaves, 2>(z, sh.red, phase);  // barrier: bcast_f visible
        lp_hub = sh.bcast_f;
    }
    const int a = a_virt - rq.head;
    const int a_slab = a_virt / (64 * E);
    const float Zq_rest = z[1];
    const float ea_q = cq(mm[1]);
    const float ea_p = cp(lp_hub);
    HubScal h;
    h.iZp = 1.f / z[0];
    h.iZq = 1.f / (Zq_rest + ea_q);
    h.c = ea_q / Zq_rest;  // q(a) / (1 - q(a)); unused when Zq_rest == 0
    const float pa = ea_p * h.iZp;
    const float qa = ea_q * h.iZq;

    bool decided = false, degenerate = false;
    int hub_slot = -1;
    if (!tokens_ok) {
        o.flags |= MDSD_FLAG_BAD_TOKEN;
        o.outcome = MDSD_BAD_TOKEN;
        decided = true;
    } else if (!(Zq_rest > 0.f)) {
        degenerate = true;
        o.flags |= MDSD_FLAG_DEGENERATE_HUB;
        if (x1 != a || x2 != a) {
            o.flags |= MDSD_FLAG_BAD_PAIR;
            o.outcome = MDSD_BAD_PAIR;
            decided = true;
        } else if (u0 * qa < pa) {
            o.outcome = 0;
            o.token = a;
            decided = true;
        }
    } else if (x2 == a && x1 != a) {
        hub_slot = 1;
        const float px = cp(in.lp1) * h.iZp, qx = cq(in.lq1) * h.iZq;
        if (u0 * qx < px) {  // pair (x, a): min(p(x)/Q(x,a), 1)
            o.outcome = 0;
            o.token = x1;
            decided = true;
        } else if (u1 * (Zq_rest * h.iZq) < pa - qa) {
            // the hub's test u1 * S_xa < p(a) - S_ax needs no sum when it holds for the bounds
            // S_xa <= sum_{y != a} q(y) and S_ax <= q(a)
            o.outcome = 1;
            o.token = a;
            decided = true;
        }
    } else if (x1 == a && x2 != a) {
        hub_slot = 0;
        const float px = cp(in.lp2) * h.iZp, qx = cq(in.lq2) * h.iZq;
        if (u0 * (h.c * qx) < fmaxf(px - qx, 0.f)) {  // pair (a, x): min(p'(x)/Q(a,x), 1)
            o.outcome = 1;
            o.token = x2;
            decided = true;
        } else if (u1 * qa < pa) {
            // the hub's test u1 * S_ax < p(a) needs no sum when it already holds for the
            // largest value S_ax can take: S_ax <= sum_{y != a} Q(a,y) = q(a)
            o.outcome = 0;
            o.token = a;
            decided = true;
        }
    } else {
        o.flags |= MDSD_FLAG_BAD_PAIR;
        o.outcome = MDSD_BAD_PAIR;
        decided = true;
    }
    if (decided && !need_full) return;

    if (degenerate) {
        // residual of the single-draft case: p with the hub removed
        pass_weights_to_slabs<ExpW>(sp, cp, &a_virt, 1, sh.slab_w);
        __syncthreads();
        float W;
        const int v = draw_from_row<DT, ExpW>(rp, cp, &a_virt, 1, sh.slab_w, u2, W);
        o.rmass = W * h.iZp;
        if (!decided) {
            o.token = v < 0 ? -1 : v - rp.head;
            if (v < 0) o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
        }
        if (rprob)
            write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
                chunk_weights<DT, ExpW>(rp, cp, &a_virt, 1, s, w);
            });
        return;
    }

    // ---- residual sums: S_xa = sum Q'(.,a), S_ax = sum Q'(a,.), slab sums of p''
    float sacc[2] = {0.f, 0.f};
    auto residual_terms = [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
        float ep[E], eq[E], t_xa[E], t_ax[E], w[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            ep[e] = cp(pa_[e]);
            eq[e] = cq(qa_[e]);
        }
        if (__builtin_expect(s == a_slab, 0)) {
            asm volatile("" ::: "memory");
            zero_excluded<E>(ep, chunk, &a_virt, 1);
            zero_excluded<E>(eq, chunk, &a_virt, 1);
        }
#pragma unroll
        for (int e = 0; e < E; ++e) spechub_terms(ep[e], eq[e], h, t_xa[e], t_ax[e], w[e]);
        sacc[0] += chunk_sum<E>(t_xa);
        sacc[1] += chunk_sum<E>(t_ax);
        store_slab_sum(sh.slab_w, s, chunk_sum<E>(w));
    };
    if constexpr (STATS) {
        // the draft row's only read.  Half a chunk at a time, so that few values are live at once.
        SlabSums<NIT> wsums;
        for_each_streamed<kStreamAhead>(sp, rq, ExpW::fill(), [&](int it, int s, int chunk, const uint4& dp, const uint4& dq) {
            constexpr int HE = E / 2;
            float part[3][2];
            auto half = [&](auto H) {
                constexpr int hv = decltype(H)::value;
                float ep[HE], eq[HE];
                unpack_half<DT, MASKED, hv>(dp, rp, ExpW::fill(), chunk, ep);
                unpack_half<DT, MASKED, hv>(dq, rq, ExpW::fill(), chunk, eq);
#pragma unroll
                for (int e = 0; e < HE; ++e) {
                    ep[e] = cp(ep[e]);
                    eq[e] = cq(eq[e]);
                }
                if (__builtin_expect(s == a_slab, 0)) {
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int e = 0; e < HE; ++e)
                        if (chunk * E + hv * HE + e == a_virt) ep[e] = eq[e] = 0.f;
                }
                float t_xa[HE], t_ax[HE], w[HE];
#pragma unroll
                for (int e = 0; e < HE; ++e) spechub_terms(ep[e], eq[e], h, t_xa[e], t_ax[e], w[e]);
                // the two halves of chunk_sum's tree
                if constexpr (HE == 4) {
                    part[0][hv] = (t_xa[0] + t_xa[1]) + (t_xa[2] + t_xa[3]);
                    part[1][hv] = (t_ax[0] + t_ax[1]) + (t_ax[2] + t_ax[3]);
                    part[2][hv] = (w[0] + w[1]) + (w[2] + w[3]);
                } else {
                    part[0][hv] = t_xa[0] + t_xa[1];
                    part[1][hv] = t_ax[0] + t_ax[1];
                    part[2][hv] = w[0] + w[1];
                }
            };
            half(std::integral_constant<int, 0>{});
            __builtin_amdgcn_sched_barrier(0);
            half(std::integral_constant<int, 1>{});
            sacc[0] += part[0][0] + part[0][1];
            sacc[1] += part[1][0] + part[1][1];
            wsums.put(it, part[2][0] + part[2][1]);
        });
        wsums.store(sh.slab_w, rp.nslab);
    } else {
        for_each2(sp, sq, residual_terms);
    }
    block_sum<kWaves, 2>(sacc, sh.red, phase);  // barrier: slab sums visible
    const float S_xa = sacc[0], S_ax = sacc[1];
    if (!decided) {
        if (hub_slot == 1) {  // pair (x, a): the hub draws on what the pairs (a,.) left of p(a)
            if (u1 * S_xa < fmaxf(pa - S_ax, 0.f)) {
                o.outcome = 1;
                o.token = a;
                decided = true;
            }
        } else if (u1 * S_ax < pa) {  // pair (a, x)
            o.outcome = 0;
            o.token = a;
            decided = true;
        }
    }
    auto sv = [&](int i) { return sh.slab_w[i]; };
    const float W = slab_total(rp.nslab, sv);
    o.rmass = W;
    bool wrote_prob = false;
    if (!decided) {
        int v;
        if constexpr (STATS)
            // the drawn slab's share of the draft row comes from memory a second time (1 KiB)
            v = icdf_slabs<E>(rp.nslab, u2, W, sv, [&](int s, float(&w)[E]) {
                spechub_chunk_w<DT, ExpW>(rp, rq, cp, cq, h, a_virt, s, w);
            });
        else
            v = draw_resident<E>(rp.nslab, u2, W, sv, [&](int it, float(&w)[E]) {
            float a_[E], b_[E];
            get_dyn(sp, it, a_);
            get_dyn(sq, it, b_);
            const int chunk = (it * kWaves + wave) * 64 + lane;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                float ep = cp(a_[e]), eq = cq(b_[e]);
                if (chunk * E + e == a_virt) ep = eq = 0.f;
                float t0, t1;
                spechub_terms(ep, eq, h, t0, t1, w[e]);
            }
        }, sh);
        if (v < 0) {
            // no residual mass: fall back to p itself
            o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
            __syncthreads();
            pass_weights_to_slabs<ExpW>(sp, cp, nullptr, 0, sh.slab_w);
            __syncthreads();
            float Wp;
            v = draw_from_row<DT, ExpW>(rp, cp, nullptr, 0, sh.slab_w, u2, Wp);
            if (rprob) {
                write_resid_prob<DT>(rprob, rp, Wp, [&](int s, float(&w)[E]) {
                    chunk_weights<DT, ExpW>(rp, cp, nullptr, 0, s, w);
                });
                wrote_prob = true;
            }
        }
        o.token = v < 0 ? -1 : v - rp.head;
    }
    if (rprob && !wrote_prob)
        write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
            spechub_chunk_w<DT, ExpW>(rp, rq, cp, cq, h, a_virt, s, w);
        });
}

// One node of SpecHub verify for logit rows that fit in registers: every load of the node queued
// before anything waits, all passes over the target row from registers.  Writes the node's
// outputs and returns its outcome and token (the same values in every lane).
template <int DT, int NIT, bool MASKED, bool STATS>
__device__ __forceinline__ NodeOut spechub_node_resident(const Params& P, const NodeId& id, Shared& sh, int& phase)
{
    const bool need_full = (P.resid_mass != nullptr) || (P.resid_prob != nullptr);
    float* rprob = P.resid_prob ? P.resid_prob + id.row * (int64_t)P.V : nullptr;
    const RowView rp = make_row<DT>(P.target, P.ld_t, id.row, P.V);
    RowView rq = rp;
    RowSrc<DT, NIT, MASKED> sp, sq;
    sp.issue(rp, ExpW::fill());
    if (id.c0 >= 0) {
        rq = make_row<DT>(P.draft, P.ld_d, id.row, P.V);
        if constexpr (!STATS) sq.issue(rq, ExpW::fill());
    }
    NodeIn in;
    fetch_node_inputs<DT, STATS>(P, id, rp, rq, in);
    NodeOut o{MDSD_NONE, -1, 0, 0.f};
    if (id.c0 < 0)
        leaf_resident<DT, NIT, MASKED>(P, rp, sp, in.u2, rprob, sh, phase, o);
    else
        spechub_resident<DT, NIT, MASKED, STATS>(P, in, rp, rq, sp, sq, need_full, rprob, sh, phase, o);
    if (threadIdx.x == 0) {
        P.outcome[id.row] = o.outcome;
        P.token[id.row] = o.token;
        if (P.resid_mass) P.resid_mass[id.row] = o.rmass;
        if (P.flags) P.flags[id.row] = o.flags;
    }
    return o;
}

// one workgroup per node
template <int DT, int NIT, bool MASKED, bool STATS>
__global__ __launch_bounds__(kWG, (NIT <= 8 ? (STATS ? kStatsWavesPerSimd : 4) : 2)) void spechub_verify_resident(const Params P)
{
    __shared__ Shared sh;
    int phase = 0;
    spechub_node_resident<DT, NIT, MASKED, STATS>(P, node_of_block(P), sh, phase);
}

// Path-only verification (Sec. 2: only the nodes the walk visits decide what a step emits): one
// workgroup per tree starts at the root, verifies a node, and moves to the accepted child until
// a node accepts nothing, a leaf has given its bonus token, or `depth` tokens are out.  Nodes
// off the path keep outcome MDSD_UNVISITED.  verify_node(id) handles one node and returns its
// outcome and token, uniform over the workgroup.
template <class VerifyNode>
__device__ __forceinline__ void walk_and_verify(const Params& P, VerifyNode verify_node)
{
    const int b = blockIdx.x;
    for (int i = threadIdx.x; i < P.N; i += kWG) {
        const int64_t r = (int64_t)b * P.N + i;
        P.outcome[r] = MDSD_UNVISITED;
        P.token[r] = -1;
        if (P.flags) P.flags[r] = 0;
        if (P.resid_mass) P.resid_mass[r] = 0.f;
    }
    int32_t* em = P.emitted + (int64_t)b * P.depth;
    for (int i = threadIdx.x; i < P.depth; i += kWG) em[i] = -1;
    // the visited nodes' entries are rewritten below by another thread of this workgroup
    __threadfence_block();
    __syncthreads();
    int n = 0, d = 0;
    for (;;) {
        NodeId id;
        id.b = b;
        id.n = n;
        if (P.first_child) {
            id.c0 = P.first_child[n];
            if (id.c0 < 1 || id.c0 + P.k > P.N) id.c0 = -1;
        } else {
            const int64_t c = (int64_t)P.k * n + 1;
            id.c0 = (c + P.k <= P.N) ? (int)c : -1;
        }
        id.row = (int64_t)b * P.N + n;
        const NodeOut o = verify_node(id);
        const int outcome = uniform(o.outcome), token = uniform(o.token);
        if (threadIdx.x == 0 && d < P.depth) em[d] = token;
        if (id.c0 < 0 || outcome < 0 || outcome >= P.k || d + 1 >= P.depth) break;
        n = id.c0 + outcome;
        ++d;
        __syncthreads();  // the next node reuses the LDS areas of this one
    }
    if (threadIdx.x == 0) P.accept_depth[b] = d;
}

template <int DT, int NIT, bool MASKED, bool STATS>
__global__ __launch_bounds__(kWG, (NIT <= 8 ? 4 : 2)) void spechub_path_resident(const Params P)
{
    __shared__ Shared sh;
    int phase = 0;
    walk_and_verify(P, [&](const NodeId& id) {
        return spechub_node_resident<DT, NIT, MASKED, STATS>(P, id, sh, phase);
    });
}

// ---------------------------------------------------------------- RRS / RRSw, rows in registers
// Alg. 1 for one internal node when the draft call left its record of the draft row (largest
// stored element, total mass): the target row sits in registers, the draft row is streamed once
// per rejected round, and a node whose first draft is accepted never reads it.  The state after
// i rejections is the residual U = max(p - c q, 0) with mass W (c_1 = 0, W_0 = 1,
// c_{i+1} = c_i + W_i rho_{i+1}): round i + 1 accepts x with probability U(x) / (W q_{i+1}(x)).
// WO (without replacement): q_{i+1} is q without the tokens rejected so far, rescaled by
// rho_{i+1} = (mass of q) / (mass left); the mass outside all k drafted tokens is summed (positive
// terms only) in the first pass over the draft row, the masses left are that plus the later drafts'.
template <int DT, int NIT, bool MASKED, bool WO>
__device__ __forceinline__ void rrs_resident(const Params& P, const NodeId& id, const RowView& rp,
                                             const RowView& rq, const RowSrc<DT, NIT, MASKED>& sp,
                                             bool need_full, float* rprob, Shared& sh, int& phase, NodeOut& o)
{
    constexpr int E = Elem<DT>::kPerChunk;
    constexpr int HE = E / 2;
    using Src = RowSrc<DT, NIT, MASKED>;
    const int k = P.k;
    const float* ur = P.u + id.row * (k + 1);
    const int32_t* xt = P.tokens + (int64_t)id.b * P.N + id.c0;
    const mdsd_row_stats st = P.stats_in[id.row];
    // tokens, the stored logits at them and the uniforms go through LDS (lane i of the first wave
    // fetches draft i), so that no lane holds arrays of them; visible after the first barrier
    if ((int)threadIdx.x < k) {
        const int i = threadIdx.x;
        const int x = xt[i];
        const bool ok = x >= 0 && x < P.V;
        sh.node_x[i] = ok ? x : -1;
        sh.node_lp[i] = ok ? load_elem<DT>(rp, x) : 0.f;
        sh.node_lq[i] = ok ? load_elem<DT>(rq, x) : 0.f;
        sh.node_u[i] = ur[i];
    }
    if (threadIdx.x == 0) sh.node_u[k] = ur[k];

    // ---- target row: shift (cheap estimate first, where there is one) and Zp
    ExpW cp, cq;
    cp.s = kLog2e / P.temp_target;
    cq.s = kLog2e / P.temp_draft;
    cq.ms = uniform(st.max_stored * cq.s);
    float z1[1];
    auto normaliser = [&](float lane_m) {
        float m1[1] = {lane_m};
        block_max<kWaves, 1>(m1, sh.red, phase);
        cp.ms = uniform(m1[0] * cp.s);
        z1[0] = 0.f;
        sp.for_each([&](int, int, const float(&pa_)[E]) {
            float wp[E];
#pragma unroll
            for (int e = 0; e < E; ++e) wp[e] = cp(pa_[e]);
            z1[0] += chunk_sum<E>(wp);
        });
        block_sum<kWaves, 1>(z1, sh.red, phase);
    };
    if constexpr (Src::kHasShiftEstimate) {
        normaliser(sp.lane_shift_estimate());
        if (__builtin_expect(!(z1[0] > 0.f && z1[0] < __builtin_inff()), 0)) normaliser(lane_max(sp));
    } else {
        normaliser(lane_max(sp));
    }
    const float iZp = uniform(1.f / z1[0]);
    const float iZq = uniform(1.f / st.rest_mass);
    bool bad = false;
    for (int i = 0; i < k; ++i) bad = bad || sh.node_x[i] < 0;
    if (bad) {
        o.flags |= MDSD_FLAG_BAD_TOKEN;
        o.outcome = MDSD_BAD_TOKEN;
        return;
    }
    const float u_last = sh.node_u[k];

    float c = 0.f, Wc = 1.f;
    bool decided = false, slabs_current = false;
    int n_rej = 0;
    float rem_k = 0.f;  // WO: unnormalised draft mass outside all k drafted tokens (after the first pass)
    // one pass over both rows: slab sums (and total) of max(p - c_new q, 0), rejected tokens masked;
    // with want_rem also the draft mass outside the drafted tokens
    auto residual_pass = [&](float c_new, bool want_rem) {
        const float c_iZq = c_new * iZq;
        // slabs of the first two tokens to mask (with more than two, every slab takes the slow check)
        const int n_mask = want_rem ? k : n_rej;
        const int s_lo = (sh.node_x[0] + rp.head) / (64 * E);
        const int s_hi = n_mask > 1 ? (sh.node_x[1] + rp.head) / (64 * E) : s_lo;
        float lane_rem = 0.f;
        SlabSums<NIT> sums;
        // Opaque copies: the weights of the target row do not change from round to round, and
        // the compiler would otherwise compute all of them once, ahead of the rounds, and hold
        // one register per element.
        int lane_o = threadIdx.x & 63, wave_o = wave_id();
        ExpW cpo = cp;
        asm volatile("" : "+v"(lane_o), "+s"(wave_o), "+s"(cpo.ms));
        for_each_streamed_at<kStreamAhead>(lane_o, wave_o, sp, rq, ExpW::fill(), [&](int it, int s, int chunk, const uint4& dp, const uint4& dq) {
            float part[2];
            auto half = [&](auto H) {
                constexpr int hv = decltype(H)::value;
                float ep[HE], eq[HE], w[HE];
                unpack_half<DT, MASKED, hv>(dp, rp, ExpW::fill(), chunk, ep);
                unpack_half<DT, MASKED, hv>(dq, rq, ExpW::fill(), chunk, eq);
#pragma unroll
                for (int e = 0; e < HE; ++e) {
                    eq[e] = cq(eq[e]);
                    w[e] = rrs_term(cpo(ep[e]), eq[e], iZp, c_iZq);
                }
                if (__builtin_expect(s == s_lo || s == s_hi || n_mask > 2, 0)) {
                    asm volatile("" ::: "memory");
                    for (int j = 0; j < n_mask; ++j) {
                        const int xvj = sh.node_x[j] + rp.head;
#pragma unroll
                        for (int e = 0; e < HE; ++e) {
                            if (chunk * E + hv * HE + e == xvj) {
                                if (j < n_rej) w[e] = 0.f;
                                eq[e] = 0.f;  // only summed with want_rem, where every drafted token is left out
                            }
                        }
                    }
                }
                if constexpr (HE == 4)
                    part[hv] = (w[0] + w[1]) + (w[2] + w[3]);
                else
                    part[hv] = w[0] + w[1];
                if constexpr (WO) {
                    if (want_rem) {
                        if constexpr (HE == 4)
                            lane_rem += (eq[0] + eq[1]) + (eq[2] + eq[3]);
                        else
                            lane_rem += eq[0] + eq[1];
                    }
                }
            };
            half(std::integral_constant<int, 0>{});
            __builtin_amdgcn_sched_barrier(0);
            half(std::integral_constant<int, 1>{});
            sums.put(it, part[0] + part[1]);
        });
        sums.store(sh.slab_w, rp.nslab);
        if constexpr (WO) {
            if (want_rem) {
                float rr[1] = {lane_rem};
                block_sum<kWaves, 1>(rr, sh.red, phase);
                rem_k = rr[0];
            }
        }
        __syncthreads();
        return slab_total(rp.nslab, [&](int j) { return sh.slab_w[j]; });
    };
    // WO: unnormalised draft mass left before round i (i >= 1): what no draft took, plus the
    // drafts still to come (a repeated token counts once)
    auto mass_left = [&](int i) {
        float m = rem_k;
        for (int j = k - 1; j >= i; --j) {
            bool dup = false;
            for (int l = 0; l < j; ++l) dup = dup || (sh.node_x[l] == sh.node_x[j]);
            if (!dup) m += cq(sh.node_lq[j]);
        }
        return m;
    };

    for (int i = 0; i < k; ++i) {
        const int xi = uniform(sh.node_x[i]);
        const float px = cp(sh.node_lp[i]) * iZp, qx = cq(sh.node_lq[i]) * iZq, ui = sh.node_u[i];
        bool seen = false;
        for (int j = 0; j < i; ++j) seen = seen || (sh.node_x[j] == xi);
        const float Ux = seen ? 0.f : fmaxf(fmaf(-c, qx, px), 0.f);
        // draft probability of x_i in this round and the factor that rescales q; without
        // replacement a repeated token has no mass left
        float Qi = qx, rho = 1.f;
        if (WO && i > 0) {
            const float left = mass_left(i);
            Qi = seen ? 0.f : cq(sh.node_lq[i]) / left;
            rho = 1.f / (left * iZq);
        }
        if (ui * Qi * Wc < Ux) {  // Alg. 1 returns at the first acceptance
            o.outcome = i;
            o.token = xi;
            decided = true;
            break;
        }
        const float c_new = fmaf(Wc, rho, c);
        n_rej = i + 1;
        if (i > 0) __syncthreads();  // earlier readers of the slab sums are done
        const float W_new = residual_pass(c_new, WO && i == 0);
        if (W_new > 0.f) {
            c = c_new;
            Wc = W_new;
            slabs_current = true;
        } else {
            o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
            slabs_current = false;
        }
        if constexpr (WO) {
            if (!(mass_left(i + 1) > 0.f)) {
                o.flags |= MDSD_FLAG_Q_EXHAUSTED;
                break;
            }
        }
    }
    if (decided && !need_full) return;
    if (!slabs_current) {
        __syncthreads();
        residual_pass(c, false);
    }
    const float c_iZq = c * iZq;
    auto cw = [&](int s, float(&w)[E]) {
        rrs_chunk_w<DT, ExpW>(rp, rq, cp, cq, iZp, c_iZq, nullptr, 0, s, w);
        const int chunk = s * 64 + (threadIdx.x & 63);
        for (int j = 0; j < n_rej; ++j) {
            const int off = sh.node_x[j] + rp.head - chunk * E;
#pragma unroll
            for (int e = 0; e < E; ++e) w[e] = (e == off) ? 0.f : w[e];
        }
    };
    auto sv = [&](int j) { return sh.slab_w[j]; };
    const float W = slab_total(rp.nslab, sv);
    o.rmass = W;
    if (!decided) {
        const int v = icdf_slabs<E>(rp.nslab, u_last, W, sv, cw);
        o.token = v < 0 ? -1 : v - rp.head;
        if (v < 0) o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
    }
    if (rprob) write_resid_prob<DT>(rprob, rp, W, cw);
}

template <int DT, int NIT, bool MASKED, bool WO>
__device__ __forceinline__ NodeOut rrs_node_resident(const Params& P, const NodeId& id, Shared& sh, int& phase)
{
    const bool need_full = (P.resid_mass != nullptr) || (P.resid_prob != nullptr);
    float* rprob = P.resid_prob ? P.resid_prob + id.row * (int64_t)P.V : nullptr;
    const RowView rp = make_row<DT>(P.target, P.ld_t, id.row, P.V);
    RowSrc<DT, NIT, MASKED> sp;
    sp.issue(rp, ExpW::fill());
    NodeOut o{MDSD_NONE, -1, 0, 0.f};
    if (id.c0 < 0) {
        leaf_resident<DT, NIT, MASKED>(P, rp, sp, P.u[id.row * (P.k + 1) + P.k], rprob, sh, phase, o);
    } else {
        const RowView rq = make_row<DT>(P.draft, P.ld_d, id.row, P.V);
        rrs_resident<DT, NIT, MASKED, WO>(P, id, rp, rq, sp, need_full, rprob, sh, phase, o);
    }
    if (threadIdx.x == 0) {
        P.outcome[id.row] = o.outcome;
        P.token[id.row] = o.token;
        if (P.resid_mass) P.resid_mass[id.row] = o.rmass;
        if (P.flags) P.flags[id.row] = o.flags;
    }
    return o;
}

template <int DT, int NIT, bool MASKED, bool WO>
__global__ __launch_bounds__(kWG, (NIT <= 8 ? kStatsWavesPerSimd : 2)) void rrs_verify_resident(const Params P)
{
    __shared__ Shared sh;
    int phase = 0;
    rrs_node_resident<DT, NIT, MASKED, WO>(P, node_of_block(P), sh, phase);
}

// One sweep over a logit row that is streamed from memory (too long for registers), instead of
// a pass for the maximum and a pass for the weights.  Each wave forms its weights against a
// reference of its own, the largest element of its first slab; when the row's maximum M is
// known the partial sums are brought to the row's units by one factor per wave,
// 2^((reference - M) s) <= 1.  Returns false (caller falls back to two passes) when the sum
// came out zero or not finite: some later element lay too far above a wave's reference.
// On success: M = maximum of the stored row, Z = sum of 2^((l - M) s); with SLABS the slab
// sums in LDS are in the same units and visible to every wave.
template <int DT, bool SLABS, class Src>
__device__ __forceinline__ bool sweep_streamed_row(const Src& src, float s, Shared& sh, int& phase, float& M,
                                                   float& Z, float* lane_max_out = nullptr)
{
    constexpr int E = Elem<DT>::kPerChunk;
    const int lane = threadIdx.x & 63, wave = wave_id();
    const float ninf = -__builtin_inff();
    float a0[E];
    load_chunk<DT>(src.r, wave * 64 + lane, ninf, a0);  // slabs past the row read as -inf
    float r = a0[0];
#pragma unroll
    for (int e = 1; e < E; ++e) r = fmaxf(r, a0[e]);
    r = wave_max(r);
    if (!(r > ninf) || !(r < __builtin_inff())) r = 0.f;  // nothing finite to refer to
    ToWeight<true> cw;
    cw.s = s;
    cw.ms = uniform(r * s);
    float lane_m = ninf, lane_z = 0.f;
    src.for_each([&](int sl, int, const float(&a)[E]) {
        float w[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            lane_m = fmaxf(lane_m, a[e]);
            w[e] = cw(a[e]);
        }
        const float cs = chunk_sum<E>(w);
        lane_z += cs;
        if constexpr (SLABS) store_slab_sum(sh.slab_w, sl, cs);
    });
    if (lane_max_out) *lane_max_out = lane_m;
    float mm[1] = {lane_m};
    block_max<kWaves, 1>(mm, sh.red, phase);
    M = mm[0];
    const float scale = uniform(__builtin_amdgcn_exp2f(fmaf(r, s, -(M * s))));
    float zz[1] = {lane_z * scale};
    block_sum<kWaves, 1>(zz, sh.red, phase);  // barrier: every slab sum is stored
    Z = zz[0];
    const bool ok = Z > 0.f && Z < __builtin_inff();
    if constexpr (SLABS) {
        if (ok) {
            for (int i = wave + kWaves * lane; i < src.r.nslab; i += kWaves * 64) sh.slab_w[i] *= scale;
        }
        __syncthreads();
    }
    return ok;
}

// ---------------------------------------------------------------- verify kernel
// Two workgroups per CU need 4 waves per SIMD, i.e. at most 128 VGPRs; the 16-chunk variant
// holds 128 VGPRs of row data alone and runs one workgroup per CU.
template <int DT, bool LOGITS, int METHOD, int NIT>
__device__ __forceinline__ NodeOut verify_node(const Params& P, const NodeId& id, Shared& sh, int& phase)
{
    constexpr int E = Elem<DT>::kPerChunk;
    using CV = ToWeight<LOGITS>;
    using Src = RowSrc<DT, NIT>;
    const int k = P.k;
    const float* ur = P.u + id.row * (k + 1);
    const bool need_full = (P.resid_mass != nullptr) || (P.resid_prob != nullptr);
    float* rprob = P.resid_prob ? P.resid_prob + id.row * (int64_t)P.V : nullptr;

    const RowView rp = make_row<DT>(P.target, P.ld_t, id.row, P.V);
    Src sp;
    int outcome = MDSD_NONE, token = -1, flags = 0;
    float rmass = 0.f;

    sp.init(rp, CV::fill());

    if (id.c0 < 0) {
        // ---- leaf: the k = 0 case of Alg. 1, token ~ p
        CV cp{0.f, 0.f};
        bool swept = false;
        if constexpr (LOGITS && NIT == 0) {
            float M, Z;
            cp.s = kLog2e / P.temp_target;
            swept = sweep_streamed_row<DT, true>(sp, cp.s, sh, phase, M, Z);
            cp.ms = M * cp.s;
        }
        if (!swept) {
            if constexpr (LOGITS) {
                float mm[1] = {lane_max(sp)};
                block_max<kWaves, 1>(mm, sh.red, phase);
                cp.s = kLog2e / P.temp_target;
                cp.ms = mm[0] * cp.s;
            }
            pass_weights_to_slabs<CV>(sp, cp, nullptr, 0, sh.slab_w);
            __syncthreads();
        }
        float W;
        const int v = draw_from_row<DT, CV>(rp, cp, nullptr, 0, sh.slab_w, ur[k], W);
        token = v < 0 ? -1 : v - rp.head;
        if (v < 0) flags |= MDSD_FLAG_ZERO_RESIDUAL;
        rmass = LOGITS ? 1.f : W;
        if (rprob)
            write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
                chunk_weights<DT, CV>(rp, cp, nullptr, 0, s, w);
            });
    } else {
        const RowView rq = make_row<DT>(P.draft, P.ld_d, id.row, P.V);
        Src sq;
        // the draft row is asked for when a pass first needs it: with the draft call's record of
        // the row at hand, a node that accepts in its first test never reads it
        bool q_asked = false;
        auto need_q = [&]() {
            if (!q_asked) sq.init(rq, CV::fill());
            q_asked = true;
        };
        const int32_t* xt = P.tokens + (int64_t)id.b * P.N + id.c0;
        CV cp{0.f, 0.f}, cq{0.f, 0.f};

        if constexpr (METHOD == kSpecHub) {
            // ---- hub (argmax of the stored draft row), softmax maxima, normalisers: Zp (logits
            // only) and the draft mass outside the hub, Zq' = sum_{y != a} eq.  With the draft
            // call's record of the row at hand, the draft row is not read for any of them.
            const bool have_stats = P.stats_in != nullptr;
            mdsd_row_stats st{0.f, 0.f, 0, 0};
            if (have_stats) {
                st = P.stats_in[id.row];
                if (st.hub < 0 || st.hub >= P.V) st.hub = -1;
            }
            float mm[2], z[2] = {0.f, 0.f};
            int a_virt;
            bool swept = false;
            if (have_stats) {
                mm[0] = 0.f;
                if constexpr (LOGITS && NIT == 0) {
                    // maximum and Zp of the streamed target row in one sweep
                    swept = sweep_streamed_row<DT, false>(sp, kLog2e / P.temp_target, sh, phase, mm[0], z[0]);
                }
                if (!swept) {
                    float m1[1] = {LOGITS ? lane_max(sp) : 0.f};
                    if constexpr (LOGITS) block_max<kWaves, 1>(m1, sh.red, phase);
                    mm[0] = m1[0];
                }
                mm[1] = st.max_stored;
                a_virt = rq.head + (st.hub < 0 ? 0 : st.hub);
            } else {
                need_q();
                const float mq_lane = lane_max(sq);
                mm[0] = LOGITS ? lane_max(sp) : 0.f;
                mm[1] = mq_lane;
                block_max<kWaves, 2>(mm, sh.red, phase);
                a_virt = block_argmax(sq, mq_lane, mm[1], sh, phase);
            }
            const int a = a_virt - rq.head;
            if constexpr (LOGITS) {
                cp.s = kLog2e / P.temp_target;
                cp.ms = mm[0] * cp.s;
                cq.s = kLog2e / P.temp_draft;
                cq.ms = mm[1] * cq.s;
            }
            const int a_slab = a_virt / (64 * E);
            if (have_stats) {
                if (LOGITS && !swept) {
                    float z1[1] = {0.f};
                    sp.for_each([&](int, int, const float(&pa_)[E]) {
                        float wp[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) wp[e] = cp(pa_[e]);
                        z1[0] += chunk_sum<E>(wp);
                    });
                    block_sum<kWaves, 1>(z1, sh.red, phase);
                    z[0] = z1[0];
                }
                z[1] = st.rest_mass;
            } else {
                for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
                    float wp[E], wq[E];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        wp[e] = cp(pa_[e]);
                        wq[e] = cq(qa_[e]);
                    }
                    if (s == a_slab) zero_excluded<E>(wq, chunk, &a_virt, 1);
                    z[0] += chunk_sum<E>(wp);
                    z[1] += chunk_sum<E>(wq);
                });
                block_sum<kWaves, 2>(z, sh.red, phase);
            }
            const float ea_q = cq(load_elem<DT>(rq, a));
            const float ea_p = cp(load_elem<DT>(rp, a));
            const float Zq_rest = z[1];
            HubScal h;
            h.iZp = LOGITS ? 1.f / z[0] : 1.f;
            h.iZq = LOGITS ? 1.f / (Zq_rest + ea_q) : 1.f;
            h.c = ea_q / Zq_rest;  // q(a) / (1 - q(a)); unused when Zq_rest == 0
            const float pa = ea_p * h.iZp;
            const float qa = ea_q * h.iZq;

            const int x1 = xt[0], x2 = xt[1];
            bool decided = false, degenerate = false;
            int hub_slot = -1;  // slot of the hub token in the pair
            if (have_stats && st.hub < 0) {  // no usable record for this node
                flags |= MDSD_FLAG_BAD_PAIR;
                outcome = MDSD_BAD_PAIR;
                decided = true;
            } else if (x1 < 0 || x1 >= P.V || x2 < 0 || x2 >= P.V) {
                flags |= MDSD_FLAG_BAD_TOKEN;
                outcome = MDSD_BAD_TOKEN;
                decided = true;
            } else if (!(Zq_rest > 0.f)) {
                degenerate = true;
                flags |= MDSD_FLAG_DEGENERATE_HUB;
                if (x1 != a || x2 != a) {
                    flags |= MDSD_FLAG_BAD_PAIR;
                    outcome = MDSD_BAD_PAIR;
                    decided = true;
                } else if (ur[0] * qa < pa) {
                    outcome = 0;
                    token = a;
                    decided = true;
                }
            } else if (x2 == a && x1 != a) {
                hub_slot = 1;
                const float px = cp(load_elem<DT>(rp, x1)) * h.iZp;
                const float qx = cq(load_elem<DT>(rq, x1)) * h.iZq;
                if (ur[0] * qx < px) {  // pair (x, a): min(p(x)/Q(x,a), 1)
                    outcome = 0;
                    token = x1;
                    decided = true;
                }
            } else if (x1 == a && x2 != a) {
                hub_slot = 0;
                const float px = cp(load_elem<DT>(rp, x2)) * h.iZp;
                const float qx = cq(load_elem<DT>(rq, x2)) * h.iZq;
                if (ur[0] * (h.c * qx) < fmaxf(px - qx, 0.f)) {  // pair (a, x): min(p'(x)/Q(a,x), 1)
                    outcome = 1;
                    token = x2;
                    decided = true;
                } else if (ur[1] * qa < pa) {
                    // S_ax <= sum_{y != a} Q(a,y) = q(a): the hub's test holds whatever the sum is
                    outcome = 0;
                    token = a;
                    decided = true;
                }
            } else {
                flags |= MDSD_FLAG_BAD_PAIR;
                outcome = MDSD_BAD_PAIR;
                decided = true;
            }

            if (!decided || need_full) {
                if (degenerate) {
                    // residual of the single-draft case: p with the hub removed
                    pass_weights_to_slabs<CV>(sp, cp, &a_virt, 1, sh.slab_w);
                    __syncthreads();
                    float W;
                    const int v = draw_from_row<DT, CV>(rp, cp, &a_virt, 1, sh.slab_w, ur[2], W);
                    rmass = W * h.iZp;
                    if (!decided) {
                        token = v < 0 ? -1 : v - rp.head;
                        if (v < 0) flags |= MDSD_FLAG_ZERO_RESIDUAL;
                    }
                    if (rprob)
                        write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
                            chunk_weights<DT, CV>(rp, cp, &a_virt, 1, s, w);
                        });
                } else {
                    // ---- residual sums: S_xa = sum Q'(.,a), S_ax = sum Q'(a,.), slab sums of p''
                    float sacc[2] = {0.f, 0.f};
                    need_q();
                    for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
                        float ep[E], eq[E], t_xa[E], t_ax[E], w[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            ep[e] = cp(pa_[e]);
                            eq[e] = cq(qa_[e]);
                        }
                        if (s == a_slab) {
                            zero_excluded<E>(ep, chunk, &a_virt, 1);
                            zero_excluded<E>(eq, chunk, &a_virt, 1);
                        }
#pragma unroll
                        for (int e = 0; e < E; ++e) spechub_terms(ep[e], eq[e], h, t_xa[e], t_ax[e], w[e]);
                        sacc[0] += chunk_sum<E>(t_xa);
                        sacc[1] += chunk_sum<E>(t_ax);
                        store_slab_sum(sh.slab_w, s, chunk_sum<E>(w));
                    });
                    block_sum<kWaves, 2>(sacc, sh.red, phase);  // barrier: slab sums visible
                    const float S_xa = sacc[0], S_ax = sacc[1];
                    if (!decided) {
                        if (hub_slot == 1) {  // pair (x, a): hub draws on what pairs (a,.) left
                            const float pa1 = fmaxf(pa - S_ax, 0.f);
                            if (ur[1] * S_xa < pa1) {
                                outcome = 1;
                                token = a;
                                decided = true;
                            }
                        } else {  // pair (a, x)
                            if (ur[1] * S_ax < pa) {
                                outcome = 0;
                                token = a;
                                decided = true;
                            }
                        }
                    }
                    auto sv = [&](int i) { return sh.slab_w[i]; };
                    auto cw = [&](int s, float(&w)[E]) {
                        spechub_chunk_w<DT, CV>(rp, rq, cp, cq, h, a_virt, s, w);
                    };
                    const float W = slab_total(rp.nslab, sv);
                    rmass = W;
                    bool wrote_prob = false;
                    if (!decided) {
                        int v = icdf_slabs<E>(rp.nslab, ur[2], W, sv, cw);
                        if (v < 0) {
                            // no residual mass: fall back to p itself
                            flags |= MDSD_FLAG_ZERO_RESIDUAL;
                            __syncthreads();
                            pass_weights_to_slabs<CV>(sp, cp, nullptr, 0, sh.slab_w);
                            __syncthreads();
                            float Wp;
                            v = draw_from_row<DT, CV>(rp, cp, nullptr, 0, sh.slab_w, ur[2], Wp);
                            if (rprob) {
                                write_resid_prob<DT>(rprob, rp, Wp, [&](int s, float(&w)[E]) {
                                    chunk_weights<DT, CV>(rp, cp, nullptr, 0, s, w);
                                });
                                wrote_prob = true;
                            }
                        }
                        token = v < 0 ? -1 : v - rp.head;
                    }
                    if (rprob && !wrote_prob) write_resid_prob<DT>(rprob, rp, W, cw);
                }
            }
        } else {
            // ---- RRS / RRSw (Alg. 1).  State: residual U = max(p - c q, 0) with mass Wc.
            constexpr bool WO = (METHOD == kRRSw);
            int xs[MDSD_MAX_K];
            bool bad = false;
            for (int i = 0; i < k; ++i) {
                xs[i] = xt[i];
                if (xs[i] < 0 || xs[i] >= P.V) bad = true;
            }
            if (bad) {
                flags |= MDSD_FLAG_BAD_TOKEN;
                outcome = MDSD_BAD_TOKEN;
            } else {
                // The draft call's record (largest stored element, total mass) stands in for the
                // statistics of the draft row.  Without replacement the mass outside the drafted
                // tokens is needed too, from the second round on: the first rejected round's pass
                // over the draft row sums it.
                const bool have_stats = P.stats_in != nullptr;
                mdsd_row_stats st{0.f, 0.f, -1, 0};
                if (have_stats) st = P.stats_in[id.row];
                float z[2] = {0.f, 0.f};
                bool swept = false;
                if constexpr (LOGITS) {
                    float mm[2];
                    if (have_stats) {
                        mm[0] = 0.f;
                        if constexpr (NIT == 0)
                            swept = sweep_streamed_row<DT, false>(sp, kLog2e / P.temp_target, sh, phase, mm[0], z[0]);
                        if (!swept) {
                            float m1[1] = {lane_max(sp)};
                            block_max<kWaves, 1>(m1, sh.red, phase);
                            mm[0] = m1[0];
                        }
                        mm[1] = st.max_stored;
                    } else {
                        need_q();
                        mm[0] = lane_max(sp);
                        mm[1] = lane_max(sq);
                        block_max<kWaves, 2>(mm, sh.red, phase);
                    }
                    cp.s = kLog2e / P.temp_target;
                    cp.ms = mm[0] * cp.s;
                    cq.s = kLog2e / P.temp_draft;
                    cq.ms = mm[1] * cq.s;
                }
                // exclusion list (virtual indices) and duplicate marks
                int xv[MDSD_MAX_K];
                bool dup[MDSD_MAX_K];
                for (int i = 0; i < k; ++i) {
                    xv[i] = xs[i] + rp.head;
                    dup[i] = false;
                    for (int j = 0; j < i; ++j) dup[i] = dup[i] || (xs[j] == xs[i]);
                }
                // normalisers; without replacement the draft sum leaves out every draft token,
                // so that the mass remaining after i removals is a sum of positive terms
                if (have_stats) {
                    if (LOGITS && !swept) {
                        float z1[1] = {0.f};
                        sp.for_each([&](int, int, const float(&pa_)[E]) {
                            float wp[E];
#pragma unroll
                            for (int e = 0; e < E; ++e) wp[e] = cp(pa_[e]);
                            z1[0] += chunk_sum<E>(wp);
                        });
                        block_sum<kWaves, 1>(z1, sh.red, phase);
                        z[0] = z1[0];
                    }
                    z[1] = st.rest_mass;
                } else {
                    need_q();
                    for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
                        float wp[E], wq[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            wp[e] = cp(pa_[e]);
                            wq[e] = cq(qa_[e]);
                        }
                        if constexpr (WO) {
                            if (slab_has_excluded<E>(s, xv, k)) zero_excluded<E>(wq, chunk, xv, k);
                        }
                        z[0] += chunk_sum<E>(wp);
                        z[1] += chunk_sum<E>(wq);
                    });
                    block_sum<kWaves, 2>(z, sh.red, phase);
                }
                float eqx[MDSD_MAX_K];
                for (int i = 0; i < k; ++i) eqx[i] = cq(load_elem<DT>(rq, xs[i]));
                // draft mass (unnormalised) left before round i: what no draft took (a sum of
                // positive terms; with a record, known after the first rejected round) plus the
                // drafts still to come, a repeated token counting once
                const bool rem_pending = WO && have_stats;
                float rem_k = rem_pending ? 0.f : z[1];
                auto mass_left = [&](int i) {
                    float m = rem_k;
                    for (int j = k - 1; j >= i; --j) m += (WO && !dup[j]) ? eqx[j] : 0.f;
                    return m;
                };
                const float Zq = have_stats ? z[1] : mass_left(0);
                const float iZp = LOGITS ? 1.f / z[0] : 1.f;
                const float iZq = LOGITS ? 1.f / Zq : 1.f;

                float c = 0.f, Wc = 1.f;
                float slab_c = -1.f;  // c of the slab sums in LDS (-1: none)
                int slab_nx = -1;
                bool decided = false;
                int n_rej = 0;  // tokens xs[0..n_rej) have been rejected
                for (int i = 0; i < k; ++i) {
                    const float px = cp(load_elem<DT>(rp, xs[i])) * iZp;
                    const float qx = eqx[i] * iZq;
                    // draft probability of x_i in this round and the factor rho that rescales q;
                    // without replacement a repeated token has no mass left (Alg. 1, red lines)
                    float Qi = qx, rho = 1.f;
                    if (WO && i > 0) {
                        const float left = mass_left(i);
                        Qi = dup[i] ? 0.f : eqx[i] / left;
                        rho = 1.f / (left * iZq);
                    }
                    bool seen = false;
                    for (int j = 0; j < i; ++j) seen = seen || (xs[j] == xs[i]);
                    const float Ux = seen ? 0.f : fmaxf(fmaf(-c, qx, px), 0.f);
                    if (ur[i] * Qi * Wc < Ux) {  // Alg. 1 returns at the first acceptance
                        outcome = i;
                        token = xs[i];
                        decided = true;
                        break;
                    }
                    // reject: U <- max(p - (c + Wc rho) q, 0)
                    const float c_new = fmaf(Wc, rho, c);
                    n_rej = i + 1;
                    if (i > 0) __syncthreads();  // earlier readers of slab_w are done
                    const float c_iZq = c_new * iZq;
                    const bool want_rem = rem_pending && i == 0;
                    float lane_rem[1] = {0.f};
                    need_q();
                    for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
                        float w[E], wq[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            wq[e] = cq(qa_[e]);
                            w[e] = rrs_term(cp(pa_[e]), wq[e], iZp, c_iZq);
                        }
                        if (slab_has_excluded<E>(s, xv, n_rej)) zero_excluded<E>(w, chunk, xv, n_rej);
                        store_slab_sum(sh.slab_w, s, chunk_sum<E>(w));
                        if (want_rem) {
                            if (slab_has_excluded<E>(s, xv, k)) zero_excluded<E>(wq, chunk, xv, k);
                            lane_rem[0] += chunk_sum<E>(wq);
                        }
                    });
                    if (want_rem) {
                        block_sum<kWaves, 1>(lane_rem, sh.red, phase);
                        rem_k = lane_rem[0];
                    }
                    __syncthreads();
                    const float W_new = slab_total(rp.nslab, [&](int j) { return sh.slab_w[j]; });
                    if (W_new > 0.f) {
                        c = c_new;
                        Wc = W_new;
                        slab_c = c_new;
                        slab_nx = n_rej;
                    } else {
                        flags |= MDSD_FLAG_ZERO_RESIDUAL;
                        slab_c = -1.f;
                    }
                    if constexpr (WO) {
                        if (!(mass_left(i + 1) > 0.f)) {
                            flags |= MDSD_FLAG_Q_EXHAUSTED;
                            break;
                        }
                    }
                }
                if (!decided || need_full) {
                    const float c_iZq = c * iZq;
                    auto cw = [&](int s, float(&w)[E]) {
                        rrs_chunk_w<DT, CV>(rp, rq, cp, cq, iZp, c_iZq, xv, n_rej, s, w);
                    };
                    if (slab_c != c || slab_nx != n_rej) {
                        // the slab sums in LDS are not those of the current residual (accepted in
                        // the first round, or a round without mass): rebuild them
                        __syncthreads();
                        need_q();
                        for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
                            float w[E];
#pragma unroll
                            for (int e = 0; e < E; ++e) w[e] = rrs_term(cp(pa_[e]), cq(qa_[e]), iZp, c_iZq);
                            if (slab_has_excluded<E>(s, xv, n_rej)) zero_excluded<E>(w, chunk, xv, n_rej);
                            store_slab_sum(sh.slab_w, s, chunk_sum<E>(w));
                        });
                        __syncthreads();
                    }
                    auto sv = [&](int j) { return sh.slab_w[j]; };
                    const float W = slab_total(rp.nslab, sv);
                    rmass = W;
                    if (!decided) {
                        const int v = icdf_slabs<E>(rp.nslab, ur[k], W, sv, cw);
                        token = v < 0 ? -1 : v - rp.head;
                        if (v < 0) flags |= MDSD_FLAG_ZERO_RESIDUAL;
                    }
                    if (rprob) write_resid_prob<DT>(rprob, rp, W, cw);
                }
            }
        }
    }

    if (threadIdx.x == 0) {
        P.outcome[id.row] = outcome;
        P.token[id.row] = token;
        if (P.resid_mass) P.resid_mass[id.row] = rmass;
        if (P.flags) P.flags[id.row] = flags;
    }
    return NodeOut{outcome, token, flags, rmass};
}

template <int DT, bool LOGITS, int METHOD, int NIT>
__global__ __launch_bounds__(kWG) void verify_kernel(const Params P)
{
    __shared__ Shared sh;
    int phase = 0;
    verify_node<DT, LOGITS, METHOD, NIT>(P, node_of_block(P), sh, phase);
}

template <int DT, bool LOGITS, int METHOD, int NIT>
__global__ __launch_bounds__(kWG) void verify_path_kernel(const Params P)
{
    __shared__ Shared sh;
    int phase = 0;
    walk_and_verify(P, [&](const NodeId& id) { return verify_node<DT, LOGITS, METHOD, NIT>(P, id, sh, phase); });
}

// ---------------------------------------------------------------- draft kernel
template <int DT, bool LOGITS, int METHOD, int NIT, bool MASKED = true>
__global__ __launch_bounds__(kWG) void draft_kernel(const Params P)
{
    constexpr int E = Elem<DT>::kPerChunk;
    using CV = ToWeight<LOGITS>;
    __shared__ Shared sh;
    int phase = 0;
    // one workgroup per node; a leaf only records that it has no hub
    const NodeId id = node_of_block(P);
    const int b = id.b, n = id.n, c0 = id.c0;
    const int64_t row = id.row;
    if (n == 0 && threadIdx.x == 0) P.tokens_out[(int64_t)b * P.N] = -1;
    if (c0 < 0) {
        if (threadIdx.x == 0) {
            if (P.hub_out) P.hub_out[row] = -1;
            if (P.flags) P.flags[row] = 0;
            if (P.stats_out) P.stats_out[row] = mdsd_row_stats{0.f, 0.f, -1, 0};
        }
        return;
    }
    const int k = P.k;
    const float* ur = P.u + row * k;
    const RowView rq = make_row<DT>(P.draft, P.ld_d, row, P.V);
    RowSrc<DT, NIT, MASKED> sq;
    sq.init(rq, CV::fill());
    int32_t* xt = P.tokens_out + (int64_t)b * P.N + c0;
    int flags = 0;

    CV cq{0.f, 0.f};
    int a_virt = rq.head;
    float mm[1] = {0.f};
    bool swept = false;
    if constexpr (LOGITS && NIT == 0) {
        // a streamed logit row: maximum, weights and slab sums in one sweep
        float Z, mq_lane;
        cq.s = kLog2e / P.temp_draft;
        swept = sweep_streamed_row<DT, true>(sq, cq.s, sh, phase, mm[0], Z, &mq_lane);
        if (swept) {
            cq.ms = mm[0] * cq.s;
            if constexpr (METHOD == kSpecHub) a_virt = block_argmax(sq, mq_lane, mm[0], sh, phase);
        }
    }
    if (!swept) {
        if (LOGITS || METHOD == kSpecHub) {
            const float mq_lane = lane_max(sq);
            mm[0] = mq_lane;
            block_max<kWaves, 1>(mm, sh.red, phase);
            if constexpr (METHOD == kSpecHub) a_virt = block_argmax(sq, mq_lane, mm[0], sh, phase);
            if constexpr (LOGITS) {
                cq.s = kLog2e / P.temp_draft;
                cq.ms = mm[0] * cq.s;
            }
        }
        pass_weights_to_slabs<CV>(sq, cq, nullptr, 0, sh.slab_w);
    }
    __syncthreads();

    // slab sums with some tokens removed: only the slabs holding a removed token change,
    // and those are recomputed with the tokens masked (never by subtraction)
    int excl[MDSD_MAX_K];
    int ov_slab[MDSD_MAX_K];
    float ov_val[MDSD_MAX_K];
    int n_excl = 0, n_ov = 0;
    auto sv = [&](int i) {
        float v = sh.slab_w[i];
        for (int j = 0; j < n_ov; ++j)
            if (ov_slab[j] == i) v = ov_val[j];
        return v;
    };
    // this lane's weights of one chunk of slab s, removed tokens counting 0: from memory when the
    // row is streamed, from the registers of the wave that owns the slab when it is resident
    auto cw = [&](int s, float(&w)[E]) { chunk_weights<DT, CV>(rq, cq, excl, n_excl, s, w); };
    auto cw_reg = [&](int it, float(&w)[E]) {
        if constexpr (NIT > 0) {
            float a[E];
            get_dyn(sq, it, a);
#pragma unroll
            for (int e = 0; e < E; ++e) w[e] = cq(a[e]);
            zero_excluded<E>(w, ((it * kWaves + wave_id()) * 64 + (int)(threadIdx.x & 63)), excl, n_excl);
        }
    };
    auto draw = [&](float u, float W) {
        if constexpr (NIT > 0) {
            // draws with replacement follow each other with no barrier in between: the result
            // slot in LDS must have been read by every wave before the next draw writes it
            if constexpr (METHOD == kRRS) __syncthreads();
            return __builtin_amdgcn_readfirstlane(draw_resident<E>(rq.nslab, u, W, sv, cw_reg, sh));
        } else {
            return icdf_slabs<E>(rq.nslab, u, W, sv, cw);
        }
    };
    auto remove_token = [&](int v) {
        excl[n_excl++] = v;
        const int s = v / (64 * E);
        float t;
        if constexpr (NIT > 0) {
            if (wave_id() == s % kWaves) {
                float w[E];
                cw_reg(s / kWaves, w);
                const float ts = wave_sum(chunk_sum<E>(w));
                if ((threadIdx.x & 63) == 0) sh.bcast_f = ts;
            }
            __syncthreads();
            t = sh.bcast_f;
        } else {
            float w[E];
            cw(s, w);
            t = wave_sum(chunk_sum<E>(w));
        }
        int j = 0;
        while (j < n_ov && ov_slab[j] != s) ++j;
        ov_slab[j] = s;
        ov_val[j] = t;
        if (j == n_ov) ++n_ov;
    };

    int out_tok[MDSD_MAX_K];
    if constexpr (METHOD == kSpecHub) {
        const float W = slab_total(rq.nslab, sv);
        const int v = draw(ur[0], W);
        // the mass outside the hub: for the second draw, and for the verify call if it asked
        float W2 = 0.f;
        if (v == a_virt || P.stats_out) {
            remove_token(a_virt);
            W2 = slab_total(rq.nslab, sv);
            if (P.stats_out && threadIdx.x == 0)
                P.stats_out[row] = mdsd_row_stats{mm[0], W2, a_virt - rq.head, 0};
        }
        if (v != a_virt) {
            out_tok[0] = v < 0 ? -1 : v - rq.head;
            out_tok[1] = a_virt - rq.head;
        } else {
            int v2 = draw(ur[1], W2);
            if (v2 < 0) {
                v2 = a_virt;
                flags |= MDSD_FLAG_DEGENERATE_HUB;
            }
            out_tok[0] = a_virt - rq.head;
            out_tok[1] = v2 - rq.head;
        }
    } else {
        int prev = rq.head;
        for (int i = 0; i < k; ++i) {
            const float W = slab_total(rq.nslab, sv);
            if (i == 0 && P.stats_out && threadIdx.x == 0)  // with replacement: maximum and total mass
                P.stats_out[row] = mdsd_row_stats{mm[0], W, -1, 0};
            int v = draw(ur[i], W);
            if (v < 0) {
                v = prev;
                flags |= MDSD_FLAG_Q_EXHAUSTED;
            } else if (METHOD == kRRSw) {
                remove_token(v);
            }
            prev = v;
            out_tok[i] = v - rq.head;
        }
    }
    if (threadIdx.x == 0) {
        for (int i = 0; i < k; ++i) xt[i] = out_tok[i];
        if (P.hub_out) P.hub_out[row] = (METHOD == kSpecHub) ? a_virt - rq.head : -1;
        if (P.flags) P.flags[row] = flags;
    }
}

// ---------------------------------------------------------------- tree walk
__global__ void tree_walk_kernel(const int32_t* outcome, const int32_t* token, int B, int N, int k,
                                 int depth, const int32_t* first_child, int32_t* accept_depth,
                                 int32_t* emitted)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t* oc = outcome + (int64_t)b * N;
    const int32_t* tk = token + (int64_t)b * N;
    int32_t* em = emitted + (int64_t)b * depth;
    for (int i = 0; i < depth; ++i) em[i] = -1;
    int n = 0, d = 0;
    for (;;) {
        if (d < depth) em[d] = tk[n];
        int c0;
        if (first_child) {
            c0 = first_child[n];
        } else {
            const int64_t c = (int64_t)k * n + 1;
            c0 = (c + k <= N) ? (int)c : -1;
        }
        const int o = oc[n];
        if (c0 < 0 || o < 0 || o >= k || d + 1 >= depth) break;
        n = c0 + o;
        if (n >= N) break;
        ++d;
    }
    accept_depth[b] = d;
}

// ---------------------------------------------------------------- Philox4x32-10
// Salmon, Moraes, Dror, Shaw, SC'11: ten rounds of two 32x32->64 multiplies,
// swap and xor with the key; the key advances by the two Weyl constants.
__global__ void philox_uniform_kernel(uint32_t k0, uint32_t k1, uint32_t stream_id, int64_t rows,
                                      int slots, float* out, uint32_t* words)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int blocks_per_row = (slots + 3) >> 2;
    if (i >= rows * blocks_per_row) return;
    const int64_t row = i / blocks_per_row;
    const int blk = (int)(i - row * blocks_per_row);
    uint32_t c0 = (uint32_t)row, c1 = (uint32_t)((uint64_t)row >> 32), c2 = (uint32_t)blk, c3 = stream_id;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0;
        c1 = l1;
        c2 = n2;
        c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    const uint32_t w[4] = {c0, c1, c2, c3};
    for (int j = 0; j < 4; ++j) {
        const int s = blk * 4 + j;
        if (s < slots) {
            if (out) out[row * slots + s] = (float)(w[j] >> 8) * (1.0f / 16777216.0f);
            if (words) words[row * slots + s] = w[j];
        }
    }
}

// ---------------------------------------------------------------- host side
static int complete_tree_nodes(int k, int depth, int64_t* n_internal)
{
    int64_t n = 0, level = 1, internal = 0;
    for (int d = 0; d < depth; ++d) {
        if (d == depth - 1) internal = n;
        n += level;
        level *= k;
        if (n > INT_MAX) return -1;
    }
    *n_internal = internal;
    return (int)n;
}

// what validate returns for a batch of no trees: the entry points then return MDSD_OK at once
static constexpr int kEmptyBatch = 1;

static int validate(const mdsd_problem* pb, int method, bool need_target, Params* P)
{
    if (!pb) return MDSD_E_NULL;
    if (pb->B == 0) return kEmptyBatch;
    if (!pb->draft || (need_target && !pb->target)) return MDSD_E_NULL;
    if (pb->dtype != MDSD_FP32 && pb->dtype != MDSD_BF16) return MDSD_E_DTYPE;
    if (pb->kind != MDSD_PROBS && pb->kind != MDSD_LOGITS) return MDSD_E_DTYPE;
    if (pb->B < 1 || pb->N < 1 || pb->V < 2 || pb->depth < 1) return MDSD_E_SHAPE;
    if (pb->ld_d < pb->V || (need_target && pb->ld_t < pb->V)) return MDSD_E_SHAPE;
    if (pb->k < 1 || pb->k > MDSD_MAX_K) return MDSD_E_K;
    if (method == kSpecHub && pb->k != 2) return MDSD_E_K;
    if (pb->kind == MDSD_LOGITS) {
        if (!(pb->temp_draft > 0.f)) return MDSD_E_TEMP;
        if (need_target && !(pb->temp_target > 0.f)) return MDSD_E_TEMP;
    }
    const int es = pb->dtype == MDSD_FP32 ? 4 : 2;
    const int per_chunk = 16 / es;
    // vocabulary bound of the per-slab partial sums kept in LDS
    if ((int64_t)pb->V + per_chunk > (int64_t)kMaxSlabs * 64 * per_chunk) return MDSD_E_SHAPE;
    if ((int64_t)pb->B * pb->N > INT_MAX) return MDSD_E_SHAPE;
    const uintptr_t at = (uintptr_t)pb->target, ad = (uintptr_t)pb->draft;
    if ((ad % es) != 0 || (need_target && (at % es) != 0)) return MDSD_E_ALIGN;
    if (need_target) {
        // every pair of rows must share its offset modulo 16 bytes
        if ((at & 15) != (ad & 15)) return MDSD_E_ALIGN;
        if (pb->B * (int64_t)pb->N > 1 && ((pb->ld_t * es) & 15) != ((pb->ld_d * es) & 15)) return MDSD_E_ALIGN;
    }
    int64_t n_internal = 0;
    if (!pb->first_child) {
        const int n = complete_tree_nodes(pb->k, pb->depth, &n_internal);
        if (n != pb->N) return MDSD_E_SHAPE;
    }
    P->target = pb->target;
    P->draft = pb->draft;
    P->ld_t = pb->ld_t;
    P->ld_d = pb->ld_d;
    P->temp_target = pb->temp_target;
    P->temp_draft = pb->temp_draft;
    P->B = pb->B;
    P->N = pb->N;
    P->V = pb->V;
    P->k = pb->k;
    P->depth = pb->depth;
    P->n_internal = (int)n_internal;
    P->first_child = pb->first_child;
    return MDSD_OK;
}

// chunks per lane that hold a whole row in registers; 0 = stream the row in every pass
static int resident_chunks(const mdsd_problem* pb)
{
    const int per_chunk = pb->dtype == MDSD_FP32 ? 4 : 8;
    // worst case head of per_chunk - 1 masked elements in front of the row
    const int64_t nchunk = ((int64_t)pb->V + 2 * per_chunk - 2) / per_chunk;
    const int64_t per_lane = (nchunk + kWG - 1) / kWG;
    if (per_lane <= 4) return 4;
    if (per_lane <= 8) return 8;
    if (per_lane <= 16) return 16;
    return 0;
}

template <int DT, bool LG, int METHOD>
static void launch_verify_n(int nit, bool path, dim3 grid, dim3 block, hipStream_t st, const Params& P)
{
    if (path) {
        // a tree's nodes follow one another: the row is streamed whatever its size would allow,
        // except for the common 8-chunk case
        if (nit == 8)
            hipLaunchKernelGGL((verify_path_kernel<DT, LG, METHOD, 8>), grid, block, 0, st, P);
        else
            hipLaunchKernelGGL((verify_path_kernel<DT, LG, METHOD, 0>), grid, block, 0, st, P);
        return;
    }
    switch (nit) {
    case 4: hipLaunchKernelGGL((verify_kernel<DT, LG, METHOD, 4>), grid, block, 0, st, P); break;
    case 8: hipLaunchKernelGGL((verify_kernel<DT, LG, METHOD, 8>), grid, block, 0, st, P); break;
    case 16: hipLaunchKernelGGL((verify_kernel<DT, LG, METHOD, 16>), grid, block, 0, st, P); break;
    default: hipLaunchKernelGGL((verify_kernel<DT, LG, METHOD, 0>), grid, block, 0, st, P); break;
    }
}

template <int DT>
static void launch_spechub_resident(int nit, bool masked, bool path, dim3 grid, dim3 block, hipStream_t st,
                                    const Params& P)
{
#define MDSD_LAUNCH_RES3(KERNEL, N, M)                                                              \
    if (P.stats_in)                                                                                 \
        hipLaunchKernelGGL((KERNEL<DT, N, M, true>), grid, block, 0, st, P);                        \
    else                                                                                            \
        hipLaunchKernelGGL((KERNEL<DT, N, M, false>), grid, block, 0, st, P)
#define MDSD_LAUNCH_RES2(N, M)                                                                      \
    if (path) {                                                                                     \
        MDSD_LAUNCH_RES3(spechub_path_resident, N, M);                                              \
    } else {                                                                                        \
        MDSD_LAUNCH_RES3(spechub_verify_resident, N, M);                                            \
    }
#define MDSD_LAUNCH_RES(N)                                                                          \
    if (masked) {                                                                                   \
        MDSD_LAUNCH_RES2(N, true);                                                                  \
    } else {                                                                                        \
        MDSD_LAUNCH_RES2(N, false);                                                                 \
    }
    if (nit == 4) {
        MDSD_LAUNCH_RES(4);
    } else if (nit == 8) {
        MDSD_LAUNCH_RES(8);
    } else {
        MDSD_LAUNCH_RES(16);
    }
#undef MDSD_LAUNCH_RES
#undef MDSD_LAUNCH_RES2
#undef MDSD_LAUNCH_RES3
}

// which shapes the RRS kernel for rows in registers is built for (the others would spill or run
// one workgroup per CU; they take the generic kernel): fp32 in every size, bf16 up to 8 chunks per
// lane and only for rows that need no masking
static bool rrs_resident_covers(int dtype, int nit, bool masked)
{
    return nit > 0 && (dtype == MDSD_FP32 || (nit <= 8 && !masked));
}

template <bool WO>
static void launch_rrs_resident(int dtype, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                                const Params& P)
{
#define MDSD_LAUNCH_RRS(DT, N, M) hipLaunchKernelGGL((rrs_verify_resident<DT, N, M, WO>), grid, block, 0, st, P)
    if (dtype == MDSD_FP32) {
        if (nit == 4) {
            if (masked) MDSD_LAUNCH_RRS(0, 4, true); else MDSD_LAUNCH_RRS(0, 4, false);
        } else if (nit == 8) {
            if (masked) MDSD_LAUNCH_RRS(0, 8, true); else MDSD_LAUNCH_RRS(0, 8, false);
        } else {
            if (masked) MDSD_LAUNCH_RRS(0, 16, true); else MDSD_LAUNCH_RRS(0, 16, false);
        }
    } else {
        if (nit == 4) MDSD_LAUNCH_RRS(1, 4, false); else MDSD_LAUNCH_RRS(1, 8, false);
    }
#undef MDSD_LAUNCH_RRS
}

// true when some element of some row may need masking: a row that does not start on a
// 16-byte boundary, or a vocabulary that is not a whole number of 16-byte chunks
static bool rows_need_mask(const mdsd_problem* pb)
{
    const int es = pb->dtype == MDSD_FP32 ? 4 : 2;
    const uintptr_t at = (uintptr_t)pb->target, ad = (uintptr_t)pb->draft;
    return (at & 15) || (ad & 15) || ((pb->ld_t * es) & 15) || ((pb->ld_d * es) & 15) || (pb->V % (16 / es));
}

// path == false: one workgroup per node.  path == true: one workgroup per tree.
template <int METHOD>
static void launch_verify(const mdsd_problem* pb, const Params& P, bool path, hipStream_t st)
{
    const dim3 grid((unsigned)(path ? P.B : P.B * P.N)), block(kWG);
    const bool lg = pb->kind == MDSD_LOGITS;
    int nit = resident_chunks(pb);
    if (METHOD == kSpecHub && lg && nit > 0) {
        if (pb->dtype == MDSD_FP32)
            launch_spechub_resident<0>(nit, rows_need_mask(pb), path, grid, block, st, P);
        else
            launch_spechub_resident<1>(nit, rows_need_mask(pb), path, grid, block, st, P);
        return;
    }
    if (METHOD != kSpecHub && lg && P.stats_in != nullptr && !path &&
        rrs_resident_covers(pb->dtype, nit, rows_need_mask(pb))) {
        // logit rows in registers, the draft call's records at hand
        launch_rrs_resident<METHOD == kRRSw>(pb->dtype, nit, rows_need_mask(pb), grid, block, st, P);
        return;
    }
    // The generic RRS rounds hold many registers beside two resident rows (8 chunks per lane and
    // row: more than 200, one workgroup per CU): from that size on the rows are streamed, which
    // measures faster (config 3, rrsw_verify: 117 -> 82 us).
    if (METHOD != kSpecHub && nit >= 8) nit = 0;
    if (pb->dtype == MDSD_FP32) {
        if (lg)
            launch_verify_n<0, true, METHOD>(nit, path, grid, block, st, P);
        else
            launch_verify_n<0, false, METHOD>(nit, path, grid, block, st, P);
    } else {
        if (lg)
            launch_verify_n<1, true, METHOD>(nit, path, grid, block, st, P);
        else
            launch_verify_n<1, false, METHOD>(nit, path, grid, block, st, P);
    }
}

template <int DT, bool LG, int METHOD>
static void launch_draft_n(int nit, bool masked, dim3 grid, dim3 block, hipStream_t st, const Params& P)
{
    // rows that need no masking of their first and last chunk: a variant without the checks,
    // for the two common register sizes
    if (!masked && nit == 4) {
        hipLaunchKernelGGL((draft_kernel<DT, LG, METHOD, 4, false>), grid, block, 0, st, P);
        return;
    }
    if (!masked && nit == 8) {
        hipLaunchKernelGGL((draft_kernel<DT, LG, METHOD, 8, false>), grid, block, 0, st, P);
        return;
    }
    switch (nit) {
    case 4: hipLaunchKernelGGL((draft_kernel<DT, LG, METHOD, 4>), grid, block, 0, st, P); break;
    case 8: hipLaunchKernelGGL((draft_kernel<DT, LG, METHOD, 8>), grid, block, 0, st, P); break;
    case 16: hipLaunchKernelGGL((draft_kernel<DT, LG, METHOD, 16>), grid, block, 0, st, P); break;
    default: hipLaunchKernelGGL((draft_kernel<DT, LG, METHOD, 0>), grid, block, 0, st, P); break;
    }
}

template <int METHOD>
static void launch_draft(const mdsd_problem* pb, const Params& P, hipStream_t st)
{
    const dim3 grid((unsigned)(P.B * P.N)), block(kWG);
    const bool lg = pb->kind == MDSD_LOGITS;
    const int nit = resident_chunks(pb);
    const int es = pb->dtype == MDSD_FP32 ? 4 : 2;
    const bool masked = ((uintptr_t)pb->draft & 15) || ((pb->ld_d * es) & 15) || (pb->V % (16 / es));
    if (pb->dtype == MDSD_FP32) {
        if (lg)
            launch_draft_n<0, true, METHOD>(nit, masked, grid, block, st, P);
        else
            launch_draft_n<0, false, METHOD>(nit, masked, grid, block, st, P);
    } else {
        if (lg)
            launch_draft_n<1, true, METHOD>(nit, masked, grid, block, st, P);
        else
            launch_draft_n<1, false, METHOD>(nit, masked, grid, block, st, P);
    }
}

static int walk(const mdsd_problem* pb, const int32_t* outcome, const int32_t* token,
                int32_t* accept_depth, int32_t* emitted, hipStream_t st)
{
    const int threads = 64;
    hipLaunchKernelGGL(tree_walk_kernel, dim3((pb->B + threads - 1) / threads), dim3(threads), 0, st,
                       outcome, token, pb->B, pb->N, pb->k, pb->depth, pb->first_child, accept_depth,
                       emitted);
    return hipGetLastError() == hipSuccess ? MDSD_OK : MDSD_E_LAUNCH;
}

static int verify_entry(int method, const mdsd_problem* pb, const int32_t* tokens, const float* u,
                        const mdsd_result* out, bool path, void* stream)
{
    Params P = {};
    const int rc = validate(pb, method, true, &P);
    if (rc == kEmptyBatch) return MDSD_OK;
    if (rc != MDSD_OK) return rc;
    if (!tokens || !u || !out || !out->outcome || !out->token) return MDSD_E_NULL;
    if ((out->accept_depth == nullptr) != (out->emitted == nullptr)) return MDSD_E_NULL;
    if (path && !out->accept_depth) return MDSD_E_NULL;
    if (path && out->resid_prob) return MDSD_E_UNSUPPORTED;
    P.accept_depth = out->accept_depth;
    P.emitted = out->emitted;
    P.tokens = tokens;
    P.u = u;
    P.outcome = out->outcome;
    P.token = out->token;
    P.resid_mass = out->resid_mass;
    P.flags = out->flags;
    P.resid_prob = out->resid_prob;
    P.stats_in = pb->draft_stats;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();
    if (method == kSpecHub)
        launch_verify<kSpecHub>(pb, P, path, st);
    else if (method == kRRS)
        launch_verify<kRRS>(pb, P, path, st);
    else
        launch_verify<kRRSw>(pb, P, path, st);
    if (hipGetLastError() != hipSuccess) return MDSD_E_LAUNCH;
    if (path) return MDSD_OK;  // the walk is part of the kernel
    if (out->accept_depth) return walk(pb, out->outcome, out->token, out->accept_depth, out->emitted, st);
    return MDSD_OK;
}

static int draft_entry(int method, const mdsd_problem* pb, const float* u, int32_t* tokens,
                       int32_t* hub, int32_t* flags, void* stream)
{
    Params P = {};
    const int rc = validate(pb, method, false, &P);
    if (rc == kEmptyBatch) return MDSD_OK;
    if (rc != MDSD_OK) return rc;
    if (!u || !tokens) return MDSD_E_NULL;
    P.u = u;
    P.tokens_out = tokens;
    P.hub_out = hub;
    P.flags = flags;
    P.stats_out = pb->draft_stats;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();
    if (method == kSpecHub)
        launch_draft<kSpecHub>(pb, P, st);
    else if (method == kRRS)
        launch_draft<kRRS>(pb, P, st);
    else
        launch_draft<kRRSw>(pb, P, st);
    return hipGetLastError() == hipSuccess ? MDSD_OK : MDSD_E_LAUNCH;
}

}  // namespace mdsd

// ---------------------------------------------------------------- C ABI
extern "C" {

size_t mdsd_workspace_bytes(const mdsd_problem* pb)
{
    (void)pb;
    return 0;  // every intermediate lives in registers and LDS
}

int spechub_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* hub, int32_t* flags,
                  void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::draft_entry(mdsd::kSpecHub, pb, u, tokens, hub, flags, stream);
}

int rrs_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* flags, void* ws,
              size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::draft_entry(mdsd::kRRS, pb, u, tokens, nullptr, flags, stream);
}

int rrsw_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* flags, void* ws,
               size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::draft_entry(mdsd::kRRSw, pb, u, tokens, nullptr, flags, stream);
}

int spechub_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                   void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kSpecHub, pb, tokens, u, out, false, stream);
}

int rrs_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
               void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kRRS, pb, tokens, u, out, false, stream);
}

int rrsw_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kRRSw, pb, tokens, u, out, false, stream);
}

int spechub_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                        void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kSpecHub, pb, tokens, u, out, true, stream);
}

int rrs_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                    void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kRRS, pb, tokens, u, out, true, stream);
}

int rrsw_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                     void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kRRSw, pb, tokens, u, out, true, stream);
}

int mdsd_tree_walk(const mdsd_problem* pb, const int32_t* outcome, const int32_t* token,
                   int32_t* accept_depth, int32_t* emitted, void* stream)
{
    if (!pb) return MDSD_E_NULL;
    if (pb->B == 0) return MDSD_OK;
    if (!outcome || !token || !accept_depth || !emitted) return MDSD_E_NULL;
    if (pb->B < 1 || pb->N < 1 || pb->depth < 1) return MDSD_E_SHAPE;
    if (pb->k < 1 || pb->k > MDSD_MAX_K) return MDSD_E_K;
    (void)hipGetLastError();
    return mdsd::walk(pb, outcome, token, accept_depth, emitted, (hipStream_t)stream);
}

int mdsd_philox_uniform(uint64_t seed, uint32_t stream_id, int64_t rows, int32_t slots, float* out,
                        uint32_t* words, void* stream)
{
    if (rows < 0 || slots < 1) return MDSD_E_SHAPE;
    if (rows == 0) return MDSD_OK;
    if (!out && !words) return MDSD_E_NULL;
    const int64_t n = rows * ((slots + 3) >> 2);
    const int threads = 256;
    const int64_t blocks = (n + threads - 1) / threads;
    if (blocks > INT_MAX) return MDSD_E_SHAPE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(mdsd::philox_uniform_kernel, dim3((unsigned)blocks), dim3(threads), 0,
                       (hipStream_t)stream, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, rows,
                       (int)slots, out, words);
    return hipGetLastError() == hipSuccess ? MDSD_OK : MDSD_E_LAUNCH;
}

const char* mdsd_strerror(int code)
{
    switch (code) {
    case MDSD_OK: return "ok";
    case MDSD_E_NULL: return "a required pointer is NULL";
    case MDSD_E_SHAPE: return "bad shape: B, N, V, ld, depth or tree/N mismatch";
    case MDSD_E_K: return "k out of range (SpecHub needs k == 2)";
    case MDSD_E_TEMP: return "temperature must be > 0";
    case MDSD_E_DTYPE: return "unknown dtype or kind";
    case MDSD_E_ALIGN: return "pointer not element-aligned, or target/draft rows differ modulo 16 bytes";
    case MDSD_E_WORKSPACE: return "workspace too small";
    case MDSD_E_LAUNCH: return "HIP launch failed";
    case MDSD_E_UNSUPPORTED: return "output not available from this entry point";
    default: return "unknown status";
    }
}

int mdsd_version(void) { return 102; }

}  // extern "C"
