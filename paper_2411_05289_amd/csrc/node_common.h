// Device code shared by every kernel family of the library: the LDS layout of a node's
// threads, the node a workgroup owns, the passes over a row (maximum, argmax,
// weights to slab sums, draws), the element arithmetic of the three methods, the leaf case,
// the path-only walk and the one-sweep statistics of a streamed row.
//
// A group of kWG threads (512 = 8 wavefronts in the main build, fewer in the builds for short
// rows: build_config.h) owns one tree node -- or, in the path-only
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
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <limits.h>
#include <stdlib.h>
#include <stdint.h>

#include "mdsd.h"
#include "params.h"
#include "resident.h"
#include "scan_core.h"

namespace MDSD_NS {

enum Method { kSpecHub = 0, kRRS = 1, kRRSw = 2 };

// SpecHub verify with draft statistics: chunks of the draft row requested ahead of their use in
// the residual pass (one is enough: a chunk pair is about 150 instructions of work for each of
// the 6 waves that share a SIMD), and the waves per SIMD the kernel is held to (6 = 80
// registers per lane = three workgroups per compute unit; 8 would spill).
constexpr int kStreamAhead = 1;
constexpr int kStatsWavesPerSimd = 6;

using ::mdsd::Params;

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
        // an entry that does not point past its own node, or leaves no room for k children, is
        // treated as a leaf (the tree walk applies the same rule, so it always ends)
        if (id.c0 <= id.n || id.c0 + P.k > P.N) id.c0 = -1;
    }
    id.row = (int64_t)id.b * P.N + id.n;
    return id;
}

// Complete trees are launched on a grid of (trees, nodes): the node number is the slow index, so
// the workgroups still start in the order "nodes with children first", and nothing has to be
// divided to find the tree and the node.  Other launches number their workgroups in one
// dimension (gridDim.y == 1) and take the division.
__device__ __forceinline__ NodeId node_of_block(const Params& P)
{
    if constexpr (kNodesPerWG > 1) {
        // several nodes per workgroup, numbered in one dimension; a slot past the last node has
        // none (b = -1) and its wavefront leaves at once
        const int64_t w = (int64_t)blockIdx.x * kNodesPerWG + node_slot();
        if (w >= (int64_t)P.B * P.N) return NodeId{-1, -1, -1, -1};
        return node_of_item(P, (int)w);
    }
    if (gridDim.y == 1) return node_of_item(P, blockIdx.x);
    NodeId id;
    // Workgroup i of a launch runs on XCD i mod 8, and with the tree as the fast index that would
    // be the tree's number mod 8 for every node: trees whose nodes cost more than others' (a
    // poorer draft model) would weigh on one XCD.  Node n of a group of 8 trees is handed round
    // inside the group instead.
    id.n = blockIdx.y;
    id.b = (P.B & 7) == 0 ? (int)(blockIdx.x ^ (blockIdx.y & 7u)) : (int)blockIdx.x;
    id.c0 = id.n < P.n_internal ? P.k * id.n + 1 : -1;
    id.row = (int64_t)id.b * P.N + id.n;
    return id;
}

// ---------------------------------------------------------------- tree walk and node outputs
// Sec. 2: follow the accepted children from the root; every visited node emits its token; stop at
// the first node without an accepted child.  A first_child entry that does not point past its own
// node or leaves no room for k children inside the tree counts as a leaf, here as in
// node_of_item(): node numbers grow along the walk, which therefore ends.
__device__ __forceinline__ int walk_first_child(const int32_t* first_child, int n, int k, int N)
{
    if (first_child) {
        const int c0 = first_child[n];
        return (c0 <= n || c0 + k > N) ? -1 : c0;
    }
    const int64_t c = (int64_t)k * n + 1;
    return (c + k <= N) ? (int)c : -1;
}

// One entry of outcome[] / token[].  COHERENT: the value was written by another workgroup of the
// same launch, possibly on another XCD, whose L2 this one does not share: written and read with
// device-scope atomic accesses (which go to memory), it is seen without flushing either cache.
template <bool COHERENT>
__device__ __forceinline__ int load_node_word(const int32_t* p)
{
    if constexpr (COHERENT)
        return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        return *p;
}

// The walk of trees of at most 64 nodes by groups of W lanes (W a power of two, N <= W <= 64):
// lane l of a group fetches node l of the group's tree b, so the whole tree arrives in one trip to
// memory and the walk runs on registers; a wavefront walks 64 / W trees side by side.  All 64 lanes
// are active; tree_ok is false in the lanes of a group that has no tree.
template <bool COHERENT>
__device__ __forceinline__ void group_walk(const int32_t* outcome, const int32_t* token, int b, bool tree_ok, int W,
                                           int N, int k, int depth, const int32_t* first_child,
                                           int32_t* accept_depth, int32_t* emitted)
{
    const int lane = threadIdx.x & 63;
    const int l = lane & (W - 1), base = lane - l;
    const bool in_tree = tree_ok && l < N;
    const int32_t* oc = outcome + (int64_t)b * N;
    const int32_t* tk = token + (int64_t)b * N;
    const int o_l = in_tree ? load_node_word<COHERENT>(oc + l) : -1;
    const int t_l = in_tree ? load_node_word<COHERENT>(tk + l) : -1;
    const int c_l = in_tree ? walk_first_child(first_child, l, k, N) : -1;
    int n = 0, d = 0, mine = -1;  // lane d of the group keeps the token emitted at depth d (d < N <= W)
    bool alive = tree_ok;
    // the same number of steps in every group (the shuffles need every lane): the longest path
    const int steps = depth < W ? depth : W;
    for (int s = 0; s < steps; ++s) {
        const int t = __shfl(t_l, base + n, 64), o = __shfl(o_l, base + n, 64), c = __shfl(c_l, base + n, 64);
        if (alive && l == d) mine = t;
        if (alive && !(c < 0 || o < 0 || o >= k || d + 1 >= depth || d + 1 >= W)) {
            n = c + o;  // < N: c + k <= N
            ++d;
        } else {
            alive = false;
        }
    }
    if (!tree_ok) return;
    int32_t* em = emitted + (int64_t)b * depth;
    for (int i = l; i < depth; i += W) em[i] = i < W ? mine : -1;
    if (l == 0) accept_depth[b] = d;
}

// The walk of tree b by one wavefront (all 64 lanes active, the same b in every lane).  Trees of
// at most 64 nodes: on registers, as above.  Larger trees: node after node from memory.
template <bool COHERENT>
__device__ __forceinline__ void wave_walk(const int32_t* outcome, const int32_t* token, int b, int N, int k,
                                          int depth, const int32_t* first_child, int32_t* accept_depth,
                                          int32_t* emitted)
{
    const int lane = threadIdx.x & 63;
    if (N <= 64) {
        group_walk<COHERENT>(outcome, token, b, true, 64, N, k, depth, first_child, accept_depth, emitted);
    } else {
        const int32_t* oc = outcome + (int64_t)b * N;
        const int32_t* tk = token + (int64_t)b * N;
        int32_t* em = emitted + (int64_t)b * depth;
        if (lane == 0) {
            for (int i = 0; i < depth; ++i) em[i] = -1;
            int n = 0, d = 0;
            for (;;) {
                const int t = load_node_word<COHERENT>(tk + n), o = load_node_word<COHERENT>(oc + n);
                if (d < depth) em[d] = t;
                const int c = walk_first_child(first_child, n, k, N);
                if (c < 0 || o < 0 || o >= k || d + 1 >= depth) break;
                n = c + o;
                ++d;
            }
            accept_depth[b] = d;
        }
    }
}

// The outputs of one node, written by the first thread of the workgroup (whose copy of them is
// always complete).  With P.tree_count the kernel also walks the trees: the workgroup that
// brings a tree's last node walks it.  Its nodes' outcomes and tokens then cross from workgroup to
// workgroup inside one launch: they are stored with device-scope atomic stores (which go to
// memory), the store is waited for, and only then is the tree's arrival counted, so whoever
// counts N arrivals finds every node's words in memory; it reads them with device-scope atomic
// loads.  No cache is flushed or invalidated.  The counter is set back to 0 for the next launch.
__device__ __forceinline__ void write_node_outputs(const Params& P, const NodeId& id, int outcome, int token,
                                                   float rmass, int flags)
{
    if (node_thread() >= kWave) return;
    const bool first = node_thread() == 0;
    if (first) {
        if (P.resid_mass) P.resid_mass[id.row] = rmass;
        if (P.flags) P.flags[id.row] = flags;
    }
    if (P.tree_count == nullptr) {
        if (first) {
            P.outcome[id.row] = outcome;
            P.token[id.row] = token;
        }
        return;
    }
    int arrived = 0;
    if (first) {
        __hip_atomic_store(P.outcome + id.row, outcome, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(P.token + id.row, token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // both stores have reached memory
        arrived = __hip_atomic_fetch_add(P.tree_count + id.b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    arrived = __builtin_amdgcn_readfirstlane(arrived);
    if (arrived != P.N - 1) return;
    wave_walk<true>(P.outcome, P.token, id.b, P.N, P.k, P.depth, P.first_child, P.accept_depth, P.emitted);
    if (first) __hip_atomic_store(P.tree_count + id.b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

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

// The same for a streamed row whose sweep remembered, per lane, the first chunk that holds the
// lane's maximum: the lanes that hold the row's maximum read that one chunk again, instead of
// streaming their share of the row a second time.
template <int DT>
__device__ __forceinline__ int block_argmax_at(const RowView& r, float m_lane, float m_block, int chunk_of_max,
                                               Shared& sh, int& phase)
{
    constexpr int E = Elem<DT>::kPerChunk;
    int idx = INT_MAX;
    if (m_lane == m_block) {
        float a[E];
        load_chunk<DT>(r, chunk_of_max, -__builtin_inff(), a);
#pragma unroll
        for (int e = E - 1; e >= 0; --e)
            if (a[e] == m_block) idx = chunk_of_max * E + e;
    }
    const int a = block_min_index<kWaves>(idx, sh.red, phase);
    return a == INT_MAX ? r.head : a;  // a row of NaNs has no maximum: stay in bounds
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
    node_barrier();
    return sh.bcast_i;
}

// Softmax statistics of a row in registers with one barrier instead of two.  Every wave shifts
// by a maximum of its own (r_w, the largest of its lanes' values lane_m: their maxima, or the
// cheap estimates of them) and sums its weights; after one barrier the waves' pairs (r_w, Z_w)
// are combined: M = max r_w, Z = sum Z_w f_w with f_w = 2^((r_w - M) s) <= 1.  The factors are
// formed from the rounded products r_w s themselves (the largest of them is the shift `ms` that
// later passes use), so that a wave's weights times its factor are the weights those passes
// compute, not merely close to them.  A wave far below the maximum contributes its true,
// negligible share.  With SLABS the slab sums left in
// LDS are in their wave's own units: slab i counts f_(i mod kWaves) times its stored value, and
// f_lane is that factor for the slabs this lane reads in slab_total() and icdf_find_slab()
// (slab = a multiple of 64 + lane).
struct RowNorm {
    float ms, Z, f_lane;  // ms = M s, the shift of 2^(l s - ms)
};

template <bool SLABS, class Src>
__device__ __forceinline__ RowNorm wave_shifted_norm(const Src& sp, float s, float lane_m, Shared& sh, int& phase)
{
    static_assert((kWaves & (kWaves - 1)) == 0 && kWaves <= 64, "waves per workgroup: a power of two");
    constexpr int E = Src::E;
    const int lane = threadIdx.x & 63, wave = wave_id();
    float r = wave_max(lane_m);
    bool has_ref = r > -__builtin_inff() && r < __builtin_inff();
    // The cheap estimates can miss every finite element of a wave: a 32-bit word whose upper
    // half is -inf reads as -inf or as a NaN (which the maximum drops) whatever its lower half
    // holds, so a wave whose finite logits all sit at even indices (rows with most tokens masked)
    // would have nothing to refer to although it holds mass.  Such a wave takes the exact
    // maximum of its elements instead (a branch the whole wave takes together, rarely).
    if (!has_ref) {
        r = wave_max(lane_max(sp));
        has_ref = r > -__builtin_inff() && r < __builtin_inff();
    }
    // a wave that really has nothing finite (its chunks lie past the row or hold -inf only)
    // shifts by 0, sums to 0 and stays out of the maximum
    if (!has_ref) r = 0.f;
    r = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, r)));
    ToWeight<true> cw;
    cw.s = s;
    cw.ms = r * s;
    float z = 0.f;
    SlabSums<Src::kNit> sums;
    sp.for_each_it([&](int it, int, int, const float(&a)[E]) {
        float w[E];
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = cw(a[e]);
        const float cs = chunk_sum<E>(w);
        z += cs;
        if constexpr (SLABS) sums.put(it, cs);
    });
    const float zw = wave_sum(z);
    if (lane == 0) {
        sh.red.buf[phase][wave][0] = has_ref ? cw.ms : -__builtin_inff();
        sh.red.buf[phase][wave][1] = zw;
    }
    if constexpr (SLABS) sums.store(sh.slab_w, sp.r.nslab);
    node_barrier();
    float ms = sh.red.buf[phase][0][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, sh.red.buf[phase][w][0]);
    float Z = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
        Z += sh.red.buf[phase][w][1] * __builtin_amdgcn_exp2f(sh.red.buf[phase][w][0] - ms);
    const float f_lane = __builtin_amdgcn_exp2f(sh.red.buf[phase][lane & (kWaves - 1)][0] - ms);
    phase ^= 1;
    return RowNorm{ms, Z, f_lane};
}

// leaf: bonus token ~ p (the k = 0 case of Alg. 1).
// EVERY_WAVE = false: only the first wave's copy of `o` is complete (the caller's first thread
// writes the node's outputs): the search for the drawn slab and inside it is then left to that
// wave, which reads the slab's chunk from memory, instead of being repeated by all eight.
template <int DT, int NIT, bool MASKED, bool EVERY_WAVE = true>
__device__ __forceinline__ void leaf_resident(const Params& P, const RowView& rp,
                                              const RowSrc<DT, NIT, MASKED>& sp, float u, float* rprob,
                                              Shared& sh, int& phase, NodeOut& o)
{
    constexpr int E = Elem<DT>::kPerChunk;
    using Src = RowSrc<DT, NIT, MASKED>;
    ExpW cp;
    cp.s = P.scale_t;
    float f_lane = 1.f;
    auto sv = [&](int i) { return sh.slab_w[i] * f_lane; };  // i = a multiple of 64 + lane
    float W;
    // the cheap estimate of the maximum as the shift where there is one; if the weights
    // overflowed or vanished with it, once more with the maximum itself
    auto slab_sums = [&](float lane_m) {
        const RowNorm n = wave_shifted_norm<true>(sp, cp.s, lane_m, sh, phase);
        cp.ms = n.ms;
        f_lane = n.f_lane;
        return slab_total(rp.nslab, sv);
    };
    if constexpr (Src::kHasShiftEstimate) {
        W = slab_sums(sp.lane_shift_estimate());
        if (__builtin_expect(!(W > 0.f && W < __builtin_inff()), 0)) {
            node_barrier();  // every wave has read the slab sums that are about to be rewritten
            W = slab_sums(lane_max(sp));
        }
    } else {
        W = slab_sums(lane_max(sp));
    }
    int v = -1;
    if constexpr (EVERY_WAVE) {
        v = draw_resident<E>(rp.nslab, u, W, sv, [&](int it, float(&w)[E]) {
            float a[E];
            get_dyn(sp, it, a);
#pragma unroll
            for (int e = 0; e < E; ++e) w[e] = cp(a[e]);
        }, sh);
    } else if (wave_id() == 0) {
        v = icdf_slabs<E>(rp.nslab, u, W, sv, [&](int s, float(&w)[E]) {
            chunk_weights<DT, ExpW>(rp, cp, nullptr, 0, s, w);
        });
    }
    o.token = v < 0 ? -1 : v - rp.head;
    if (v < 0) o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
    o.rmass = 1.f;
    if (rprob)
        write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
            chunk_weights<DT, ExpW>(rp, cp, nullptr, 0, s, w);
        });
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform(float v) { return as_f(__builtin_amdgcn_readfirstlane(as_i(v))); }

// Path-only verification (Sec. 2: only the nodes the walk visits decide what a step emits): one
// workgroup per tree starts at the root, verifies a node, and moves to the accepted child until
// a node accepts nothing, a leaf has given its bonus token, or `depth` tokens are out.  Nodes
// off the path keep outcome MDSD_UNVISITED.  verify_node(id) handles one node and returns its
// outcome and token, uniform over the workgroup.
template <class VerifyNode>
__device__ __forceinline__ void walk_and_verify(const Params& P, VerifyNode verify_node)
{
    const int b = (int)blockIdx.x * kNodesPerWG + node_slot();
    if (b >= P.B) return;
    for (int i = node_thread(); i < P.N; i += kWG) {
        const int64_t r = (int64_t)b * P.N + i;
        P.outcome[r] = MDSD_UNVISITED;
        P.token[r] = -1;
        if (P.flags) P.flags[r] = 0;
        if (P.resid_mass) P.resid_mass[r] = 0.f;
    }
    int32_t* em = P.emitted + (int64_t)b * P.depth;
    for (int i = node_thread(); i < P.depth; i += kWG) em[i] = -1;
    // the visited nodes' entries are rewritten below by another thread of this workgroup
    __threadfence_block();
    node_barrier();
    int n = 0, d = 0;
    for (;;) {
        NodeId id;
        id.b = b;
        id.n = n;
        if (P.first_child) {
            id.c0 = P.first_child[n];
            if (id.c0 <= n || id.c0 + P.k > P.N) id.c0 = -1;
        } else {
            const int64_t c = (int64_t)P.k * n + 1;
            id.c0 = (c + P.k <= P.N) ? (int)c : -1;
        }
        id.row = (int64_t)b * P.N + n;
        const NodeOut o = verify_node(id);
        const int outcome = uniform(o.outcome), token = uniform(o.token);
        if (node_thread() == 0 && d < P.depth) em[d] = token;
        if (id.c0 < 0 || outcome < 0 || outcome >= P.k || d + 1 >= P.depth) break;
        n = id.c0 + outcome;
        ++d;
        node_barrier();  // the next node reuses the LDS areas of this one
    }
    if (node_thread() == 0) P.accept_depth[b] = d;
}

// One sweep over a logit row that is streamed from memory (too long for registers), instead of
// a pass for the maximum and a pass for the weights.  Each wave forms its weights against a
// reference of its own, the largest element of its first slab; when the row's maximum M is
// known the partial sums are brought to the row's units by one factor per wave,
// 2^((reference - M) s) <= 1.  Returns false (caller falls back to two passes) when the sum
// came out zero or not finite (some later element lay too far above a wave's reference) or a
// wave's factor is below 2^-100 or above 2^100 (the latter only for a wave whose first slab held
// nothing finite, which refers to 0: its weights may then have lost their low bits).
// On success: M = maximum of the stored row, Z = sum of 2^((l - M) s); with SLABS the slab
// sums in LDS are in the same units and visible to every wave.
template <int DT, bool SLABS, int AHEAD = 1, class Src>
__device__ __forceinline__ bool sweep_streamed_row(const Src& src, float s, Shared& sh, int& phase, float& M,
                                                   float& Z, float* lane_max_out = nullptr,
                                                   int* lane_max_chunk_out = nullptr)
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
    int lane_m_chunk = 0;  // the first of this lane's chunks that holds lane_m
    src.template for_each<AHEAD>([&](int sl, int chunk, const float(&a)[E]) {
        float w[E];
        float cm = a[0];
#pragma unroll
        for (int e = 1; e < E; ++e) cm = fmaxf(cm, a[e]);
        if (lane_max_chunk_out) lane_m_chunk = cm > lane_m ? chunk : lane_m_chunk;
        lane_m = fmaxf(lane_m, cm);
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = cw(a[e]);
        const float cs = chunk_sum<E>(w);
        lane_z += cs;
        if constexpr (SLABS) store_slab_sum(sh.slab_w, sl, cs);
    });
    if (lane_max_out) *lane_max_out = lane_m;
    if (lane_max_chunk_out) *lane_max_chunk_out = lane_m_chunk;
    float mm[1] = {lane_m};
    block_max<kWaves, 1>(mm, sh.red, phase);
    M = mm[0];
    // A wave whose reference lies far below the maximum would scale its sums by a factor near
    // or below the smallest normal number and lose them: then the sweep does not count.
    // (formed from the rounded shifts, so that a wave's weights times its factor are the weights
    // a later pass computes with the shift M s, bit for bit)
    const float down = cw.ms - M * s;
    const float scale = uniform(__builtin_amdgcn_exp2f(down));
    float zz[1] = {!(fabsf(down) <= 100.f) ? __builtin_inff() : lane_z * scale};
    block_sum<kWaves, 1>(zz, sh.red, phase);  // barrier: every slab sum is stored
    Z = zz[0];
    const bool ok = Z > 0.f && Z < __builtin_inff();
    if constexpr (SLABS) {
        if (ok) {
            for (int i = wave + kWaves * lane; i < src.r.nslab; i += kWaves * 64) sh.slab_w[i] *= scale;
        }
        node_barrier();
    }
    return ok;
}

}  // namespace MDSD_NS
