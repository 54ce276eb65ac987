// SpecHub verification (Alg. 3) for logit rows that fit in registers: the kernel bench.py times.
// Device code and kernels; the launchers are in the translation units that include this file
// (spechub_resident.hip: the main build; half_verify.hip: 256 threads per node).
#pragma once
#include "launch.h"

namespace MDSD_NS {

// Waves per SIMD the kernels are held to.  512 threads per node: with the draft call's records 6
// (80 registers, three workgroups per CU), without them 4, with 16 chunks per lane 2.  256 threads
// per node (16 chunks per lane, records at hand): 4 = 128 registers = four nodes per CU.
template <int NIT, bool STATS>
constexpr int kVerifyWavesPerSimd = kWG == 256 ? (STATS ? 4 : 2) : (NIT <= 8 ? (STATS ? kStatsWavesPerSimd : 4) : (STATS ? 4 : 2));

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

// then the stored logits at the tokens those loads named.  All of them are asked for at once,
// at indices brought into the row (a look-up inside a branch would be waited for inside it, and
// the next one would cost another trip to memory); what an unusable token read is dropped.
template <int DT, bool STATS>
__device__ __forceinline__ void fetch_node_lookups(const NodeId& id, int V, const RowView& rp, const RowView& rq,
                                                   NodeIn& in)
{
    if (id.c0 >= 0) {
        const int c1 = min(max(in.x1, 0), V - 1), c2 = min(max(in.x2, 0), V - 1);
        const float lp1 = load_elem<DT>(rp, c1), lq1 = load_elem<DT>(rq, c1);
        const float lp2 = load_elem<DT>(rp, c2), lq2 = load_elem<DT>(rq, c2);
        float lpa = 0.f;
        if constexpr (STATS) lpa = load_elem<DT>(rp, max(in.hub, 0));
        in.lp1 = in.tokens_ok ? lp1 : 0.f;
        in.lq1 = in.tokens_ok ? lq1 : 0.f;
        in.lp2 = in.tokens_ok ? lp2 : 0.f;
        in.lq2 = in.tokens_ok ? lq2 : 0.f;
        if constexpr (STATS) in.lpa = in.hub >= 0 ? lpa : 0.f;
    }
}

template <int DT, bool STATS>
__device__ __forceinline__ void fetch_node_inputs(const Params& P, const NodeId& id, const RowView& rp,
                                                  const RowView& rq, NodeIn& in)
{
    fetch_node_scalars<STATS>(P, id, in);
    fetch_node_lookups<DT, STATS>(id, P.V, rp, rq, in);
}

// internal node, SpecHub (Alg. 3)
// STATS: the hub and the draft row's normalisers come with the node (the draft call left
// them); the draft row is then only needed for the residual sums, and is asked for only once
// the first test has failed.
// EVERY_WAVE = false: only the first wave's copy of `o` is complete (the caller's first thread
// writes the node's outputs), and the final draw is left to that wave.
template <int DT, int NIT, bool MASKED, bool STATS, bool EVERY_WAVE = true>
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
    cp.s = P.scale_t;
    cq.s = P.scale_d;
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
            const RowNorm n = wave_shifted_norm<false>(sp, cp.s, lane_m, sh, phase);
            cp.ms = n.ms;
            z1[0] = n.Z;
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
        if constexpr (STATS) {
            // the drawn slab's share of both rows comes from memory a second time (2 KiB); W is
            // the same in every wave, so is the choice between the draw and the fall-back below
            v = -1;
            if (W > 0.f && (EVERY_WAVE || wave == 0))
                v = icdf_slabs<E>(rp.nslab, u2, W, sv, [&](int s, float(&w)[E]) {
                    spechub_chunk_w<DT, ExpW>(rp, rq, cp, cq, h, a_virt, s, w);
                });
        } else
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
        if (STATS ? !(W > 0.f) : v < 0) {
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
        if (v < 0) o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
        o.token = v < 0 ? -1 : v - rp.head;
    }
    if (rprob && !wrote_prob)
        write_resid_prob<DT>(rprob, rp, W, [&](int s, float(&w)[E]) {
            spechub_chunk_w<DT, ExpW>(rp, rq, cp, cq, h, a_virt, s, w);
        });
}

// One node of SpecHub verify for logit rows that fit in registers: every load of the node queued
// before anything waits, all passes over the target row from registers.  Writes the node's
// outputs and returns its outcome and token (with EVERY_WAVE the same values in every lane;
// without it only the first wave's copy is complete).
template <int DT, int NIT, bool MASKED, bool STATS, bool EVERY_WAVE = true>
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
        leaf_resident<DT, NIT, MASKED, EVERY_WAVE>(P, rp, sp, in.u2, rprob, sh, phase, o);
    else
        spechub_resident<DT, NIT, MASKED, STATS, EVERY_WAVE>(P, in, rp, rq, sp, sq, need_full, rprob, sh, phase, o);
    write_node_outputs(P, id, o.outcome, o.token, o.rmass, o.flags);
    return o;
}

// one workgroup per node
template <int DT, int NIT, bool MASKED, bool STATS>
__global__ __launch_bounds__(kWG, (kVerifyWavesPerSimd<NIT, STATS>)) void spechub_verify_resident(const Params P)
{
    __shared__ Shared sh;
    int phase = 0;
    // one node per workgroup: nobody but the thread that writes the outputs needs them
    spechub_node_resident<DT, NIT, MASKED, STATS, false>(P, node_of_block(P), sh, phase);
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

}  // namespace MDSD_NS
