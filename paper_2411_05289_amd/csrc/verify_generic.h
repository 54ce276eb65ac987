// The generic verify kernel: every method, probabilities or logits, rows in registers or
// streamed, one workgroup per node or (path-only) per tree.  Instantiated per method in
// verify_generic_*.hip.
#pragma once
#include "launch.h"

namespace MDSD_NS {

// The softmax scales arrive in scalar registers.  The streamed passes of the SpecHub form of this
// kernel measured 4 % slower with the scale as a scalar operand of their multiply-adds than with
// the scale in a vector register (config 4), so it is moved there once; the RRS forms have no
// register to spare for it (one more would cost them a wave per SIMD) and keep the scalar.
__device__ __forceinline__ float in_vgpr(float x)
{
    asm volatile("" : "+v"(x));
    return x;
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
            cp.s = (METHOD == kSpecHub ? in_vgpr(P.scale_t) : P.scale_t);
            swept = sweep_streamed_row<DT, true>(sp, cp.s, sh, phase, M, Z);
            cp.ms = M * cp.s;
        }
        if (!swept) {
            if constexpr (LOGITS) {
                float mm[1] = {lane_max(sp)};
                block_max<kWaves, 1>(mm, sh.red, phase);
                cp.s = (METHOD == kSpecHub ? in_vgpr(P.scale_t) : P.scale_t);
                cp.ms = mm[0] * cp.s;
            }
            pass_weights_to_slabs<CV>(sp, cp, nullptr, 0, sh.slab_w);
            node_barrier();
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
        // one wavefront per node: the rows are a few hundred bytes and every trip to memory is a
        // quarter of the node's life, so the draft row is asked for together with the target row
        if constexpr (kWaves == 1) need_q();
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
                    swept = sweep_streamed_row<DT, false>(sp, in_vgpr(P.scale_t), sh, phase, mm[0], z[0]);
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
                cp.s = in_vgpr(P.scale_t);
                cp.ms = mm[0] * cp.s;
                cq.s = in_vgpr(P.scale_d);
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
                for_each2<2>(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
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
                    node_barrier();
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
                    for_each2<2>(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
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
                            node_barrier();
                            pass_weights_to_slabs<CV>(sp, cp, nullptr, 0, sh.slab_w);
                            node_barrier();
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
                            swept = sweep_streamed_row<DT, false>(sp, P.scale_t, sh, phase, mm[0], z[0]);
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
                    cp.s = P.scale_t;
                    cp.ms = mm[0] * cp.s;
                    cq.s = P.scale_d;
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
                    if (i > 0) node_barrier();  // earlier readers of slab_w are done
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
                    node_barrier();
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
                        node_barrier();
                        need_q();
                        for_each2(sp, sq, [&](int s, int chunk, const float(&pa_)[E], const float(&qa_)[E]) {
                            float w[E];
#pragma unroll
                            for (int e = 0; e < E; ++e) w[e] = rrs_term(cp(pa_[e]), cq(qa_[e]), iZp, c_iZq);
                            if (slab_has_excluded<E>(s, xv, n_rej)) zero_excluded<E>(w, chunk, xv, n_rej);
                            store_slab_sum(sh.slab_w, s, chunk_sum<E>(w));
                        });
                        node_barrier();
                    }
                    auto sv = [&](int j) { return sh.slab_w[j]; };
                    const float W = slab_total(rp.nslab, sv);
                    // the mass the rejections took p down to: nothing rejected, nothing taken
                    // (rows of probabilities are used as given and need not sum to 1)
                    rmass = n_rej == 0 ? 1.f : W;
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

    write_node_outputs(P, id, outcome, token, rmass, flags);
    return NodeOut{outcome, token, flags, rmass};
}

template <int DT, bool LOGITS, int METHOD, int NIT>
__global__ __launch_bounds__(kWG * kNodesPerWG) void verify_kernel(const Params P)
{
    __shared__ Shared shs[kNodesPerWG];
    Shared& sh = shs[node_slot()];
    int phase = 0;
    const NodeId id = node_of_block(P);
    if (id.b < 0) return;
    verify_node<DT, LOGITS, METHOD, NIT>(P, id, sh, phase);
}

template <int DT, bool LOGITS, int METHOD, int NIT>
__global__ __launch_bounds__(kWG * kNodesPerWG) void verify_path_kernel(const Params P)
{
    __shared__ Shared shs[kNodesPerWG];
    Shared& sh = shs[node_slot()];
    int phase = 0;
    walk_and_verify(P, [&](const NodeId& id) { return verify_node<DT, LOGITS, METHOD, NIT>(P, id, sh, phase); });
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

template <int METHOD>
static void launch_verify_generic(int dtype, bool logits, int nit, bool path, dim3 grid, dim3 block, hipStream_t st,
                                  const Params& P)
{
    if (dtype == MDSD_FP32) {
        if (logits)
            launch_verify_n<0, true, METHOD>(nit, path, grid, block, st, P);
        else
            launch_verify_n<0, false, METHOD>(nit, path, grid, block, st, P);
    } else {
        if (logits)
            launch_verify_n<1, true, METHOD>(nit, path, grid, block, st, P);
        else
            launch_verify_n<1, false, METHOD>(nit, path, grid, block, st, P);
    }
}

}  // namespace MDSD_NS
