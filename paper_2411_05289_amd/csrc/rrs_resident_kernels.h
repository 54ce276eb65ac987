// RRS and RRS without replacement (Alg. 1) for logit rows that fit in registers.
// Device code and kernels; the launchers are in the translation units that include this file
// (rrs_resident.hip: the main build; half_verify.hip: 256 threads per node).
#pragma once
#include "launch.h"

namespace MDSD_NS {

// ---------------------------------------------------------------- RRS / RRSw, rows in registers
// Alg. 1 for one internal node when the draft call left its record of the draft row (largest
// stored element, total mass): the target row sits in registers, the draft row is streamed once
// per rejected round, and a node whose first draft is accepted never reads it.  The state after
// i rejections is the residual U = max(p - c q, 0) with mass W (c_1 = 0, W_0 = 1,
// c_{i+1} = c_i + W_i rho_{i+1}): round i + 1 accepts x with probability U(x) / (W q_{i+1}(x)).
// WO (without replacement): q_{i+1} is q without the tokens rejected so far, rescaled by
// rho_{i+1} = (mass of q) / (mass left); the mass outside all k drafted tokens is summed (positive
// terms only) in the first pass over the draft row, the masses left are that plus the later drafts'.
// The first pass over the draft row leaves its first kDraftChunksKept chunks per lane in LDS, so
// that the passes of later rounds read only the rest of it from memory.
// (40 KB per node at 512 threads, three nodes per CU; 28 KB at 256 threads, four nodes per CU)
template <int NIT>
constexpr int kDraftChunksKept = kWG == 256 ? (NIT < 7 ? NIT : 7) : (NIT < 5 ? NIT : 5);

template <int DT, int NIT, bool MASKED, bool WO>
__device__ __forceinline__ void rrs_resident(const Params& P, const NodeId& id, const RowView& rp,
                                             const RowView& rq, const RowSrc<DT, NIT, MASKED>& sp,
                                             bool need_full, float* rprob, Shared& sh,
                                             uint4 (*q_kept)[kWG], int& phase, NodeOut& o)
{
    constexpr int E = Elem<DT>::kPerChunk;
    constexpr int HE = E / 2;
    using Src = RowSrc<DT, NIT, MASKED>;
    const int k = P.k;
    const float* ur = P.u + id.row * (k + 1);
    const int32_t* xt = P.tokens + (int64_t)id.b * P.N + id.c0;
    const mdsd_row_stats st = P.stats_in[id.row];
    // tokens, the stored logits at them and the uniforms go through LDS (lane i of the first wave
    // fetches draft i), so that no lane holds arrays of them; visible after the first barrier.
    // The tokens and uniforms come over the scalar path (their addresses are the same in every
    // lane), so that waiting for a token does not wait for the row behind it; the look-ups at the
    // tokens are then queued right behind the row, at indices brought into it, and arrive with it.
    int x = -1;
    float u_mine = 0.f;
    for (int i = 0; i < k; ++i) {
        const int xi = xt[i];
        const float ui = ur[i];
        if ((int)threadIdx.x == i) {
            x = xi;
            u_mine = ui;
        }
    }
    const float u_k = ur[k];
    {
        const bool ok = x >= 0 && x < P.V;
        const int xc = ok ? x : 0;
        if ((int)threadIdx.x < k) {
            const float lp = load_elem<DT>(rp, xc), lq = load_elem<DT>(rq, xc);
            sh.node_x[threadIdx.x] = ok ? x : -1;
            sh.node_lp[threadIdx.x] = ok ? lp : 0.f;
            sh.node_lq[threadIdx.x] = ok ? lq : 0.f;
            sh.node_u[threadIdx.x] = u_mine;
        }
    }
    if (threadIdx.x == 0) sh.node_u[k] = u_k;

    // ---- target row: shift (cheap estimate first, where there is one) and Zp
    ExpW cp, cq;
    cp.s = P.scale_t;
    cq.s = P.scale_d;
    cq.ms = uniform(st.max_stored * cq.s);
    float z1[1];
    auto normaliser = [&](float lane_m) {
        const RowNorm n = wave_shifted_norm<false>(sp, cp.s, lane_m, sh, phase);
        cp.ms = uniform(n.ms);
        z1[0] = n.Z;
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
    float c = 0.f, Wc = 1.f;
    bool decided = false, slabs_current = false;
    int n_rej = 0;
    float rem_k = 0.f;  // WO: unnormalised draft mass outside all k drafted tokens (after the first pass)
    // one pass over both rows: slab sums (and total) of max(p - c_new q, 0), rejected tokens masked;
    // with want_rem also the draft mass outside the drafted tokens
    auto residual_pass = [&](float c_new, bool want_rem, auto KEPT) {
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
        for_each_streamed_cached<1, kDraftChunksKept<NIT>, decltype(KEPT)::value>(lane_o, wave_o, sp, rq, ExpW::fill(), q_kept, [&](int it, int s, int chunk, const uint4& dp, const uint4& dq) {
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
                        const int off = sh.node_x[j] + rp.head - (chunk * E + hv * HE);
#pragma unroll
                        for (int e = 0; e < HE; ++e) {
                            if (off == e) {
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
        const float W_new = i == 0 ? residual_pass(c_new, WO, std::false_type{})
                                   : residual_pass(c_new, false, std::true_type{});
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
        residual_pass(c, false, std::false_type{});  // rare: all of the draft row from memory again
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
    o.rmass = n_rej == 0 ? 1.f : W;
    if (!decided) {
        // (the kernel's first thread writes the outputs: the first wave's draw is the one that counts)
        int v = -1;
        if (wave_id() == 0) v = icdf_slabs<E>(rp.nslab, sh.node_u[k], W, sv, cw);
        o.token = v < 0 ? -1 : v - rp.head;
        if (v < 0) o.flags |= MDSD_FLAG_ZERO_RESIDUAL;
    }
    if (rprob) write_resid_prob<DT>(rprob, rp, W, cw);
}

template <int DT, int NIT, bool MASKED, bool WO>
__device__ __forceinline__ NodeOut rrs_node_resident(const Params& P, const NodeId& id, Shared& sh,
                                                     uint4 (*q_kept)[kWG], int& phase)
{
    const bool need_full = (P.resid_mass != nullptr) || (P.resid_prob != nullptr);
    float* rprob = P.resid_prob ? P.resid_prob + id.row * (int64_t)P.V : nullptr;
    const RowView rp = make_row<DT>(P.target, P.ld_t, id.row, P.V);
    RowSrc<DT, NIT, MASKED> sp;
    sp.issue(rp, ExpW::fill());
    NodeOut o{MDSD_NONE, -1, 0, 0.f};
    if (id.c0 < 0) {
        leaf_resident<DT, NIT, MASKED, false>(P, rp, sp, P.u[id.row * (P.k + 1) + P.k], rprob, sh, phase, o);
    } else {
        const RowView rq = make_row<DT>(P.draft, P.ld_d, id.row, P.V);
        rrs_resident<DT, NIT, MASKED, WO>(P, id, rp, rq, sp, need_full, rprob, sh, q_kept, phase, o);
    }
    write_node_outputs(P, id, o.outcome, o.token, o.rmass, o.flags);
    return o;
}

template <int DT, int NIT, bool MASKED, bool WO>
__global__ __launch_bounds__(kWG, (kWG == 256 || NIT > 8 ? 4 : kStatsWavesPerSimd)) void rrs_verify_resident(const Params P)
{
    __shared__ Shared sh;
    __shared__ uint4 q_kept[kDraftChunksKept<NIT>][kWG];
    int phase = 0;
    rrs_node_resident<DT, NIT, MASKED, WO>(P, node_of_block(P), sh, q_kept, phase);
}

}  // namespace MDSD_NS
