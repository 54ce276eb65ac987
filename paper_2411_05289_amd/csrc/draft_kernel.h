// The draft kernel: the k draft tokens of every internal node (SpecHub: the pair from Q;
// RRS: k independent draws; RRSw: k draws without replacement), and the record of the draft row
// that the verify call can take over.  Instantiated per method in draft_*.hip.
#pragma once
#include "launch.h"

namespace MDSD_NS {

// ---------------------------------------------------------------- draft kernel
template <int DT, bool LOGITS, int METHOD, int NIT, bool MASKED = true>
__global__ __launch_bounds__(kWG * kNodesPerWG) void draft_kernel(const Params P)
{
    constexpr int E = Elem<DT>::kPerChunk;
    using CV = ToWeight<LOGITS>;
    __shared__ Shared shs[kNodesPerWG];
    Shared& sh = shs[node_slot()];
    int phase = 0;
    // one group of kWG threads per node; a leaf only records that it has no hub
    const NodeId id = node_of_block(P);
    if (id.b < 0) return;
    const int b = id.b, n = id.n, c0 = id.c0;
    const int64_t row = id.row;
    if (n == 0 && node_thread() == 0) P.tokens_out[(int64_t)b * P.N] = -1;
    if (c0 < 0) {
        if (node_thread() == 0) {
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
        int mq_chunk = 0;
        cq.s = P.scale_d;
        swept = sweep_streamed_row<DT, true, 2>(sq, cq.s, sh, phase, mm[0], Z, &mq_lane,
                                                METHOD == kSpecHub ? &mq_chunk : nullptr);
        if (swept) {
            cq.ms = mm[0] * cq.s;
            if constexpr (METHOD == kSpecHub) a_virt = block_argmax_at<DT>(rq, mq_lane, mm[0], mq_chunk, sh, phase);
        }
    }
    if (!swept) {
        if (LOGITS || METHOD == kSpecHub) {
            const float mq_lane = lane_max(sq);
            mm[0] = mq_lane;
            block_max<kWaves, 1>(mm, sh.red, phase);
            if constexpr (METHOD == kSpecHub) a_virt = block_argmax(sq, mq_lane, mm[0], sh, phase);
            if constexpr (LOGITS) {
                cq.s = P.scale_d;
                cq.ms = mm[0] * cq.s;
            }
        }
        pass_weights_to_slabs<CV>(sq, cq, nullptr, 0, sh.slab_w);
    }
    node_barrier();

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
            if constexpr (METHOD == kRRS) node_barrier();
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
            node_barrier();
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

    // Streamed rows: a token is taken out with the chunk that a load already brought (`raw`, the
    // chunk of slab s), so that its removal costs no trip to memory of its own
    auto set_override = [&](int s, float t) {
        int j = 0;
        while (j < n_ov && ov_slab[j] != s) ++j;
        ov_slab[j] = s;
        ov_val[j] = t;
        if (j == n_ov) ++n_ov;
    };
    auto remove_token_with = [&](int v, int s, const uint4& raw) {
        excl[n_excl++] = v;
        float a[E], w[E];
        finish_chunk<DT>(rq, s * 64 + (int)(threadIdx.x & 63), raw, CV::fill(), a);
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = cq(a[e]);
        zero_excluded<E>(w, s * 64 + (int)(threadIdx.x & 63), excl, n_excl);
        set_override(s, wave_sum(chunk_sum<E>(w)));
    };

    int out_tok[MDSD_MAX_K];
    if constexpr (METHOD == kSpecHub) {
        // streamed rows: the hub's chunk is asked for at once and arrives while the slab sums are searched
        uint4 hub_raw = make_uint4(0, 0, 0, 0);
        const int hub_slab = a_virt / (64 * E);
        if constexpr (NIT == 0) hub_raw = fetch_chunk(rq, hub_slab * 64 + (int)(threadIdx.x & 63));
        const float W = slab_total(rq.nslab, sv);
        const int v = draw(ur[0], W);
        // the mass outside the hub: for the second draw, and for the verify call if it asked
        float W2 = 0.f;
        if (v == a_virt || P.stats_out) {
            if constexpr (NIT == 0)
                remove_token_with(a_virt, hub_slab, hub_raw);
            else
                remove_token(a_virt);
            W2 = slab_total(rq.nslab, sv);
            if (P.stats_out && node_thread() == 0)
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
    } else if constexpr (NIT > 0 && METHOD == kRRS && kWaves > 1) {
        // rows in registers, k independent draws from one distribution: every wave finds the slab of
        // every draw, the wave that owns a drawn slab searches it, and all k results cross through
        // LDS behind one barrier instead of one barrier per draw (a node with a single wavefront has
        // no barriers to save and takes the plain loop below)
        const float W = slab_total(rq.nslab, sv);
        if (P.stats_out && node_thread() == 0) P.stats_out[row] = mdsd_row_stats{mm[0], W, -1, 0};
        for (int i = 0; i < k; ++i) {
            SlabHit h{-1, 0.f, 0.f};
            const bool found = icdf_find_slab(rq.nslab, ur[i], W, sv, h);  // the same in every wave
            if (found && wave_id() == h.slab % kWaves) {
                float w[E];
                cw_reg(h.slab / kWaves, w);
                const int v = icdf_in_slab<E>(w, h);
                if ((threadIdx.x & 63) == 0) sh.node_x[i] = v;
            }
            if (!found && node_thread() == 0) sh.node_x[i] = -1;
        }
        node_barrier();
        int prev = rq.head;
        for (int i = 0; i < k; ++i) {
            int v = sh.node_x[i];
            if (v < 0) {
                v = prev;
                flags |= MDSD_FLAG_Q_EXHAUSTED;
            }
            prev = v;
            out_tok[i] = v - rq.head;
        }
    } else if constexpr (NIT == 0 && METHOD == kRRS) {
        // streamed rows, k independent draws from one distribution: the slabs of up to four draws are
        // found first (slab sums, no memory), their chunks asked for together, and the draws finished as
        // the chunks arrive -- one trip to memory per four draws instead of one per draw
        const float W = slab_total(rq.nslab, sv);
        if (P.stats_out && node_thread() == 0) P.stats_out[row] = mdsd_row_stats{mm[0], W, -1, 0};
        int prev = rq.head;
        constexpr int kBatch = 4;
        for (int i0 = 0; i0 < k; i0 += kBatch) {
            SlabHit h[kBatch];
            uint4 raw[kBatch];
            bool found[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                h[j] = SlabHit{0, 0.f, 0.f};
                found[j] = i0 + j < k && icdf_find_slab(rq.nslab, ur[i0 + j < k ? i0 + j : 0], W, sv, h[j]);
                raw[j] = fetch_chunk(rq, (found[j] ? h[j].slab : 0) * 64 + (int)(threadIdx.x & 63));
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (i0 + j < k) {
                    int v = -1;
                    if (found[j]) {
                        float a[E], w[E];
                        finish_chunk<DT>(rq, h[j].slab * 64 + (int)(threadIdx.x & 63), raw[j], CV::fill(), a);
#pragma unroll
                        for (int e = 0; e < E; ++e) w[e] = cq(a[e]);
                        v = icdf_in_slab<E>(w, h[j]);
                    }
                    if (v < 0) {
                        v = prev;
                        flags |= MDSD_FLAG_Q_EXHAUSTED;
                    }
                    prev = v;
                    out_tok[i0 + j] = v - rq.head;
                }
            }
        }
    } else {
        int prev = rq.head;
        for (int i = 0; i < k; ++i) {
            const float W = slab_total(rq.nslab, sv);
            if (i == 0 && P.stats_out && node_thread() == 0)  // with replacement: maximum and total mass
                P.stats_out[row] = mdsd_row_stats{mm[0], W, -1, 0};
            int v;
            if constexpr (NIT == 0 && METHOD == kRRSw) {
                // streamed rows, without replacement: the drawn slab's chunk serves the draw and the
                // removal of the drawn token
                SlabHit h{-1, 0.f, 0.f};
                v = -1;
                if (icdf_find_slab(rq.nslab, ur[i], W, sv, h)) {
                    const uint4 raw = fetch_chunk(rq, h.slab * 64 + (int)(threadIdx.x & 63));
                    float a[E], w[E];
                    finish_chunk<DT>(rq, h.slab * 64 + (int)(threadIdx.x & 63), raw, CV::fill(), a);
#pragma unroll
                    for (int e = 0; e < E; ++e) w[e] = cq(a[e]);
                    zero_excluded<E>(w, h.slab * 64 + (int)(threadIdx.x & 63), excl, n_excl);
                    v = icdf_in_slab<E>(w, h);
                    if (v >= 0 && i + 1 < k) remove_token_with(v, h.slab, raw);  // the last draw removes nothing
                }
                if (v < 0) {
                    v = prev;
                    flags |= MDSD_FLAG_Q_EXHAUSTED;
                }
            } else {
                v = draw(ur[i], W);
                if (v < 0) {
                    v = prev;
                    flags |= MDSD_FLAG_Q_EXHAUSTED;
                } else if (METHOD == kRRSw && i + 1 < k) {
                    remove_token(v);  // (the last draw removes nothing)
                }
            }
            prev = v;
            out_tok[i] = v - rq.head;
        }
    }
    if (node_thread() == 0) {
        for (int i = 0; i < k; ++i) xt[i] = out_tok[i];
        if (P.hub_out) P.hub_out[row] = (METHOD == kSpecHub) ? a_virt - rq.head : -1;
        if (P.flags) P.flags[row] = flags;
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
static void launch_draft_method(int dtype, bool logits, int nit, bool masked, dim3 grid, dim3 block, hipStream_t st,
                                const Params& P)
{
    if (dtype == MDSD_FP32) {
        if (logits)
            launch_draft_n<0, true, METHOD>(nit, masked, grid, block, st, P);
        else
            launch_draft_n<0, false, METHOD>(nit, masked, grid, block, st, P);
    } else {
        if (logits)
            launch_draft_n<1, true, METHOD>(nit, masked, grid, block, st, P);
        else
            launch_draft_n<1, false, METHOD>(nit, masked, grid, block, st, P);
    }
}

}  // namespace MDSD_NS
