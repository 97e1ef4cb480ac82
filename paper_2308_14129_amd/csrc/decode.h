// The closing work of one batch step (device side), carried by extra workgroups of the GRU
// kernel's grid (k_gru.hip):
//   decode_events   per event, from the rows of the distinct queries: the two logits of the
//                   decoder g of the paper's Sec. II-C and the three embedding rows
//   expand_queries  the optional inspection outputs, per query
//   finish_ahead    finishing pass (prepare.h) for the batch that the embedding launch has just
//                   prepared for the next step
// None of them touches the model state, so the same launch can run the GRU of the batch the NEXT
// step applies beside them.  gfx950 only.
#pragma once

#include "kernels_common.h"
#include "prepare.h"

namespace tig {

struct DecodeParams {
    int M, E, Ep, K;
    int n_event_blocks;    // one event per wavefront
    int n_expand_blocks;   // one query per wavefront (inspection outputs), 0 if none is wanted
    int n_fin_row_blocks;  // row references of the batch prepared ahead, grid-stride over its rows
    int n_fin_slot_blocks; // its slots, one entry per thread
};

__device__ inline int row_of_entry(const QuerySet &qs, int i, int entries)
{
    int s = qs.slot[i];
    if (s < 0) {
        const int rep = -s - 1;
        s = rep < entries ? qs.slot[rep] : 0;
    }
    return s >= 0 && s < entries ? s : 0;  // (a row per entry at most; anything else is not a row)
}

// score(a, b) = w_d2 . relu(W_d1 [emb_a | emb_b] + b_d1) + b_d2 from the per-row halves of layer 1
// that the embedding kernel left; the embedding rows of the event's three queries are copies of
// their distinct rows.  One wavefront, event b.
__device__ inline void decode_event(const StepArgs &a, const PackedWeights &w, const DecodeParams &p, int b)
{
    const int lane = lane_id();
    int row[3];
    row[0] = row_of_entry(a.qs, 2 * b, 2 * a.count);
    row[1] = row_of_entry(a.qs, 2 * b + 1, 2 * a.count);
    row[2] = a.roles == 3 ? 2 * a.count + b : row[1];
    const float b2 = w.dec_b2[0];
    // every load of a 128-dim chunk is requested before the first is used
    float part[2] = {0.0f, 0.0f};
    for (int j0 = 0; j0 < p.E; j0 += 2 * kWave) {
        float da[2], db[2][2], em[3][2], b1[2], w2[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = j0 + lane + kWave * u;
            const bool in = j < p.E;
            da[u] = in ? a.dec_a[(size_t)row[0] * p.Ep + j] : 0.0f;
            db[0][u] = in ? a.dec_b[(size_t)row[1] * p.Ep + j] : 0.0f;
            db[1][u] = in ? a.dec_b[(size_t)row[2] * p.Ep + j] : 0.0f;
            b1[u] = in ? w.dec_b1f[j] : 0.0f;
            w2[u] = in ? w.dec_w2[j] : 0.0f;
#pragma unroll
            for (int r = 0; r < 3; ++r)
                em[r][u] = in ? a.emb_u[(size_t)row[r] * p.E + j] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = j0 + lane + kWave * u;
            if (j < p.E) {
                const float x = da[u] + b1[u];
                part[0] += w2[u] * fmaxf(x + db[0][u], 0.0f);
                part[1] += w2[u] * fmaxf(x + db[1][u], 0.0f);
#pragma unroll
                for (int r = 0; r < 3; ++r)
                    if (r < a.roles)
                        a.emb[((size_t)r * a.count + b) * p.E + j] = em[r][u];
            }
        }
    }
    const float s_pos = wave_sum_uniform(part[0]) + b2;
    const float s_neg = wave_sum_uniform(part[1]) + b2;
    if (lane == 0) {
        a.score_pos[b] = s_pos;
        if (a.roles == 3)
            a.score_neg[b] = s_neg;
    }
}

// Inspection outputs of query q, in the order [sources | destinations | negatives].  One wavefront.
__device__ inline void expand_query(const StepArgs &a, const DecodeParams &p, int q)
{
    const int lane = lane_id();
    const int role = q / a.count, b = q - role * a.count;
    const int row = role < 2 ? row_of_entry(a.qs, 2 * b + role, 2 * a.count) : 2 * a.count + b;
    if (lane < p.K) {
        const size_t o = (size_t)q * p.K + lane, i = (size_t)row * p.K + lane;
        if (a.out_nbr_node)
            a.out_nbr_node[o] = a.qs.nbr[i];
        if (a.out_nbr_eid)
            a.out_nbr_eid[o] = a.qs.eid[i];
        if (a.out_nbr_ts)
            a.out_nbr_ts[o] = a.qs.ts[i];
    }
    if (lane == 0 && a.out_nbr_cnt)
        a.out_nbr_cnt[q] = a.qs.cnt[row];
    if (role < 2 && lane == 1 && a.out_is_winner && a.win_flags)
        a.out_is_winner[2 * b + role] = a.win_flags[2 * b + role];
}

// Block `blk` of the closing work; `waves` wavefronts per block.  Blocks beyond the params' counts
// do nothing.
__device__ inline void closing_block(const StepArgs &a, const PackedWeights &w, const DecodeParams &p, int blk,
                                     int waves)
{
    if (blk < p.n_event_blocks) {
        const int b = blk * waves + wave_id();
        if (b < a.count)
            decode_event(a, w, p, b);
        return;
    }
    blk -= p.n_event_blocks;
    if (blk < p.n_expand_blocks) {
        const int q = blk * waves + wave_id();
        if (q < a.roles * a.count)
            expand_query(a, p, q);
        return;
    }
    blk -= p.n_expand_blocks;
    // Finishing pass for the batch that the embedding launch has just prepared: its row
    // references against the batch the NEXT step will apply, and its slots.
    const QuerySet &nq = a.ded.qs;
    if (blk < p.n_fin_row_blocks) {
        const RefCtx c{a.num_nodes, a.fin_msg_key, a.fin_msg_first_eid, a.fin_msg_count};
        int n_u = *nq.n_u;
        n_u = n_u < 2 * a.fin_count ? n_u : 2 * a.fin_count;
        for (int row = blk * waves + wave_id(); row < n_u; row += p.n_fin_row_blocks * waves)
            finish_row(c, nq, p.K, row);
    } else if (blk - p.n_fin_row_blocks < p.n_fin_slot_blocks) {
        const int i = (blk - p.n_fin_row_blocks) * waves * kWave + (int)threadIdx.x;
        if (i < 2 * a.fin_count)
            finish_slots(nq, i, 2 * a.fin_count);
    }
}

}  // namespace tig
