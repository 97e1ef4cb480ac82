// Training step (paper Sec. II-C: the decoder's edge probabilities "provide the self-supervised
// signals for training"; Alg. 2: "Training and compute loss", "Backward and Optimize"), device side.
// gfx950 only, fp32.
//
// The step's forward pass is recomputed here with the intermediates a backward pass needs kept in
// memory (separate query / output projections and merge layers; the attention core in the
// re-associated form stated above k_tr_attn_fwd), then the loss (binary cross-entropy on the logits
// of each event against one negative), the hand-written backward pass and a plain SGD update of the
// fp32 master weights; the folded, lane-ordered weights that the inference kernels read are rebuilt
// from the masters afterwards (pack.hip).
//   k_tr_gather     the distinct queries as matrices: query rows, key / value rows of the filled
//                   neighbour slots, the list of those slots (a negative's neighbours are looked up here)
//   k_rowgemm       every layer product of the forward AND the backward pass over all rows at once on
//                   the matrix cores (fp32 16x16x4): query projection, q~ and the heads' outputs (one
//                   product per head in one launch), output projection, merge MLP, decoder, and
//                   their transposed products dX = dY W -- all over queries or events, none over slots
//   k_tr_attn_fwd / k_tr_attn_bwd   scores, softmax, weighted sums of the raw key / value rows of
//                   one query per wavefront, and their backward down to the raw rows' gradients
//   k_tr_pairs / k_tr_logit / k_tr_pair_scatter   around the decoder's two contractions: the decoder's
//                   input rows per (pair, event), logits and loss terms, and the gradients of those
//                   rows added into the distinct embedding rows' gradients
//   k_tr_scatter    the gradient w.r.t. state rows that this step's GRU wrote goes to those rows;
//                   time-encoding partial sums per query
//   k_tr_gru_gates / k_tr_gru_time   the GRU's backward pass over the applied winners: message rows
//                   from the memory as the step found it, gradients of the gate pre-activations (the
//                   gates themselves are left by the step's GRU launch), time-encoding gradient
//   k_gemm_tn       every weight gradient is dW = D^T X over the rows' stored (delta, input) pairs:
//                   a [out x in] contraction over thousands of rows on the matrix cores (fp32
//                   16x16x4), split over the row range, partial results added with atomics; they run
//                   on a second stream beside the rest of the backward pass (forked when their rows
//                   are complete, joined ahead of the update)
//   k_colsum        bias and time-encoding gradients: column sums of stored per-row values
//   k_tr_update     memory overwrite, sum of the loss terms and the SGD update in one launch
// Weight matrices are kept twice, [out x in] and transposed: a thread that owns an output reads
// the transposed copy, a thread that owns an input the native one, so both directions are
// coalesced.
#include <hip/hip_runtime.h>

#include <cstring>

#include "kernels_common.h"
#include "prepare.h"
#include "rowgemm.h"
#include "winners.h"

namespace tig {

namespace {

constexpr int kTrThreads = 256;

__device__ inline const float *state_row(const StepArgs &a, int M, int32_t ref)
{
    if (ref == kRefNone)
        return nullptr;
    if (ref >= 0)
        return (int64_t)ref < a.num_nodes ? a.mem + (size_t)ref * M : nullptr;
    return ~ref < 2 * a.msg_count ? a.staging + (size_t)(~ref) * M : nullptr;
}

// sin of the time-encoding phase (see time_enc): the derivative of Phi needs it
__device__ inline float time_enc_sin(double w_rev, double b_rev, double x)
{
    const double phase = fma(w_rev, x, b_rev);
    return __builtin_amdgcn_sinf((float)__builtin_amdgcn_fract(phase));
}

struct TrainDims {
    int M, T, F, E, K, H, da, dh, dkv, Dmsg;
};

// fp32 master weights ([out x in]), their transposes ([in x out]) and the step's buffers (device)
struct TrainBufs {
    const float *W_i, *b_i, *W_h, *b_h, *W_Q, *b_Q, *W_K, *b_K, *W_V, *b_V, *W_O, *b_O, *W_m1, *b_m1, *W_m2, *b_m2,
        *W_d1, *b_d1, *w_d2, *b_d2;
    const float *T_i, *T_h, *T_Q, *T_K, *T_V, *T_O, *T_m1, *T_m2, *T_d1;
    // per distinct query (compact row x: sources / destinations first, then the negatives)
    float *QIN, *QV, *O_, *PROB, *X1, *H1, *D_EMB, *DZ1, *D_ATTN, *DQV, *TG;
    float *QT, *KVB, *DKVB, *DQT;  // per head q~, the weighted sums of the key / value rows, and their gradients [H x dkv]
    float *DOUT, *DSU, *DQIN;  // gradients of the heads' outputs [da], of the own state through the merge layer [M], of the query row [da]
    int32_t *HAS;              // 1 for a query with at least one filled neighbour slot
    // per filled neighbour slot: slot k of query x is row slot0[x] + k (the filled slots of a step are packed)
    float *KV, *DKV;
    // per (pair, event): pair 0 = (source, destination), pair 1 = (source, negative); row p * count + b
    float *CAT, *DY, *G_, *DCAT, *DLOGIT, *LOSS;
    // per applied winner r, and per entry of the applied batch
    float *MSG, *GATES, *DGI, *DGH, *DPHI, *D_STAG;
    int32_t *n_rows;  // [1] distinct queries of the step (written by the forward kernel's block 0)
    int32_t *slot0;   // [3B] first row of a query's filled slots in the per-slot matrices
    int32_t *n_live;  // [1] filled slots of the step (cleared with the gradients)
};

// compact row of query-set row q
__device__ inline int compact_row(int q, int n_u, int count) { return q < 2 * count ? q : n_u + (q - 2 * count); }

// ------------------------------------------------------------------------------------------
constexpr int kRowWaves = kTrThreads / kWave;  // rows per workgroup of the per-row kernels (one wavefront each)

__device__ inline double shfl_f64(double v, int src)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl(lo, src);
    hi = __shfl(hi, src);
    return __hiloint2double(hi, lo);
}

// First per-slot row of query x; cnt drops to 0 if the rows would leave the per-slot matrices.
__device__ inline size_t slot_rows(const StepArgs &a, const TrainBufs &t, int x, int K, int &cnt)
{
    const int sb = cnt > 0 ? t.slot0[x] : 0;
    if (sb < 0 || sb + cnt > 3 * a.count * K)
        cnt = 0;
    return (size_t)(cnt > 0 ? sb : 0);
}

// The step's distinct queries laid out as matrices (one wavefront per query): the query row
// [s_u | Phi(0)], the own state as the tail of the merge layer's input, the key / value rows
// [s_v | e | Phi(t - t_k)] of the filled neighbour slots, and the list of those slots.  A negative's
// neighbours are looked up here.
constexpr int kGatherWaves = 16;  // queries per workgroup of k_tr_gather

__global__ void __launch_bounds__(kGatherWaves *kWave) k_tr_gather(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t)
{
    __shared__ int wg_cnt[kGatherWaves], wg_base;
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + a.count;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *t.n_rows = n_rows;
        if (a.rows_seen) {
            // hints for the host, as the embedding launch of an ordinary step leaves them: they size
            // the next step's launches (the GRU's column slices follow the winner count)
            a.rows_seen[0] = n_rows;
            if (a.msg_count > 0)
                a.rows_seen[1] = *a.n_win;
        }
    }
    const int x = (int)blockIdx.x * kGatherWaves + wave_id();
    const bool live_row = x < n_rows;  // (uniform over the wavefront; every wavefront reaches the barriers)
    const int lane = lane_id();
    const int M = d.M, F = d.F, K = d.K, da = d.da, dkv = d.dkv;
    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    int cnt = 0;
    int32_t sref = kRefNone, my_ref = kRefNone, my_eid = -1;
    double my_ts = 0.0, t_q = 0.0;
    if (!live_row) {
    } else if (x >= n_u) {
        const int b = x - n_u;
        t_q = a.ts[a.first_eid + b];
        cnt = finish_negative(a, K, b, my_ref, my_eid, my_ts);
        sref = resolve_ref(ref_ctx(a), a.neg[b]);
        if (lane == 0)
            a.qs.self_ref[q] = sref;
    } else {
        t_q = a.qs.t[q];
        cnt = a.qs.cnt[q];
        sref = a.qs.self_ref[q];
        if (lane < K) {
            my_ref = a.qs.ref[(size_t)q * K + lane];
            my_eid = a.qs.eid[(size_t)q * K + lane];
            my_ts = a.qs.ts[(size_t)q * K + lane];
        }
    }
    cnt = cnt < 0 ? 0 : (cnt > K ? K : cnt);
    // the filled slots of the step are packed into the per-slot matrices (most rows of a step are
    // negatives without history), in the order the workgroups happen to arrive: one addition to the
    // step's counter per workgroup (one per query queued thousands of them on the one address)
    if (lane == 0)
        wg_cnt[wave_id()] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int i = 0; i < kGatherWaves; ++i)
            total += wg_cnt[i];
        wg_base = total > 0 ? atomicAdd(t.n_live, total) : 0;
    }
    __syncthreads();
    if (!live_row)
        return;
    int sb = wg_base;
    for (int i = 0; i < wave_id(); ++i)
        sb += wg_cnt[i];
    if (cnt > 0 && (sb < 0 || sb + cnt > 3 * a.count * K))
        cnt = 0;  // (not reachable while the counter is cleared every step)
    if (lane == 0) {
        t.HAS[x] = cnt > 0 ? 1 : 0;
        t.slot0[x] = cnt > 0 ? sb : -1;
    }
    const float *self = state_row(a, M, sref);
    for (int j = lane; j < da; j += kWave) {
        const float v = j < M ? (self ? self[j] : 0.0f) : time_enc(pw.time_w_rev[j - M], pw.time_b_rev[j - M], 0.0);
        t.QIN[(size_t)x * da + j] = v;
        if (j < M)
            t.X1[(size_t)x * (da + M) + da + j] = v;
    }
    // kGC slots at a time, every piece of their rows requested before the first store: a lane's memory
    // operations complete in order (a load behind a store waits for the store's round trip), and a load
    // inside a branch is waited for at the end of the branch, so every load here is unconditional (from
    // an address that is valid in any case, the value dropped) and the slots' references are scalars.
    constexpr int kGC = 5, kGP = 2;  // slots x 64-column pieces of a row per batch
    for (int k0 = 0; k0 < cnt; k0 += kGC) {
        const float *row[kGC];   // (scalar registers: k is the same in every lane)
        const float *feat[kGC];
        double dt[kGC];
#pragma unroll
        for (int u = 0; u < kGC; ++u) {
            const int k = k0 + u < cnt ? k0 + u : cnt - 1;
            row[u] = state_row(a, M, __builtin_amdgcn_readlane(my_ref, k));
            const int32_t eid = __builtin_amdgcn_readlane(my_eid, k);
            feat[u] = eid >= 0 ? a.edge_feat + (size_t)eid * F : nullptr;
            dt[u] = t_q - readlane_f64(my_ts, k);
        }
        for (int i0 = 0; i0 < dkv; i0 += kGP * kWave) {
            float v[kGC][kGP];
            double tw[kGP], tb[kGP];
#pragma unroll
            for (int c = 0; c < kGP; ++c) {
                const int i = i0 + c * kWave + lane;
                const bool is_state = i < M, is_feat = i >= M && i < M + F, is_time = i >= M + F && i < dkv;
                const int jt = is_time ? i - M - F : 0;
                tw[c] = pw.time_w_rev[jt];
                tb[c] = pw.time_b_rev[jt];
#pragma unroll
                for (int u = 0; u < kGC; ++u) {
                    const float *src = is_state ? row[u] : (is_feat ? feat[u] : nullptr);
                    const int off = is_state ? i : i - M;
                    const float got = (src ? src : a.mem)[src ? off : 0];
                    v[u][c] = src ? got : 0.0f;
                }
            }
#pragma unroll
            for (int c = 0; c < kGP; ++c) {
                const int i = i0 + c * kWave + lane;
                const bool is_time = i >= M + F && i < dkv;
#pragma unroll
                for (int u = 0; u < kGC; ++u)
                    if (k0 + u < cnt && i < dkv)
                        t.KV[((size_t)sb + k0 + u) * dkv + i] = is_time ? time_enc(tw[c], tb[c], dt[u]) : v[u][c];
            }
        }
    }
}

// The attention core runs in a re-associated form that is the same function in exact arithmetic: with
// q~_h = W_K,h^T Qv_h the score of slot k under head h is <q~_h, kv_k> / sqrt(d_h) plus a constant
// over the slots (the key bias), which the softmax cancels; and the head's output is
// W_V,h (sum_k p_hk kv_k) + b_V,h because the p_hk sum to one.  Every matrix product of the attention
// is then a product over QUERIES (q~, the output, and in the backward pass their transposes) instead
// of over the three times as many filled neighbour slots; what is left per slot are dot products
// and weighted sums of the raw key / value rows, done here by one wavefront per query: the lanes lie
// along the row (coalesced loads), CH slots' rows are requested together, and a dot product is
// one wave reduction.
constexpr int kMaxTrainHeads = 4;
// CC: 64-column pieces of a row that a lane holds; CH: slots per register chunk.  Instantiated for rows
// of up to 256 columns with ten slots in flight and for rows of up to 512 columns with four.
constexpr int kAttnMaxCC = 8;

// kvr[u][c] = column c * 64 + lane of the raw row of slot k0 + u (the last filled slot again beyond cnt)
template <int CC, int CH>
__device__ inline void load_kv_chunk(float (&kvr)[CH][CC], const float *KV, size_t sb, int k0, int cnt, int dkv, int lane)
{
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        const int k = k0 + u < cnt ? k0 + u : cnt - 1;
#pragma unroll
        for (int c = 0; c < CC; ++c) {
            const int i = c * kWave + lane;
            kvr[u][c] = c * kWave < dkv && i < dkv ? KV[(sb + k) * dkv + i] : 0.0f;  // (the first test is uniform)
        }
    }
}

// v[h][c] = column c * 64 + lane of head h's row of a per-query [H x dkv] array
template <int HT, int CC>
__device__ inline void load_head_rows(float (&v)[HT][CC], const float *rows, int H, int dkv, int lane)
{
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int c = 0; c < CC; ++c) {
            const int i = c * kWave + lane;
            v[h][c] = h < H && c * kWave < dkv && i < dkv ? rows[(size_t)h * dkv + i] : 0.0f;
        }
}

// lane h * K + k: <head h's row of v, raw row of slot k> for k < cnt (other lanes: `other`)
template <int HT, int CC, int CH>
__device__ inline float slot_dots(const float (&v)[HT][CC], const float *KV, size_t sb, int cnt, int H, int K, int dkv,
                                  int lane, float other)
{
    float res = other;
    for (int k0 = 0; k0 < cnt; k0 += CH) {
        float kvr[CH][CC];
        load_kv_chunk<CC, CH>(kvr, KV, sb, k0, cnt, dkv, lane);
#pragma unroll
        for (int u = 0; u < CH; ++u)
#pragma unroll
            for (int h = 0; h < HT; ++h)
                if (h < H && k0 + u < cnt) {  // (uniform)
                    float part = 0.0f;
#pragma unroll
                    for (int c = 0; c < CC; ++c)
                        part += v[h][c] * kvr[u][c];
                    const float sum = wave_sum_uniform(part);
                    if (lane == h * K + k0 + u)
                        res = sum;
                }
    }
    return res;
}

// Scores, softmax, and the weighted sums KVB[x][h] = sum_k p_hk kv_k of one query per wavefront, from
// QT = q~ and the raw rows KV of its filled slots: lane h * K + k holds slot k of head h.
template <int HT, int CC, int CH>
__global__ void __launch_bounds__(kTrThreads) k_tr_attn_fwd(StepArgs a, TrainDims d, TrainBufs t)
{
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + a.count;
    const int x = (int)blockIdx.x * kRowWaves + wave_id();
    if (x >= n_rows)
        return;
    const int lane = lane_id();
    const int K = d.K, H = d.H, dh = d.dh, dkv = d.dkv;
    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    int cnt = a.qs.cnt[q];
    cnt = cnt < 0 ? 0 : (cnt > K ? K : cnt);
    const size_t sb = slot_rows(a, t, x, K, cnt);
    float *kvb = t.KVB + (size_t)x * H * dkv;
    if (cnt == 0) {
        for (int j = lane; j < H * dkv; j += kWave)
            kvb[j] = 0.0f;
        if (lane < H * K)
            t.PROB[(size_t)x * H * K + lane] = 0.0f;
        return;
    }
    const float scale = 1.0f / sqrtf((float)dh);
    float sc;
    {
        float qtr[HT][CC];
        load_head_rows<HT, CC>(qtr, t.QT + (size_t)x * H * dkv, H, dkv, lane);
        sc = slot_dots<HT, CC, CH>(qtr, t.KV, sb, cnt, H, K, dkv, lane, -INFINITY) * scale;
    }
    // softmax over the filled slots of the lane's head (every lane walks the head of lane % (H * K))
    const int hl = (lane % (H * K)) / K;
    float mx = -INFINITY;
    for (int k = 0; k < cnt; ++k)
        mx = fmaxf(mx, __shfl(sc, hl * K + k));
    const bool mine = lane < H * K && lane - hl * K < cnt;
    const float ex = mine ? expf(sc - mx) : 0.0f;
    float sum = 0.0f;
    for (int k = 0; k < cnt; ++k)
        sum += __shfl(ex, hl * K + k);
    const float pr = mine ? ex / sum : 0.0f;
    if (lane < H * K)
        t.PROB[(size_t)x * H * K + lane] = pr;
    float acc[HT][CC];
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int c = 0; c < CC; ++c)
            acc[h][c] = 0.0f;
    for (int k0 = 0; k0 < cnt; k0 += CH) {
        float kvr[CH][CC];
        load_kv_chunk<CC, CH>(kvr, t.KV, sb, k0, cnt, dkv, lane);
#pragma unroll
        for (int u = 0; u < CH; ++u)
#pragma unroll
            for (int h = 0; h < HT; ++h)
                if (h < H && k0 + u < cnt) {  // (uniform: the shuffles are executed by every lane)
                    const float p = __shfl(pr, h * K + k0 + u);
#pragma unroll
                    for (int c = 0; c < CC; ++c)
                        acc[h][c] += p * kvr[u][c];
                }
    }
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int c = 0; c < CC; ++c)
            if (h < H && c * kWave + lane < dkv)
                kvb[(size_t)h * dkv + c * kWave + lane] = acc[h][c];
}

// ------------------------------------------------------------------------------------------
__device__ inline int row_of_entry_tr(const QuerySet &qs, int i, int entries)
{
    int s = qs.slot[i];
    if (s < 0) {
        const int rep = -s - 1;
        s = rep < entries ? qs.slot[rep] : 0;
    }
    return s >= 0 && s < entries ? s : 0;
}

// The decoder runs as contractions over all (pair, event) rows (pair 0 = (source, destination), pair
// 1 = (source, negative); row p * count + b) with three small kernels around them.
// k_tr_pairs, one wavefront per event: the three embedding rows of the event go out, and the two
// input rows [emb_source | emb_destination], [emb_source | emb_negative] of the decoder are laid out.
__global__ void __launch_bounds__(kTrThreads) k_tr_pairs(StepArgs a, TrainDims d, TrainBufs t)
{
    const int E = d.E, B = a.count;
    const int b = (int)blockIdx.x * kRowWaves + wave_id();
    if (b >= B)
        return;
    const int lane = lane_id();
    const int r0 = row_of_entry_tr(a.qs, 2 * b, 2 * B), r1 = row_of_entry_tr(a.qs, 2 * b + 1, 2 * B), r2 = 2 * B + b;
    for (int j = lane; j < E; j += kWave) {
        const float es = a.emb_u[(size_t)r0 * E + j], ed = a.emb_u[(size_t)r1 * E + j], en = a.emb_u[(size_t)r2 * E + j];
        a.emb[(size_t)b * E + j] = es;
        a.emb[((size_t)B + b) * E + j] = ed;
        a.emb[((size_t)2 * B + b) * E + j] = en;
        t.CAT[(size_t)b * 2 * E + j] = es;
        t.CAT[(size_t)b * 2 * E + E + j] = ed;
        t.CAT[((size_t)B + b) * 2 * E + j] = es;
        t.CAT[((size_t)B + b) * 2 * E + E + j] = en;
    }
}

// k_tr_logit, one wavefront per (pair, event) row, after G_ = relu(W_d1 cat + b_d1): the logit, its
// loss term and the gradient of the hidden layer's pre-activation.
__global__ void __launch_bounds__(kTrThreads) k_tr_logit(StepArgs a, TrainDims d, TrainBufs t)
{
    const int E = d.E, B = a.count;
    const int pr = (int)blockIdx.x * kRowWaves + wave_id();
    if (pr >= 2 * B)
        return;
    const int lane = lane_id();
    const int p = pr >= B ? 1 : 0, b = pr - p * B;
    float part = 0.0f;
    for (int j = lane; j < E; j += kWave)
        part += t.w_d2[j] * t.G_[(size_t)pr * E + j];
    const float logit = wave_sum_uniform(part) + t.b_d2[0];
    // d softplus(sign * logit) / d logit = sign * sigmoid(sign * logit), averaged over the batch
    const float sign = p == 0 ? -1.0f : 1.0f;
    const float z = sign * logit;
    const float dlogit = sign / (1.0f + expf(-z)) / (float)B;
    if (lane == 0) {
        (p == 0 ? a.score_pos : a.score_neg)[b] = logit;
        t.DLOGIT[pr] = dlogit;
        t.LOSS[pr] = (z > 0.0f ? z + log1pf(expf(-z)) : log1pf(expf(z))) / (float)B;
    }
    for (int j = lane; j < E; j += kWave)
        t.DY[(size_t)pr * E + j] = t.G_[(size_t)pr * E + j] > 0.0f ? dlogit * t.w_d2[j] : 0.0f;
}

// k_tr_pair_scatter, one wavefront per event, after DCAT = DY W_d1: the gradients of the event's two
// decoder input rows are added to the gradients of the three distinct embedding rows they were
// copied from (rows of sources and destinations are shared by many events: atomics).
__global__ void __launch_bounds__(kTrThreads) k_tr_pair_scatter(StepArgs a, TrainDims d, TrainBufs t)
{
    const int E = d.E, B = a.count;
    const int b = (int)blockIdx.x * kRowWaves + wave_id();
    if (b >= B)
        return;
    const int lane = lane_id();
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * B ? n_u : 2 * B;
    const int xs = compact_row(row_of_entry_tr(a.qs, 2 * b, 2 * B), n_u, B);
    const int xd = compact_row(row_of_entry_tr(a.qs, 2 * b + 1, 2 * B), n_u, B);
    const int xn = compact_row(2 * B + b, n_u, B);
    const float *g0 = t.DCAT + (size_t)b * 2 * E, *g1 = t.DCAT + ((size_t)B + b) * 2 * E;
    for (int j = lane; j < E; j += kWave) {
        atomicAdd(&t.D_EMB[(size_t)xs * E + j], g0[j] + g1[j]);
        atomicAdd(&t.D_EMB[(size_t)xd * E + j], g0[E + j]);
        atomicAdd(&t.D_EMB[(size_t)xn * E + j], g1[E + j]);
    }
}

// ------------------------------------------------------------------------------------------
// Backward of scores / softmax / weighted sums of one query per wavefront: from the gradient of the
// weighted sums (DKVB) to the gradient of q~ (DQT) and to the gradients of the raw key / value rows of
// its filled slots (DKV), which are complete with it.
template <int HT, int CC, int CH>
__global__ void __launch_bounds__(kTrThreads) k_tr_attn_bwd(StepArgs a, TrainDims d, TrainBufs t)
{
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + a.count;
    const int x = (int)blockIdx.x * kRowWaves + wave_id();
    if (x >= n_rows)
        return;
    const int lane = lane_id();
    const int K = d.K, H = d.H, dh = d.dh, dkv = d.dkv;
    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    int cnt = a.qs.cnt[q];
    cnt = cnt < 0 ? 0 : (cnt > K ? K : cnt);
    const size_t sb = slot_rows(a, t, x, K, cnt);
    float *dqt = t.DQT + (size_t)x * H * dkv;
    if (cnt == 0) {
        for (int j = lane; j < H * dkv; j += kWave)
            dqt[j] = 0.0f;
        return;
    }
    const float scale = 1.0f / sqrtf((float)dh);
    float g_kvb[HT][CC];
    load_head_rows<HT, CC>(g_kvb, t.DKVB + (size_t)x * H * dkv, H, dkv, lane);
    // lane h * K + k: d p_hk = <kv_k, d KVB_h>
    const float dp = slot_dots<HT, CC, CH>(g_kvb, t.KV, sb, cnt, H, K, dkv, lane, 0.0f);
    const float pr = lane < H * K ? t.PROB[(size_t)x * H * K + lane] : 0.0f;  // (zero beyond the filled slots)
    const int hl = (lane % (H * K)) / K;
    float dot = 0.0f;
    for (int k = 0; k < cnt; ++k)
        dot += __shfl(pr, hl * K + k) * __shfl(dp, hl * K + k);
    const float dsv = pr * (dp - dot) * scale;  // gradient of <q~_h, kv_k>
    float g_qt[HT][CC], acc[HT][CC];
    load_head_rows<HT, CC>(g_qt, t.QT + (size_t)x * H * dkv, H, dkv, lane);
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int c = 0; c < CC; ++c)
            acc[h][c] = 0.0f;
    for (int k0 = 0; k0 < cnt; k0 += CH) {
        float kvr[CH][CC];
        load_kv_chunk<CC, CH>(kvr, t.KV, sb, k0, cnt, dkv, lane);
#pragma unroll
        for (int u = 0; u < CH; ++u)
            if (k0 + u < cnt) {  // (uniform: the shuffles are executed by every lane)
                float dk[CC];  // d kv_k = sum_h p_hk d KVB_h + d s_hk q~_h
#pragma unroll
                for (int c = 0; c < CC; ++c)
                    dk[c] = 0.0f;
#pragma unroll
                for (int h = 0; h < HT; ++h)
                    if (h < H) {
                        const float ds = __shfl(dsv, h * K + k0 + u), p = __shfl(pr, h * K + k0 + u);
#pragma unroll
                        for (int c = 0; c < CC; ++c) {
                            acc[h][c] += ds * kvr[u][c];
                            dk[c] += p * g_kvb[h][c] + ds * g_qt[h][c];
                        }
                    }
#pragma unroll
                for (int c = 0; c < CC; ++c)
                    if (c * kWave + lane < dkv)
                        t.DKV[(sb + k0 + u) * dkv + c * kWave + lane] = dk[c];
            }
    }
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int c = 0; c < CC; ++c)
            if (h < H && c * kWave + lane < dkv)
                dqt[(size_t)h * dkv + c * kWave + lane] = acc[h][c];
}

// What is left of a query's backward pass after the matrix products, one wavefront per query: the
// gradients w.r.t. state rows that this step's GRU wrote (own row: from the merge layer and the
// query projection; neighbour rows: from the key / value rows) are added to those staged rows'
// gradients; the time-encoding partial sums [gw | gb] of the row are written out.
// A hub node's staged row is a neighbour of most queries of a batch: its thousands of row additions
// would queue up on the same addresses.  A workgroup therefore collects the additions of its
// kScatterRows queries (one per wavefront) in an LDS table of kScatterSlots rows (open addressing by staged row with a
// few probes: a hub's row that lost its place to another row would send all its additions to memory; a row that
// finds no place goes to memory directly) and adds every table row to memory once.
constexpr int kScatterRows = 16, kScatterSlots = 64, kScatterProbes = 8, kTrScatterThreads = 1024;

__global__ void __launch_bounds__(kTrScatterThreads) k_tr_scatter(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int M = d.M, T = d.T, F = d.F, K = d.K, da = d.da, dkv = d.dkv;
    int *tag = (int *)smem;                        // [slots] staged row held by the slot, -1: none
    float *acc = (float *)(tag + kScatterSlots);   // [slots x M]
    for (int i = threadIdx.x; i < kScatterSlots; i += kTrScatterThreads)
        tag[i] = -1;
    for (int i = threadIdx.x; i < kScatterSlots * M; i += kTrScatterThreads)
        acc[i] = 0.0f;
    __syncthreads();
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + a.count;
    const int lane = lane_id();
    const int x_end = ((int)blockIdx.x + 1) * kScatterRows < n_rows ? ((int)blockIdx.x + 1) * kScatterRows : n_rows;
    for (int x = (int)blockIdx.x * kScatterRows + wave_id(); x < x_end; x += kTrScatterThreads / kWave) {
        const int q = x < n_u ? x : 2 * a.count + (x - n_u);
        int cnt = a.qs.cnt[q];
        cnt = cnt < 0 ? 0 : (cnt > K ? K : cnt);
        const size_t sb = (size_t)__builtin_amdgcn_readfirstlane((int)slot_rows(a, t, x, K, cnt));
        cnt = __builtin_amdgcn_readfirstlane(cnt);  // (both are the same in every lane: scalars from here on)
        const double t_q = a.qs.t[q];
        // lane k < cnt: neighbour slot k, lane cnt: the query's own row.  Each claims the table row of
        // its staged row (or finds it claimed by another staged row: then the additions go to memory).
        int my_srow = -1, my_lds = -1;  // staged row; its row of the table, or -1: additions go to memory
        double my_dt = 0.0;
        if (lane <= cnt) {
            const int32_t rf = lane < cnt ? a.qs.ref[(size_t)q * K + lane] : a.qs.self_ref[q];
            if (lane < cnt)
                my_dt = t_q - a.qs.ts[(size_t)q * K + lane];
            if (rf < 0 && rf != kRefNone && ~rf < 2 * a.msg_count) {
                my_srow = ~rf;
                int h = my_srow & (kScatterSlots - 1);
                for (int probe = 0; probe < kScatterProbes && my_lds < 0; ++probe) {
                    const int old = atomicCAS(&tag[h], -1, my_srow);
                    if (old == -1 || old == my_srow)
                        my_lds = h;
                    h = (h + 1) & (kScatterSlots - 1);
                }
            }
        }
        // A lane's memory operations complete in order and a conditional load makes the compiler wait
        // right behind it: the row's loads are unconditional (clamped indices), requested in batches
        // ahead of their use, and what follows them in the common case are LDS additions, which the
        // memory counter does not see.
        constexpr int kSB = 10, kMP = 2;  // neighbour slots x 64-column pieces of a state row per batch
        constexpr int kTP = 2, kTC = 10;  // 64-dim pieces of the time encoding x slots per batch of its gradient values
        if (cnt > 0) {  // (uniform)
            for (int k0 = 0; k0 < cnt; k0 += kSB)
                for (int m0 = 0; m0 < M; m0 += kMP * kWave) {
                    float v[kSB][kMP];
#pragma unroll
                    for (int u = 0; u < kSB; ++u) {
                        const int k = k0 + u < cnt ? k0 + u : cnt - 1;
#pragma unroll
                        for (int c = 0; c < kMP; ++c) {
                            const int i = m0 + c * kWave + lane;
                            v[u][c] = t.DKV[(sb + k) * dkv + (i < M ? i : 0)];
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kSB; ++u)
                        if (k0 + u < cnt) {  // (uniform)
                            const int row = __builtin_amdgcn_readlane(my_lds, k0 + u);
                            if (row >= 0) {
#pragma unroll
                                for (int c = 0; c < kMP; ++c) {
                                    const int i = m0 + c * kWave + lane;
                                    if (i < M)
                                        atomicAdd(&acc[(size_t)row * M + i], v[u][c]);
                                }
                            }
                        }
                }
        }
        {   // the query's own row
            const int srow = __builtin_amdgcn_readlane(my_srow, cnt), row = __builtin_amdgcn_readlane(my_lds, cnt);
            if (srow >= 0)
                for (int i = lane; i < M; i += kWave) {
                    const float v = t.DSU[(size_t)x * M + i] + (cnt > 0 ? t.DQIN[(size_t)x * da + i] : 0.0f);
                    if (row >= 0)
                        atomicAdd(&acc[(size_t)row * M + i], v);
                    else
                        atomicAdd(&t.D_STAG[(size_t)srow * M + i], v);
                }
        }
        // neighbour rows that found no place in the table (rare): straight to memory
        for (unsigned long long left = __ballot(lane < cnt && my_srow >= 0 && my_lds < 0); left != 0ull; left &= left - 1ull) {
            const int k = __ffsll((long long)left) - 1;
            const int srow = __builtin_amdgcn_readlane(my_srow, k);
            for (int i = lane; i < M; i += kWave)
                atomicAdd(&t.D_STAG[(size_t)srow * M + i], t.DKV[(sb + k) * dkv + i]);
        }
        for (int j0 = 0; j0 < T; j0 += kTP * kWave) {
            float gw[kTP], gb[kTP], gq[kTP];
            double w_rev[kTP], b_rev[kTP];
#pragma unroll
            for (int p = 0; p < kTP; ++p) {
                const int j = j0 + p * kWave + lane < T ? j0 + p * kWave + lane : 0;
                gq[p] = cnt > 0 ? t.DQIN[(size_t)x * da + M + j] : 0.0f;
                w_rev[p] = pw.time_w_rev[j];
                b_rev[p] = pw.time_b_rev[j];
            }
#pragma unroll
            for (int p = 0; p < kTP; ++p) {
                gw[p] = 0.0f;
                // Phi(0)_j = cos(b_j): only the phase takes a gradient from the query row
                gb[p] = cnt > 0 ? -time_enc_sin(w_rev[p], b_rev[p], 0.0) * gq[p] : 0.0f;
            }
            for (int k0 = 0; k0 < cnt; k0 += kTC) {
                float g[kTP][kTC];
#pragma unroll
                for (int u = 0; u < kTC; ++u) {
                    const int k = k0 + u < cnt ? k0 + u : cnt - 1;
#pragma unroll
                    for (int p = 0; p < kTP; ++p) {
                        const int j = j0 + p * kWave + lane < T ? j0 + p * kWave + lane : 0;
                        g[p][u] = t.DKV[(sb + k) * dkv + M + F + j];
                    }
                }
#pragma unroll
                for (int u = 0; u < kTC; ++u)
                    if (k0 + u < cnt) {  // (uniform: the shuffle is executed by every lane)
                        const double dt = shfl_f64(my_dt, k0 + u);
#pragma unroll
                        for (int p = 0; p < kTP; ++p) {
                            const float sn = time_enc_sin(w_rev[p], b_rev[p], dt);
                            gw[p] += -sn * (float)dt * g[p][u];
                            gb[p] += -sn * g[p][u];
                        }
                    }
            }
#pragma unroll
            for (int p = 0; p < kTP; ++p) {
                const int j = j0 + p * kWave + lane;
                if (j < T) {
                    t.TG[(size_t)x * 2 * T + j] = gw[p];
                    t.TG[(size_t)x * 2 * T + T + j] = gb[p];
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kScatterSlots * M; i += kTrScatterThreads) {
        const int srow = tag[i / M];
        if (srow >= 0 && srow < 2 * a.msg_count)
            atomicAdd(&t.D_STAG[(size_t)srow * M + (i % M)], acc[i]);
    }
}

// ------------------------------------------------------------------------------------------
// The GRU's backward pass over the applied winners' rows: the message rows as the step found the
// memory and the gradients of the gate pre-activations (k_tr_gru_gates, one wavefront per winner; the
// gates themselves were left by the step's GRU launch); after DPHI = DGI W_i[:, 2M : 2M + T] the time
// encoding's gradient (k_tr_gru_time).
__device__ inline bool win_ok(const StepArgs &a, const WinDesc &w)
{
    return w.node >= 0 && (int64_t)w.node < a.num_nodes && w.other >= 0 && (int64_t)w.other < a.num_nodes &&
           w.entry >= 0 && w.entry < 2 * a.msg_count && w.b >= 0 && w.b < a.msg_count;
}

__global__ void __launch_bounds__(kTrThreads) k_tr_gru_gates(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t)
{
    int n_win = *a.n_win;
    n_win = n_win < 2 * a.msg_count ? n_win : 2 * a.msg_count;
    const int M = d.M, T = d.T, F = d.F, D = d.Dmsg;
    const int lane = lane_id();
    for (int r = (int)blockIdx.x * kRowWaves + wave_id(); r < n_win; r += (int)gridDim.x * kRowWaves) {
        const WinDesc w = a.win[r];
        const bool ok = win_ok(a, w);
        // the winner's message row from the memory as the step found it (the weight gradients' input rows)
        const double dt = ok ? w.t - a.lu[w.node] : 0.0;
        for (int j = lane; j < D; j += kWave) {
            float v = 0.0f;
            if (ok) {
                if (j < M)
                    v = a.mem[(size_t)w.node * M + j];
                else if (j < 2 * M)
                    v = a.mem[(size_t)w.other * M + (j - M)];
                else if (j < 2 * M + T)
                    v = time_enc(pw.time_w_rev[j - 2 * M], pw.time_b_rev[j - 2 * M], dt);
                else
                    v = a.edge_feat[(size_t)(a.msg_first_eid + w.b) * F + (j - 2 * M - T)];
            }
            t.MSG[(size_t)r * D + j] = v;
        }
        // gradients of the gate pre-activations
        const float *gt = t.GATES + (size_t)r * 4 * M;  // r, z, n, W_hn h + b_hn as the step's GRU launch left them
        float *dgi = t.DGI + (size_t)r * 3 * M, *dgh = t.DGH + (size_t)r * 3 * M;
        for (int j = lane; j < M; j += kWave) {
            const float rg = gt[j], zg = gt[M + j], ng = gt[2 * M + j], ghn = gt[3 * M + j];
            const float dh = ok ? t.D_STAG[(size_t)w.entry * M + j] : 0.0f;
            const float h = ok ? a.mem[(size_t)w.node * M + j] : 0.0f;  // s_self = the first M entries of the message
            const float dn = dh * (1.0f - zg);
            const float dz = dh * (h - ng);
            const float dpre_n = dn * (1.0f - ng * ng);
            const float dpre_r = dpre_n * ghn * rg * (1.0f - rg);
            const float dpre_z = dz * zg * (1.0f - zg);
            dgi[j] = dpre_r;
            dgi[M + j] = dpre_z;
            dgi[2 * M + j] = dpre_n;
            dgh[j] = dpre_r;
            dgh[M + j] = dpre_z;
            dgh[2 * M + j] = dpre_n * rg;
        }
    }
}

// gw[j] += sum_r -sin(phase_rj) dt_r DPHI[r][j], gb[j] += sum_r -sin(phase_rj) DPHI[r][j] over the applied
// winners: a thread per column and slice of the winners.  g_time: [gw | gb], 2T floats.
__global__ void __launch_bounds__(kTrThreads) k_tr_gru_time(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t, float *g_time)
{
    int n_win = *a.n_win;
    n_win = n_win < 2 * a.msg_count ? n_win : 2 * a.msg_count;
    const int T = d.T;
    const int j = (int)blockIdx.x * kTrThreads + (int)threadIdx.x;
    if (j >= T)
        return;
    const int per = (n_win + (int)gridDim.y - 1) / (int)gridDim.y;
    const int lo = (int)blockIdx.y * per, hi = lo + per < n_win ? lo + per : n_win;
    if (lo >= hi)
        return;
    const double w_rev = pw.time_w_rev[j], b_rev = pw.time_b_rev[j];
    float gw = 0.0f, gb = 0.0f;
    for (int r = lo; r < hi; ++r) {
        const WinDesc w = a.win[r];
        const double dt = win_ok(a, w) ? w.t - a.lu[w.node] : 0.0;
        const float v = -time_enc_sin(w_rev, b_rev, dt) * t.DPHI[(size_t)r * T + j];
        gw += (float)dt * v;
        gb += v;
    }
    atomicAdd(&g_time[j], gw);
    atomicAdd(&g_time[T + j], gb);
}

// ------------------------------------------------------------------------------------------
// C[Mo x No] += A[rows x Mo]^T B[rows x No].  A workgroup of eight wavefronts takes one 32 x 32 block
// of C and one slice of the rows; the wavefronts split the slice, add their blocks up in LDS, and
// the workgroup adds the result to C with one atomic per element (the atomics, not the products, bound
// these contractions: few of them).
// csum != NULL: also csum[Mo] += the column sums of A (the bias gradient that goes with the weight
// gradient: A^T times a column of ones), by the workgroups of the first block column.
constexpr int kTnWaves = 8;
// blockIdx.y = z names one product of a batch (one per attention head): C + z * zC, A + z * zA,
// B + z * zB, csum + z * zS (element offsets).
struct TnBatch {
    int zC, zA, zB, zS;
};
__global__ void __launch_bounds__(kTnWaves *kWave) k_gemm_tn(float *C, int ldc, const float *A, int lda, const float *B, int ldb,
                                                              int Mo, int No, RowCount rc, int n_slices, float *csum, TnBatch zb)
{
    C += (size_t)blockIdx.y * zb.zC;
    A += (size_t)blockIdx.y * zb.zA;
    B += (size_t)blockIdx.y * zb.zB;
    if (csum)
        csum += (size_t)blockIdx.y * zb.zS;
    __shared__ float red[kTnWaves][1024];
    __shared__ float reds[kTnWaves][32];
    const int w = threadIdx.x / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int tiles_n = (No + 31) / 32, tiles_m = (Mo + 31) / 32;
    const int slice = (int)blockIdx.x % n_slices;
    const int tile = (int)blockIdx.x / n_slices;
    if (tile >= tiles_m * tiles_n)
        return;
    const int m0 = (tile / tiles_n) * 32, n0 = (tile % tiles_n) * 32;
    const int rows = row_count(rc);
    const int per = (rows + n_slices - 1) / n_slices;
    const int s_lo = slice * per, s_hi = s_lo + per < rows ? s_lo + per : rows;
    if (s_lo >= s_hi)
        return;  // (uniform over the workgroup)
    const int sub = ((s_hi - s_lo + kTnWaves - 1) / kTnWaves + 3) / 4 * 4;
    const int k_lo = s_lo + w * sub, k_hi = k_lo + sub < s_hi ? k_lo + sub : s_hi;
    const bool with_sum = csum != nullptr && n0 == 0;  // (uniform over the workgroup)
    floatx4 acc[2][2], accs[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        accs[i] = floatx4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[i][j] = floatx4{0, 0, 0, 0};
    }
    const int c = lane & 15, g = lane >> 4;
    constexpr int kU = 4;  // k-steps whose loads are issued together
    for (int k = k_lo; k < k_hi; k += 4 * kU) {
        float av[kU][2], bv[kU][2];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kk = k + 4 * u + g;
            const bool kin = kk < k_hi;
            const int row = kk;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int mm = m0 + 16 * i + c, nn = n0 + 16 * i + c;
                av[u][i] = kin && mm < Mo ? A[(size_t)row * lda + mm] : 0.0f;
                bv[u][i] = kin && nn < No ? B[(size_t)row * ldb + nn] : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][i], bv[u][j], acc[i][j], 0, 0, 0);
                if (with_sum)
                    accs[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][i], 1.0f, accs[i], 0, 0, 0);
            }
        }
    }
    // element ((i * 2 + j) * 4 + v) * 64 + lane of a wavefront's block is C[m0 + 16 i + 4 g + v][n0 + 16 j + c]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                red[w][((i * 2 + j) * 4 + v) * kWave + lane] = acc[i][j][v];
    if (c == 0) {  // every column of the sum block holds the same value: column 0 keeps it
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                reds[w][16 * i + 4 * g + v] = accs[i][v];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 1024; e += kTnWaves * kWave) {
        float sum = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kTnWaves; ++ww)
            sum += red[ww][e];
        const int l = e & (kWave - 1), v = (e / kWave) & 3, j = (e / (4 * kWave)) & 1, i = e / (8 * kWave);
        const int mm = m0 + 16 * i + 4 * (l >> 4) + v, nn = n0 + 16 * j + (l & 15);
        if (mm < Mo && nn < No)
            atomicAdd(&C[(size_t)mm * ldc + nn], sum);
    }
    if (with_sum && threadIdx.x < 32) {
        float sum = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kTnWaves; ++ww)
            sum += reds[ww][threadIdx.x];
        if (m0 + (int)threadIdx.x < Mo)
            atomicAdd(&csum[m0 + threadIdx.x], sum);
    }
}

// out[j] += sum over the rows of A[row][j]
__global__ void __launch_bounds__(256) k_colsum(float *out, const float *A, int lda, int cols, RowCount rc, int n_slices)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int slice = blockIdx.y;
    if (j >= cols)
        return;
    const int rows = row_count(rc);
    const int per = (rows + n_slices - 1) / n_slices;
    const int lo = slice * per, hi = lo + per < rows ? lo + per : rows;
    float acc = 0.0f;
#pragma unroll 8
    for (int r = lo; r < hi; ++r)
        acc += A[(size_t)r * lda + j];
    if (lo < hi)
        atomicAdd(&out[j], acc);
}

// The transposed copies of all weight matrices in one launch: blockIdx.y names the matrix.
struct TransposeJobs {
    float *dst[9];
    const float *src[9];
    int rows[9], cols[9];
};
__global__ void k_transpose(TransposeJobs J)  // dst[c][r] = src[r][c]
{
    const int m = blockIdx.y;
    const int rows = J.rows[m], cols = J.cols[m];
    const float *src = J.src[m];
    float *dst = J.dst[m];
    const size_t n = (size_t)rows * cols, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const size_t r = i / cols, c = i - r * cols;
        dst[c * rows + r] = src[i];
    }
}

// The memory overwrite (the GRU's backward read the memory as the step found it), the sum of the loss
// terms (one workgroup, if terms != NULL) and the SGD update (the workgroups beyond, if lr != 0), which
// share nothing; the step's query set is empty again afterwards (its counter is cleared for the set's
// next preparation).
__global__ void __launch_bounds__(256) k_tr_update(StepArgs a, int M, int commit_blocks, const float *terms, int n_terms,
                                                   float *loss_out, float *P, const float *G, size_t n_params, float lr)
{
    if (blockIdx.x == 0 && threadIdx.x == 0)
        *a.qs.n_u = 0;
    if ((int)blockIdx.x < commit_blocks) {
        overwrite_memory(a, M, (int)(blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave),
                         (int)(commit_blocks * (blockDim.x / kWave)));
        return;
    }
    const int loss_blocks = loss_out ? 1 : 0;
    if ((int)blockIdx.x >= commit_blocks + loss_blocks) {
        const size_t i = (size_t)((int)blockIdx.x - commit_blocks - loss_blocks) * blockDim.x + threadIdx.x;
        if (lr != 0.0f && i < n_params)
            P[i] -= lr * G[i];
        return;
    }
    __shared__ float red[256];
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int i = threadIdx.x; i < n_terms; i += 4 * 256)
#pragma unroll
        for (int u = 0; u < 4; ++u)
            acc[u] += i + u * 256 < n_terms ? terms[i + u * 256] : 0.0f;
    red[threadIdx.x] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st)
            red[threadIdx.x] += red[threadIdx.x + st];
        __syncthreads();
    }
    if (threadIdx.x == 0)
        *loss_out = red[0];
}

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

}  // namespace

// ---- host side ---------------------------------------------------------------------------------

struct TrainLayout {
    float *P, *G;       // master weights and their gradients, the fields of tig_weights in order
    size_t n_params;
    tig_weights w, g;   // pointers into P and G
    float *T_i, *T_h, *T_Q, *T_K, *T_V, *T_O, *T_m1, *T_m2, *T_d1;
    TrainBufs b;
    void *pack_scratch;
    size_t zero_lo, zero_hi;  // byte range (from the base) that every step clears: G, D_EMB, D_STAG
    size_t bytes;
};

static TrainDims train_dims(const Dims &d)
{
    return TrainDims{d.M, d.T, d.F, d.E, d.K, d.H, d.da, d.dh, d.dkv, d.Dmsg};
}

static TrainLayout train_layout(const Dims &d, void *base)
{
    TrainLayout L;
    memset(&L, 0, sizeof(L));
    char *p = (char *)base;
    size_t off = 0;
    auto take = [&](size_t n_floats) -> float * {
        float *q = base ? (float *)(p + off) : nullptr;
        off += align_up(4 * (n_floats ? n_floats : 1));
        return q;
    };
    const size_t M = d.M, T = d.T, E = d.E, K = d.K, H = d.H, da = d.da, dkv = d.dkv, D = d.Dmsg;
    const size_t B = d.max_batch, R = 3 * B, S = R * K, U = 2 * B;
    const size_t counts[22] = {T, T, 3 * M * D, 3 * M, 3 * M * M, 3 * M, da * da, da, da * dkv, da, da * dkv, da,
                               da * da, da, E * (da + M), E, E * E, E, E * 2 * E, E, E, 1};
    size_t n = 0;
    for (size_t c : counts)
        n += c;
    L.n_params = n;
    L.P = take(n);
    // cleared every step: gradients, gradient of the embeddings, gradient of the staged rows
    L.zero_lo = off;
    L.G = take(n);
    L.b.D_EMB = take(R * E);
    L.b.D_STAG = take(U * M);
    L.b.n_live = (int32_t *)take(64);
    L.zero_hi = off;
    const float **wf[22] = {&L.w.time_w, &L.w.time_b, &L.w.W_i, &L.w.b_i, &L.w.W_h, &L.w.b_h, &L.w.W_Q, &L.w.b_Q,
                            &L.w.W_K, &L.w.b_K, &L.w.W_V, &L.w.b_V, &L.w.W_O, &L.w.b_O, &L.w.W_m1, &L.w.b_m1,
                            &L.w.W_m2, &L.w.b_m2, &L.w.W_d1, &L.w.b_d1, &L.w.w_d2, &L.w.b_d2};
    const float **gf[22] = {&L.g.time_w, &L.g.time_b, &L.g.W_i, &L.g.b_i, &L.g.W_h, &L.g.b_h, &L.g.W_Q, &L.g.b_Q,
                            &L.g.W_K, &L.g.b_K, &L.g.W_V, &L.g.b_V, &L.g.W_O, &L.g.b_O, &L.g.W_m1, &L.g.b_m1,
                            &L.g.W_m2, &L.g.b_m2, &L.g.W_d1, &L.g.b_d1, &L.g.w_d2, &L.g.b_d2};
    size_t o = 0;
    for (int i = 0; i < 22; ++i) {
        *wf[i] = L.P ? L.P + o : nullptr;
        *gf[i] = L.G ? L.G + o : nullptr;
        o += counts[i];
    }
    L.w.struct_size = L.g.struct_size = sizeof(tig_weights);
    L.T_i = take(3 * M * D);
    L.T_h = take(3 * M * M);
    L.T_Q = take(da * da);
    L.T_K = take(da * dkv);
    L.T_V = take(da * dkv);
    L.T_O = take(da * da);
    L.T_m1 = take(E * (da + M));
    L.T_m2 = take(E * E);
    L.T_d1 = take(E * 2 * E);
    TrainBufs &b = L.b;
    b.QIN = take(R * da);
    b.QV = take(R * da);
    b.O_ = take(R * da);
    b.PROB = take(R * H * K);
    b.X1 = take(R * (da + M));
    b.H1 = take(R * E);
    b.DZ1 = take(R * E);
    b.D_ATTN = take(R * da);
    b.DQV = take(R * da);
    b.TG = take(R * 2 * T);
    b.DOUT = take(R * da);
    b.DSU = take(R * M);
    b.DQIN = take(R * da);
    b.HAS = (int32_t *)take(R);
    b.KV = take(S * dkv);
    b.QT = take(R * H * dkv);
    b.KVB = take(R * H * dkv);
    b.DKVB = take(R * H * dkv);
    b.DQT = take(R * H * dkv);
    b.DKV = take(S * dkv);
    b.CAT = take(U * 2 * E);
    b.DY = take(U * E);
    b.G_ = take(U * E);
    b.DCAT = take(U * 2 * E);
    b.DLOGIT = take(U);
    b.LOSS = take(U);
    b.MSG = take(U * D);
    b.DGI = take(U * 3 * M);
    b.DGH = take(U * 3 * M);
    b.GATES = take(U * 4 * M);
    b.DPHI = take(U * T);
    b.n_rows = (int32_t *)take(64);
    b.slot0 = (int32_t *)take(R);
    L.pack_scratch = base ? p + off : nullptr;
    off += align_up(pack_scratch_bytes(d));
    L.bytes = off;
    b.W_i = L.w.W_i; b.b_i = L.w.b_i; b.W_h = L.w.W_h; b.b_h = L.w.b_h; b.W_Q = L.w.W_Q; b.b_Q = L.w.b_Q;
    b.W_K = L.w.W_K; b.b_K = L.w.b_K; b.W_V = L.w.W_V; b.b_V = L.w.b_V; b.W_O = L.w.W_O; b.b_O = L.w.b_O;
    b.W_m1 = L.w.W_m1; b.b_m1 = L.w.b_m1; b.W_m2 = L.w.W_m2; b.b_m2 = L.w.b_m2; b.W_d1 = L.w.W_d1; b.b_d1 = L.w.b_d1;
    b.w_d2 = L.w.w_d2; b.b_d2 = L.w.b_d2;
    b.T_i = L.T_i; b.T_h = L.T_h; b.T_Q = L.T_Q; b.T_K = L.T_K; b.T_V = L.T_V; b.T_O = L.T_O; b.T_m1 = L.T_m1;
    b.T_m2 = L.T_m2; b.T_d1 = L.T_d1;
    return L;
}

static int scatter_lds(const Dims &d) { return 4 * kScatterSlots * (d.M + 1); }

size_t train_workspace_bytes(const Dims &d) { return train_layout(d, nullptr).bytes; }

hipError_t prepare_train(const Dims &d)
{
    return hipFuncSetAttribute((const void *)k_tr_scatter, hipFuncAttributeMaxDynamicSharedMemorySize, scatter_lds(d));
}

bool train_supported(const Dims &d)
{
    // (the attention kernels keep slot k of head h in lane h * K + k of a query's wavefront)
    return d.prec == TIG_FP32 && scatter_lds(d) <= 64 * 1024 && d.H * d.K <= kWave && d.K < kWave && d.H <= kMaxTrainHeads && d.dkv <= kAttnMaxCC * kWave;
}

static hipError_t transpose_all(const Dims &d, const TrainLayout &L, hipStream_t s)
{
    struct Job {
        float *dst;
        const float *src;
        int rows, cols;
    };
    const Job jobs[] = {{L.T_i, L.w.W_i, 3 * d.M, d.Dmsg}, {L.T_h, L.w.W_h, 3 * d.M, d.M}, {L.T_Q, L.w.W_Q, d.da, d.da},
                        {L.T_K, L.w.W_K, d.da, d.dkv},     {L.T_V, L.w.W_V, d.da, d.dkv},  {L.T_O, L.w.W_O, d.da, d.da},
                        {L.T_m1, L.w.W_m1, d.E, d.da + d.M}, {L.T_m2, L.w.W_m2, d.E, d.E},  {L.T_d1, L.w.W_d1, d.E, 2 * d.E}};
    TransposeJobs J;
    size_t most = 0;
    for (int i = 0; i < 9; ++i) {
        J.dst[i] = jobs[i].dst;
        J.src[i] = jobs[i].src;
        J.rows[i] = jobs[i].rows;
        J.cols[i] = jobs[i].cols;
        const size_t n = (size_t)jobs[i].rows * jobs[i].cols;
        most = n > most ? n : most;
    }
    hipLaunchKernelGGL(k_transpose, dim3((unsigned)((most + 1023) / 1024), 9), dim3(256), 0, s, J);
    return hipGetLastError();
}

// Copies the caller's weights into the master buffer, builds the transposes, re-folds the packed weights.
hipError_t train_attach(const Dims &d, const tig_weights &w, void *workspace, void *packed, PackedWeights *pw,
                        hipStream_t s)
{
    const TrainLayout L = train_layout(d, workspace);
    const float *const src[22] = {w.time_w, w.time_b, w.W_i, w.b_i, w.W_h, w.b_h, w.W_Q, w.b_Q, w.W_K, w.b_K, w.W_V,
                                  w.b_V, w.W_O, w.b_O, w.W_m1, w.b_m1, w.W_m2, w.b_m2, w.W_d1, w.b_d1, w.w_d2, w.b_d2};
    const float *const dst[22] = {L.w.time_w, L.w.time_b, L.w.W_i, L.w.b_i, L.w.W_h, L.w.b_h, L.w.W_Q, L.w.b_Q,
                                  L.w.W_K, L.w.b_K, L.w.W_V, L.w.b_V, L.w.W_O, L.w.b_O, L.w.W_m1, L.w.b_m1,
                                  L.w.W_m2, L.w.b_m2, L.w.W_d1, L.w.b_d1, L.w.w_d2, L.w.b_d2};
    for (int i = 0; i < 22; ++i) {
        const size_t n = (i + 1 < 22 ? dst[i + 1] : L.P + L.n_params) - dst[i];
        hipError_t e = hipMemcpyAsync((void *)dst[i], src[i], 4 * n, hipMemcpyDefault, s);
        if (e != hipSuccess)
            return e;
    }
    hipError_t e = transpose_all(d, L, s);
    if (e == hipSuccess)
        e = pack_weights(d, L.w, packed, L.pack_scratch, pw, s);
    return e;
}

hipError_t train_copy_out(const Dims &d, void *workspace, bool grads, const tig_weights &out, hipStream_t s)
{
    const TrainLayout L = train_layout(d, workspace);
    const tig_weights &src = grads ? L.g : L.w;
    const float *const sp[22] = {src.time_w, src.time_b, src.W_i, src.b_i, src.W_h, src.b_h, src.W_Q, src.b_Q,
                                 src.W_K, src.b_K, src.W_V, src.b_V, src.W_O, src.b_O, src.W_m1, src.b_m1,
                                 src.W_m2, src.b_m2, src.W_d1, src.b_d1, src.w_d2, src.b_d2};
    const float *const dp[22] = {out.time_w, out.time_b, out.W_i, out.b_i, out.W_h, out.b_h, out.W_Q, out.b_Q,
                                 out.W_K, out.b_K, out.W_V, out.b_V, out.W_O, out.b_O, out.W_m1, out.b_m1,
                                 out.W_m2, out.b_m2, out.W_d1, out.b_d1, out.w_d2, out.b_d2};
    const float *end = (grads ? L.G : L.P) + L.n_params;
    for (int i = 0; i < 22; ++i) {
        if (!dp[i])
            continue;
        const size_t n = (i + 1 < 22 ? sp[i + 1] : end) - sp[i];
        const hipError_t e = hipMemcpyAsync((void *)dp[i], sp[i], 4 * n, hipMemcpyDefault, s);
        if (e != hipSuccess)
            return e;
    }
    return hipStreamSynchronize(s);
}

// Everything of a training step after the GRU launch: forward in direct form, loss, backward, SGD,
// re-folding of the packed weights, memory overwrite.
hipError_t launch_train(const Dims &d, const StepArgs &a, void *workspace, void *packed, PackedWeights *pw, float lr,
                        float *loss_out, hipStream_t s, const TrainSide *side)
{
    const TrainLayout L = train_layout(d, workspace);
    const TrainDims td = train_dims(d);
    const TrainBufs &b = L.b;
    const PackedWeights pwv = *pw;
    hipError_t e = launch_fill_zero((char *)workspace + L.zero_lo, L.zero_hi - L.zero_lo, s);
    if (e != hipSuccess)
        return e;
    const int B = a.count, R = 3 * B, K = d.K;
    const int M = d.M, T = d.T, E = d.E, H = d.H, da = d.da, dh = d.dh, dkv = d.dkv, D = d.Dmsg;
    const RowCount rows{b.n_rows, 0, 1, R}, live{b.n_live, 0, 1, R * K}, pairs{nullptr, 0, 1, 2 * B},
        wins{a.n_win, 0, 1, 2 * a.msg_count};
    // one layer product over all rows (or over the filled slots: `slots`)
    auto vec_ok = [](const float *p, int ld) { return (((uintptr_t)p & 15) == 0 && ld % 4 == 0) ? 1 : 0; };
    auto layer = [&](float *C, int ldc, const float *A, int lda, const float *W, int ldw, const float *bias, int N, int Kd,
                     bool slots = false) {
        RowGemm g = {};
        g.A = A, g.lda = lda, g.W = W, g.ldw = ldw, g.bias = bias, g.C = C, g.ldc = ldc, g.N = N, g.Kd = Kd;
        g.rc = slots ? live : rows;
        g.vecA = vec_ok(A, lda), g.vecW = vec_ok(W, ldw);
        return g;
    };
    auto run = [&](const RowGemm &g, int nz = 1) { launch_rowgemm(g, nz, s); };
    const dim3 per_row((R + kRowWaves - 1) / kRowWaves);
    // The weight gradients, C += A^T B together with the bias gradient csum += column sums of A, run on
    // the side stream as soon as their rows are complete (fork(i): the rows of group i are), beside the
    // rest of the backward pass, which leaves most compute units idle.
    const hipStream_t ws = side ? side->stream : s;
    hipError_t fe = hipSuccess;
    auto fork = [&](int i) {
        if (!side || fe != hipSuccess)
            return;
        fe = hipEventRecord(side->fork[i], s);
        if (fe == hipSuccess)
            fe = hipStreamWaitEvent(side->stream, side->fork[i], 0);
    };
    auto gemm = [&](const float *C, const float *csum, int Mo, int No, const float *A, const float *Bm, const RowCount &rc,
                    int ldb = 0, int lda = 0, int nz = 1, TnBatch zb = TnBatch{0, 0, 0, 0}) {
        const int tiles = ((Mo + 31) / 32) * ((No + 31) / 32);
        // about 512 workgroups of eight wavefronts per contraction; a wavefront keeps at least 32 rows
        int n_slices = 512 / (tiles * nz);
        const int most = rc.rows_max / (32 * kTnWaves);
        n_slices = n_slices > most ? most : n_slices;
        n_slices = n_slices < 1 ? 1 : n_slices;
        hipLaunchKernelGGL(k_gemm_tn, dim3(tiles * n_slices, nz), dim3(kTnWaves * kWave), 0, ws, (float *)C, No, A,
                           lda ? lda : Mo, Bm, ldb ? ldb : No, Mo, No, rc, n_slices, (float *)csum, zb);
    };
    auto colsum = [&](const float *out, const float *A, int lda, int cols, const RowCount &rc) {
        int n_slices = rc.rows_max / 64;
        n_slices = n_slices < 1 ? 1 : (n_slices > 256 ? 256 : n_slices);
        hipLaunchKernelGGL(k_colsum, dim3((cols + 255) / 256, n_slices), dim3(256), 0, ws, (float *)out, A, lda, cols, rc,
                           n_slices);
    };
    // ---- forward, direct form
    hipLaunchKernelGGL(k_tr_gather, dim3((R + kGatherWaves - 1) / kGatherWaves), dim3(kGatherWaves * kWave), 0, s, a, pwv, td, b);
    run(layer(b.QV, da, b.QIN, da, b.W_Q, da, b.b_Q, da, da));
    {   // q~_h = W_K,h^T Qv_h, every head in one launch
        RowGemm g = layer(b.QT, H * dkv, b.QV, da, b.T_K, da, nullptr, dkv, dh);
        g.zA = dh, g.zW = dh, g.zC = dkv;
        g.vecA = g.vecA && dh % 4 == 0, g.vecW = g.vecW && dh % 4 == 0;
        run(g, H);
    }
    const bool narrow = dkv <= 4 * kWave;
    if (H <= 2 && narrow)
        hipLaunchKernelGGL((k_tr_attn_fwd<2, 4, 10>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    else if (H <= 2)
        hipLaunchKernelGGL((k_tr_attn_fwd<2, kAttnMaxCC, 4>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    else if (narrow)
        hipLaunchKernelGGL((k_tr_attn_fwd<kMaxTrainHeads, 4, 6>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    else
        hipLaunchKernelGGL((k_tr_attn_fwd<kMaxTrainHeads, kAttnMaxCC, 4>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    {   // o_h = W_V,h KVB_h + b_V,h
        RowGemm g = layer(b.O_, da, b.KVB, H * dkv, b.W_V, dkv, b.b_V, dh, dkv);
        g.zA = dkv, g.zW = dh * dkv, g.zC = dh, g.zBias = dh;
        g.vecA = g.vecA && dkv % 4 == 0, g.vecW = g.vecW && (dh * dkv) % 4 == 0;
        run(g, H);
    }
    {   // attn = W_O o + b_O into the head of the merge layer's input; the zero vector without neighbours
        RowGemm g = layer(b.X1, da + M, b.O_, da, b.W_O, da, b.b_O, da, da);
        g.rowmask = b.HAS;
        run(g);
    }
    {
        RowGemm g = layer(b.H1, E, b.X1, da + M, b.W_m1, da + M, b.b_m1, E, da + M);
        g.relu = 1;
        run(g);
    }
    {   // emb = W_m2 h1 + b_m2 straight to the rows of the query set
        RowGemm g = layer(a.emb_u, E, b.H1, E, b.W_m2, E, b.b_m2, E, E);
        g.remap_nu = a.qs.n_u, g.remap_2b = 2 * B;
        run(g);
    }
    {   // decoder: input rows, hidden layer, logits and loss terms; then back to the embedding rows
        const dim3 per_event((B + kRowWaves - 1) / kRowWaves), per_pair((2 * B + kRowWaves - 1) / kRowWaves);
        hipLaunchKernelGGL(k_tr_pairs, per_event, dim3(kTrThreads), 0, s, a, td, b);
        RowGemm g = layer(b.G_, E, b.CAT, 2 * E, b.W_d1, 2 * E, b.b_d1, E, 2 * E);
        g.rc = pairs, g.relu = 1;
        run(g);
        hipLaunchKernelGGL(k_tr_logit, per_pair, dim3(kTrThreads), 0, s, a, td, b);
        fork(0);
        gemm(L.g.W_d1, L.g.b_d1, E, 2 * E, b.DY, b.CAT, pairs);
        gemm(L.g.w_d2, L.g.b_d2, 1, E, b.DLOGIT, b.G_, pairs);
        g = layer(b.DCAT, 2 * E, b.DY, E, b.T_d1, E, nullptr, 2 * E, E);
        g.rc = pairs;
        run(g);
        hipLaunchKernelGGL(k_tr_pair_scatter, per_event, dim3(kTrThreads), 0, s, a, td, b);
    }
    // ---- backward: dX = dY W through the transposed copies
    {   // dz1 = (W_m2^T d_emb) where z1 > 0
        RowGemm g = layer(b.DZ1, E, b.D_EMB, E, b.T_m2, E, nullptr, E, E);
        g.gate = b.H1, g.ldg = E;
        run(g);
        fork(1);  // merge MLP
        gemm(L.g.W_m2, L.g.b_m2, E, E, b.D_EMB, b.H1, rows);
        gemm(L.g.W_m1, L.g.b_m1, E, da + M, b.DZ1, b.X1, rows);
    }
    {   // [d_attn | d s_u] = W_m1^T dz1; without neighbours attn is the constant 0
        RowGemm g = layer(b.D_ATTN, da, b.DZ1, E, b.T_m1, E, nullptr, da + M, E);
        g.rowmask = b.HAS;
        g.n_split = da, g.W_hi = b.T_m1 + (size_t)da * E, g.bias_hi = nullptr, g.C_hi = b.DSU, g.ldc_hi = M;
        g.vecW = g.vecW && vec_ok(g.W_hi, E);
        run(g);
    }
    run(layer(b.DOUT, da, b.D_ATTN, da, b.T_O, da, nullptr, da, da));
    {   // d KVB_h = W_V,h^T d o_h
        RowGemm g = layer(b.DKVB, H * dkv, b.DOUT, da, b.T_V, da, nullptr, dkv, dh);
        g.zA = dh, g.zW = dh, g.zC = dkv;
        g.vecA = g.vecA && dh % 4 == 0, g.vecW = g.vecW && dh % 4 == 0;
        run(g, H);
    }
    if (H <= 2 && narrow)
        hipLaunchKernelGGL((k_tr_attn_bwd<2, 4, 10>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    else if (H <= 2)
        hipLaunchKernelGGL((k_tr_attn_bwd<2, kAttnMaxCC, 4>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    else if (narrow)
        hipLaunchKernelGGL((k_tr_attn_bwd<kMaxTrainHeads, 4, 6>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    else
        hipLaunchKernelGGL((k_tr_attn_bwd<kMaxTrainHeads, kAttnMaxCC, 4>), per_row, dim3(kTrThreads), 0, s, a, td, b);
    fork(2);  // attention: dW_V,h = d o_h^T KVB_h, dW_K,h = Qv_h^T d q~_h over the queries (the key bias takes no gradient)
    gemm(L.g.W_O, L.g.b_O, da, da, b.D_ATTN, b.O_, rows);
    gemm(L.g.W_V, L.g.b_V, dh, dkv, b.DOUT, b.KVB, rows, H * dkv, da, H, TnBatch{dh * dkv, dh, dkv, dh});
    gemm(L.g.W_K, nullptr, dh, dkv, b.QV, b.DQT, rows, H * dkv, da, H, TnBatch{dh * dkv, dh, dkv, 0});
    {   // d Qv_h = W_K,h d q~_h
        RowGemm g = layer(b.DQV, da, b.DQT, H * dkv, b.W_K, dkv, nullptr, dh, dkv);
        g.zA = dkv, g.zW = dh * dkv, g.zC = dh;
        g.vecA = g.vecA && dkv % 4 == 0, g.vecW = g.vecW && (dh * dkv) % 4 == 0;
        run(g, H);
    }
    fork(5);
    gemm(L.g.W_Q, L.g.b_Q, da, da, b.DQV, b.QIN, rows);
    run(layer(b.DQIN, da, b.DQV, da, b.T_Q, da, nullptr, da, da));
    hipLaunchKernelGGL(k_tr_scatter, dim3((R + kScatterRows - 1) / kScatterRows), dim3(kTrScatterThreads), scatter_lds(d), s, a,
                       pwv, td, b);
    fork(3);  // time encoding: per-row partial sums [gw | gb]; the two gradients are neighbours in the gradient buffer
    colsum(L.g.time_w, b.TG, 2 * T, 2 * T, rows);
    if (a.msg_count > 0) {
        // GRU backward over the applied winners (their number is known on the device only)
        const int wg = (2 * a.msg_count + kRowWaves - 1) / kRowWaves;
        const dim3 per_win(wg < 256 ? wg : 256);
        hipLaunchKernelGGL(k_tr_gru_gates, per_win, dim3(kTrThreads), 0, s, a, pwv, td, b);
        fork(4);  // state update
        gemm(L.g.W_i, L.g.b_i, 3 * M, D, b.DGI, b.MSG, wins);
        gemm(L.g.W_h, L.g.b_h, 3 * M, M, b.DGH, b.MSG, wins, D);  // h = the first M columns of the message rows
        RowGemm g = layer(b.DPHI, T, b.DGI, 3 * M, b.T_i + (size_t)2 * M * 3 * M, 3 * M, nullptr, T, 3 * M);
        g.rc = wins;
        run(g);
        hipLaunchKernelGGL(k_tr_gru_time, dim3((T + kTrThreads - 1) / kTrThreads, 128), dim3(kTrThreads), 0, s, a, pwv, td, b,
                           (float *)L.g.time_w);
    }
    if ((e = hipGetLastError()) != hipSuccess || (e = fe) != hipSuccess)
        return e;
    if (side) {  // the step's stream goes on when the last weight gradient is complete
        if ((e = hipEventRecord(side->join, side->stream)) != hipSuccess || (e = hipStreamWaitEvent(s, side->join, 0)) != hipSuccess)
            return e;
    }
    // the memory overwrite comes last: the GRU's backward read the memory as the step found it
    {
        const int commit_blocks = a.msg_count > 0 ? 32 : 0;
        const int sgd_blocks = lr != 0.0f ? (int)((L.n_params + 255) / 256) : 0;
        int blocks = commit_blocks + (loss_out ? 1 : 0) + sgd_blocks;
        blocks = blocks > 0 ? blocks : 1;  // (block 0 clears the query set's counter whatever else there is to do)
        hipLaunchKernelGGL(k_tr_update, dim3(blocks), dim3(256), 0, s, a, M, commit_blocks, b.LOSS, 2 * B, loss_out, L.P,
                           L.G, L.n_params, lr);
    }
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    if (lr != 0.0f) {
        if ((e = transpose_all(d, L, s)) != hipSuccess)
            return e;
        // the step's own forward pass reads the masters and their transposes; of the prepared weights
        // only the state update's (and the time encoding's) are read by a training step, so only they
        // follow every update; the rest is re-folded when an inference step next needs it
        e = pack_weights(d, L.w, packed, L.pack_scratch, pw, s, kPackGru);
    }
    return e;
}

float *train_gates_buffer(const Dims &d, void *workspace) { return train_layout(d, workspace).b.GATES; }

hipError_t train_refold_embed(const Dims &d, void *workspace, void *packed, PackedWeights *pw, hipStream_t s)
{
    const TrainLayout L = train_layout(d, workspace);
    return pack_weights(d, L.w, packed, L.pack_scratch, pw, s, kPackEmbed);
}

}  // namespace tig
