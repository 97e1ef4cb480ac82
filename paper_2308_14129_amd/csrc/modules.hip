// Other instances of the general architecture (paper Sec. II-C "Training approach for TIGs": the
// messages of a node within a batch "can be aggregated by ... mean message", the state update "can
// be chosen from ... GRU, RNN", the embedding function f is "identity, time projection or
// attention"; Sec. II-A: nodes may carry static features), device side.  gfx950 only, fp32.
//
// A context with an attached module selection runs its batch step here instead of in the fused
// kernels of the headline instance (last message, GRU, attention), in plain per-row kernels:
//   k_mod_update   one workgroup per node of the applied batch: aggregated message (the last one, or
//                  the mean of all the node's messages of the batch, every one built from the memory
//                  at the start of the step), then the GRU or the plain recurrent cell -> staged row
//   k_mod_commit   memory overwrite M <- s_i(t) and last_update, after every message has been built
//   k_mod_simple   identity / time-projection embedding of every query, straight to the output
//   k_mr_items / k_mr_attn + k_rowgemm   attention embedding with node features and / or two stacked
//                  layers: every layer product as one contraction over all items of the layer, the
//                  attention core per item in its re-associated form (stated above k_mr_items); a
//                  negative's neighbours are looked up by k_mr_items
//   k_mod_hop2     two stacked attention layers (the embedding module's sum over the 2-hop temporal
//                  neighbourhood): the K most recent events, before the QUERY's time, of every
//                  neighbour of every distinct query; the first layer then runs over each used
//                  (query, neighbour) pair and each query itself, the second layer over those rows
//   k_mod_decode   eight events per workgroup: both logits (and, for the attention embedding, the
//                  per-query embedding rows out of the distinct rows)
// Weight matrices are read through transposed copies ([in x out]) so that a thread that owns an
// output reads consecutive addresses.
#include <hip/hip_runtime.h>

#include "kernels_common.h"
#include "prepare.h"
#include "rowgemm.h"
#include "winners.h"

namespace tig {

namespace {

constexpr int kModThreads = 256;
constexpr int kModWaves = kModThreads / kWave;
constexpr int kEV = 8;   // events per decoder workgroup

struct ModDims {
    int M, T, F, E, K, H, da, dh, dkv, Dmsg;
    int G;  // gate blocks of the state update: 3 (GRU: r, z, n) or 1 (plain recurrent cell)
    int agg, upd, emb;
};

// The dimensions the second layer sees: its input rows are E wide.
ModDims second_layer_dims(ModDims d)
{
    d.M = d.E;
    d.da = d.E + d.T;
    d.dkv = d.E + d.F + d.T;
    d.dh = d.da / d.H;
    return d;
}

ModDims mod_dims(const Dims &d, const ModParams &p)
{
    return ModDims{d.M, d.T, d.F, d.E, d.K, d.H, d.da, d.dh, d.dkv, d.Dmsg, p.upd == TIG_UPD_GRU ? 3 : 1, p.agg, p.upd, p.emb};
}

// y[j] = bias[j] + sum_i WT[i * out + j] * x[i]   (x, y in LDS)
__device__ inline void matvec_t(const float *WT, int in, int out, const float *x, const float *bias, float *y)
{
    for (int j = threadIdx.x; j < out; j += kModThreads) {
        float acc = bias ? bias[j] : 0.0f;
#pragma unroll 16
        for (int i = 0; i < in; ++i)  // (unrolled: sixteen independent loads in flight, not one per step)
            acc += WT[(size_t)i * out + j] * x[i];
        y[j] = acc;
    }
}

// r_i(t): the state row the embedding module reads for node v (memory row plus the static feature
// row), element j; a node id outside the graph reads as a zero row
__device__ inline float repr_elem(const StepArgs &a, const ModParams &p, int M, int32_t v, int j)
{
    if (v < 0 || (int64_t)v >= a.num_nodes)
        return 0.0f;
    float x = a.mem[(size_t)v * M + j];
    if (p.node_feat)
        x += p.node_feat[(size_t)v * M + j];
    return x;
}

// ------------------------------------------------------------------------------------------
// Mean aggregator, first half: one wavefront per (event, role) entry of the applied batch adds the
// columns of its message that differ between a node's messages -- [s'_other | Phi(dt) | e] -- to the
// accumulation row of the entry that won the node's last message (named by the node's key), in
// double.  A hub node collects thousands of messages per batch, and additions to one address queue
// up: a workgroup first collects its kMsgEntries entries' rows in an LDS table of kMsgSlots rows
// (direct-mapped by accumulation row; a row whose place is taken goes to memory directly) and adds
// every table row to memory once, dealt out over the node's kAccCopies copies.  The rows in memory
// are all zero between steps: k_mod_update clears what it has read.
constexpr int kMsgThreads = 1024, kMsgEntries = 64, kMsgSlots = 16;

__global__ void __launch_bounds__(kMsgThreads) k_mod_msgsum(StepArgs a, ModDims d, ModParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int M = d.M, T = d.T, F = d.F, rest = M + T + F;
    double *acc = (double *)smem;                    // [slots x rest]
    int *tag = (int *)(acc + kMsgSlots * rest);      // [slots] accumulation row held by the slot, -1: none
    int *cnt = tag + kMsgSlots;                      // [slots] messages collected in it
    for (int i = threadIdx.x; i < kMsgSlots * rest; i += kMsgThreads)
        acc[i] = 0.0;
    if (threadIdx.x < kMsgSlots) {
        tag[threadIdx.x] = -1;
        cnt[threadIdx.x] = 0;
    }
    __syncthreads();
    const int lane = lane_id();
    const int i_end = ((int)blockIdx.x + 1) * kMsgEntries < 2 * a.msg_count ? ((int)blockIdx.x + 1) * kMsgEntries : 2 * a.msg_count;
    for (int i = (int)blockIdx.x * kMsgEntries + wave_id(); i < i_end; i += kMsgThreads / kWave) {
        const int64_t e = a.msg_first_eid + (i >> 1);
        const int32_t u = (i & 1) ? a.dst[e] : a.src[e];
        const int32_t o = (i & 1) ? a.src[e] : a.dst[e];
        if (u < 0 || (int64_t)u >= a.num_nodes)
            continue;
        const int32_t ref = ref_of_key(ref_ctx(a), u, a.msg_key[u]);
        if (ref >= 0 || ref == kRefNone)
            continue;  // (not reachable: every node of the applied batch has a winning entry in it)
        const int row = ~ref;
        const bool ok = o >= 0 && (int64_t)o < a.num_nodes;
        const double dt = a.ts[e] - a.lu[u];
        const int slot = row & (kMsgSlots - 1);
        int old = 0;
        if (lane == 0)
            old = atomicCAS(&tag[slot], -1, row);
        old = __shfl(old, 0);
        const bool in_lds = old == -1 || old == row;
        double *dst = in_lds ? acc + (size_t)slot * rest
                             : p.acc + ((size_t)row * kAccCopies + ((i >> 1) & (kAccCopies - 1))) * rest;
        for (int j = lane; j < rest; j += kWave) {
            float v;
            if (j < M)
                v = ok ? a.mem[(size_t)o * M + j] : 0.0f;
            else if (j < M + T)
                v = time_enc(p.time_w_rev[j - M], p.time_b_rev[j - M], dt);
            else
                v = a.edge_feat[(size_t)e * F + (j - M - T)];
            if (in_lds)
                atomicAdd(&dst[j], (double)v);
            else
                unsafeAtomicAdd(&dst[j], (double)v);
        }
        if (lane == 0) {
            if (in_lds)
                atomicAdd(&cnt[slot], 1);
            else
                atomicAdd(&p.acc_cnt[row], 1);
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kMsgSlots * rest; idx += kMsgThreads) {
        const int slot = idx / rest, j = idx - slot * rest;
        const int row = tag[slot];
        if (row < 0 || row >= 2 * a.msg_count)
            continue;
        unsafeAtomicAdd(&p.acc[((size_t)row * kAccCopies + ((int)blockIdx.x & (kAccCopies - 1))) * rest + j], acc[idx]);
        if (j == 0)
            atomicAdd(&p.acc_cnt[row], cnt[slot]);
    }
}

// Aggregated message + state update of one node of the applied batch (the batch's winner list names
// each node once, with its last event).
__global__ void __launch_bounds__(kModThreads) k_mod_update(StepArgs a, ModDims d, ModParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int M = d.M, T = d.T, F = d.F, D = d.Dmsg, GM = d.G * d.M;
    const int rest = M + T + F;                 // message columns that differ between a node's messages
    float *msg = (float *)smem;                 // [D]
    float *h = msg + D;                         // [M]
    float *gi = h + M;                          // [GM]
    float *gh = gi + GM;                        // [GM]

    int n_win = *a.n_win;
    n_win = n_win < 2 * a.msg_count ? n_win : 2 * a.msg_count;
    const int r = (int)blockIdx.x;
    if (r >= n_win)
        return;
    const WinDesc w = a.win[r];
    if (w.node < 0 || (int64_t)w.node >= a.num_nodes || w.other < 0 || (int64_t)w.other >= a.num_nodes ||
        w.entry < 0 || w.entry >= 2 * a.msg_count)
        return;  // (not a descriptor of this batch)
    for (int j = threadIdx.x; j < M; j += kModThreads) {
        const float v = a.mem[(size_t)w.node * M + j];
        h[j] = v;
        msg[j] = v;
    }
    if (d.agg == TIG_AGG_LAST) {
        const double lu0 = a.lu[w.node];
        const int64_t eid = a.msg_first_eid + (w.entry >> 1);
        for (int j = threadIdx.x; j < rest; j += kModThreads) {
            float v;
            if (j < M)
                v = a.mem[(size_t)w.other * M + j];
            else if (j < M + T)
                v = time_enc(p.time_w_rev[j - M], p.time_b_rev[j - M], w.t - lu0);
            else
                v = a.edge_feat[(size_t)eid * F + (j - M - T)];
            msg[M + j] = v;
        }
    } else {
        double *acc = p.acc + (size_t)w.entry * kAccCopies * rest;
        const int n = p.acc_cnt[w.entry];
        const double inv = 1.0 / (double)(n > 0 ? n : 1);
        for (int j = threadIdx.x; j < rest; j += kModThreads) {
            double sum = 0.0;
#pragma unroll
            for (int c = 0; c < kAccCopies; ++c) {  // (fixed order: the result does not depend on the adds' order beyond fp64 rounding)
                sum += acc[(size_t)c * rest + j];
                acc[(size_t)c * rest + j] = 0.0;
            }
            msg[M + j] = (float)(sum * inv);
        }
        __syncthreads();  // (every thread has read the count)
        if (threadIdx.x == 0)
            p.acc_cnt[w.entry] = 0;
    }
    __syncthreads();
    matvec_t(p.T_i, D, GM, msg, p.b_i, gi);
    matvec_t(p.T_h, M, GM, h, p.b_h, gh);
    __syncthreads();
    for (int j = threadIdx.x; j < M; j += kModThreads) {
        float out;
        if (d.upd == TIG_UPD_GRU) {
            const float rr = 1.0f / (1.0f + expf(-(gi[j] + gh[j])));
            const float zz = 1.0f / (1.0f + expf(-(gi[M + j] + gh[M + j])));
            const float nn = tanhf(gi[2 * M + j] + rr * gh[2 * M + j]);
            out = (1.0f - zz) * nn + zz * h[j];
        } else {
            out = tanhf(gi[j] + gh[j]);
        }
        a.staging[(size_t)w.entry * M + j] = out;
    }
}

__global__ void __launch_bounds__(kModThreads) k_mod_commit(StepArgs a, int M)
{
    overwrite_memory(a, M, (int)(blockIdx.x * kModWaves + threadIdx.x / kWave), (int)(gridDim.x * kModWaves));
}

// ------------------------------------------------------------------------------------------
// Identity / time-projection embedding: emb[q] = r_u(t), or (1 + (t - last_update[u]) w_p) * r_u(t),
// for the queries [sources | destinations | negatives]; also the winner flags out.
__global__ void __launch_bounds__(kModThreads) k_mod_simple(StepArgs a, ModDims d, ModParams p)
{
    const int M = d.M;
    const size_t n = (size_t)a.roles * a.count * M;
    const size_t idx = (size_t)blockIdx.x * kModThreads + threadIdx.x;
    if (idx < (size_t)2 * a.count && a.out_is_winner && a.win_flags)
        a.out_is_winner[idx] = a.win_flags[idx];
    if (idx >= n)
        return;
    const int q = (int)(idx / M), j = (int)(idx - (size_t)q * M);
    const int role = q / a.count, b = q - role * a.count;
    const int64_t e = a.first_eid + b;
    const int32_t u = role == 0 ? a.src[e] : (role == 1 ? a.dst[e] : a.neg[b]);
    float v = repr_elem(a, p, M, u, j);
    if (d.emb == TIG_EMB_TIME_PROJECTION && u >= 0 && (int64_t)u < a.num_nodes)
        v = (float)((1.0 + (a.ts[e] - a.lu[u]) * (double)p.time_proj_w[j]) * (double)v);
    a.emb[idx] = v;
}

// ------------------------------------------------------------------------------------------
// Two layers: the neighbour tables of the second hop.  One workgroup per query row (distinct source /
// destination queries, then the negatives, whose own table is looked up first): wavefront w takes the
// neighbours k = w, w + waves, ... and looks up the K most recent events of neighbour k before the
// QUERY's time into row q * K + k of the second-hop tables.
__global__ void __launch_bounds__(kModThreads) k_mod_hop2(StepArgs a, ModDims d, ModParams p)
{
    __shared__ int s_cnt;
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + (a.roles == 3 ? a.count : 0);
    const int x = (int)blockIdx.x;
    if (x >= n_rows)
        return;
    const int K = d.K;
    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    if (x >= n_u && threadIdx.x < kWave) {
        int32_t rf, ee;
        double ts_k;
        (void)finish_negative(a, K, x - n_u, rf, ee, ts_k);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const int c = a.qs.cnt[q];
        s_cnt = c < 0 ? 0 : (c > K ? K : c);
    }
    __syncthreads();
    const int cnt = s_cnt;
    const double t_q = a.qs.t[q];
    for (int k = wave_id(); k < cnt; k += kModWaves) {
        int32_t nb, ee;
        double tt;
        (void)nbr_lookup_wave(a, K, a.qs.nbr[(size_t)q * K + k], t_q, -1, p.hop2, q * K + k, nb, ee, tt);
    }
}

// ------------------------------------------------------------------------------------------
// The attention embedding as contractions over all ITEMS of a layer at once (an item is a distinct
// query or, in the first of two layers, neighbour j of a distinct query at the query's time): every
// layer product is one k_rowgemm launch over the items instead of one pass over the weight matrices
// per item (forty thousand workgroups streaming 0.7 MB each from L2 bounded the per-item kernel),
// and the attention core runs in the re-associated form that is the same function in exact
// arithmetic -- q~_h = W_K,h^T Qv_h, score <q~_h, kv_k> / sqrt(d_h) (the key bias adds a constant
// over the slots that the softmax cancels), head output W_V,h (sum_k p_hk kv_k) + b_V,h -- so that no
// product runs over neighbour slots and the raw key / value rows [row of the neighbour | e |
// Phi(t - t_k)] are never stored: the attention kernel forms them in registers.
//   k_mr_items   one wavefront per distinct query: the item list (first of two layers: the used
//                (query, slot) pairs and the queries themselves, packed in the order the workgroups
//                arrive), query rows [own row | Phi(0)] and the own row as the tail of the merge
//                layer's input
//   k_mr_attn    one wavefront per item: scores, softmax, weighted sums of the raw rows
enum MrMode { kMrSingle = 0, kMrFirst = 1, kMrSecond = 2 };
constexpr int kMrWaves = 16;
constexpr int kMrCH = 4;   // slots per register chunk
constexpr int kMrCC = 8;   // 64-column pieces of a raw row a lane can hold at most: rows of up to 512 columns
constexpr int kMrMaxHeads = 4;

// The item of (query row x, slot j) once the item list is complete: an index, or the pair's
// representative's.
__device__ inline int mr_item_of(const ModParams &p, size_t dense)
{
    int c = p.mr_ci[dense];
    if (c < 0)
        c = p.mr_ci[(size_t)(-c - 1)];
    return c < 0 ? 0 : c;
}

// First of two layers: equal (node, t) pairs -- a hub is a neighbour of most queries of a second, and
// is a query itself -- are one item.  Pair (u, t) of (x, j) index `dense` claims a slot of the table
// (open addressing; a slot changes once per step, from empty to claimed); returns the index that
// represents the pair: its own, or the first claimant's.
__device__ inline int mr_claim(const StepArgs &a, const ModParams &p, int K, int n_u, int dense, int32_t u, double t)
{
    uint32_t h = query_hash(u, t) & p.mr_tab_mask;
    for (uint32_t probes = 0; probes <= p.mr_tab_mask; ++probes) {
        uint32_t cur = __hip_atomic_load(&p.mr_tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cur == 0u) {
            const uint32_t old = atomicCAS(&p.mr_tab[h], 0u, (uint32_t)dense + 1u);
            if (old == 0u)
                return dense;
            cur = old;
        }
        const int other = (int)(cur - 1u);
        const int xo = other / (K + 1), jo = other - xo * (K + 1);
        if (xo < n_u + a.count) {
            const int qo = xo < n_u ? xo : 2 * a.count + (xo - n_u);
            const int32_t uo = jo < K ? a.qs.nbr[(size_t)qo * K + jo] : a.qs.node[qo];
            if (uo == u && a.qs.t[qo] == t)
                return other;
        }
        h = (h + 1) & p.mr_tab_mask;
    }
    return dense;
}

// One wavefront per distinct query row x; its items are the used slots j < cnt of its neighbour table
// and -- slot K -- the query itself (one layer, and the second of two: that one only).
template <int MODE>
__global__ void __launch_bounds__(kMrWaves *kWave) k_mr_items(StepArgs a, ModDims d, ModParams p)
{
    __shared__ int wg_items[kMrWaves], wg_base;
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + (a.roles == 3 ? a.count : 0);
    const int M = d.M, E = d.E, K = d.K, da = d.da;
    const int lane = lane_id();
    const int x = (int)blockIdx.x * kMrWaves + wave_id();
    const bool valid = x < n_rows;  // (uniform over the wavefront; every wavefront reaches the barriers)
    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    int cnt_x = 0;
    if (valid) {
        if (MODE == kMrSingle && x >= n_u) {  // a negative: its neighbours are looked up here
            int32_t rf, ee;
            double ts_k;
            cnt_x = finish_negative(a, K, x - n_u, rf, ee, ts_k);
        } else {
            cnt_x = a.qs.cnt[q];
        }
        cnt_x = cnt_x < 0 ? 0 : (cnt_x > K ? K : cnt_x);
    }
    const int32_t u_self = !valid ? -1 : (MODE == kMrSingle && x >= n_u ? a.neg[x - n_u] : a.qs.node[q]);
    // lane `it` of the wavefront: candidate item `it` of the row (slots first, the query itself last)
    const int n_cand = !valid ? 0 : (MODE == kMrFirst ? cnt_x + 1 : 1);
    const int my_j = MODE == kMrFirst && lane < cnt_x ? lane : K;
    int32_t my_u = u_self;
    bool is_item = lane < n_cand;
    if (MODE == kMrFirst && lane < n_cand) {
        if (my_j < K)
            my_u = a.qs.nbr[(size_t)q * K + my_j];
        const int dense = x * (K + 1) + my_j;
        const int rep = mr_claim(a, p, K, n_u, dense, my_u, a.qs.t[q]);
        is_item = rep == dense;
        if (!is_item)
            p.mr_ci[dense] = -rep - 1;
    }
    const unsigned long long items = __ballot(is_item);
    const int n_it = __popcll(items);
    int ci0 = x;
    if (MODE == kMrFirst) {  // the items are packed in the order the workgroups arrive: one addition per workgroup
        if (lane == 0)
            wg_items[wave_id()] = n_it;
        __syncthreads();
        if (threadIdx.x == 0) {
            int total = 0;
            for (int i = 0; i < kMrWaves; ++i)
                total += wg_items[i];
            wg_base = total > 0 ? atomicAdd(p.mr_n, total) : 0;
        }
        __syncthreads();
        ci0 = wg_base;
        for (int i = 0; i < wave_id(); ++i)
            ci0 += wg_items[i];
        if (ci0 < 0 || ci0 + n_it > 3 * a.count * (K + 1))
            return;  // (not reachable while the counter is cleared every step)
    }
    int rank = 0;
    for (unsigned long long left = items; left != 0ull; left &= left - 1ull, ++rank) {
        const int it = __ffsll((long long)left) - 1;  // (uniform)
        const int j = __shfl(my_j, it);
        const int32_t u = __shfl(my_u, it);
        const int ci = ci0 + rank;
        const bool hop = j < K;
        int cnt_item = cnt_x;
        if (hop) {
            const int c = p.hop2.cnt[(size_t)q * K + j];
            cnt_item = c < 0 ? 0 : (c > K ? K : c);
        }
        if (lane == 0) {
            p.mr_itq[ci] = q;
            p.mr_itj[ci] = j;
            p.mr_has[ci] = cnt_item > 0 ? 1 : 0;
            if (MODE == kMrFirst)
                p.mr_ci[(size_t)x * (K + 1) + j] = ci;
        }
        // the item's own row: the node's state row (+ features), or -- second layer -- its first-layer row
        const float *own1 = MODE == kMrSecond ? p.h1 + (size_t)mr_item_of(p, (size_t)x * (K + 1) + K) * E : nullptr;
        for (int jj = lane; jj < da; jj += kWave) {
            float v;
            if (jj >= M)
                v = time_enc(p.time_w_rev[jj - M], p.time_b_rev[jj - M], 0.0);
            else
                v = MODE == kMrSecond ? own1[jj] : repr_elem(a, p, M, u, jj);
            p.mr_qin[(size_t)ci * da + jj] = v;
            if (jj < M)
                p.mr_x1[(size_t)ci * (da + M) + da + jj] = v;
        }
    }
}

// CC: 64-column pieces of a raw row (dkv <= 64 CC)
template <int MODE, int HT, int CC>
__global__ void __launch_bounds__(kModThreads) k_mr_attn(StepArgs a, ModDims d, ModParams p)
{
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + (a.roles == 3 ? a.count : 0);
    int n_items = n_rows;
    if (MODE == kMrFirst) {
        n_items = *p.mr_n;
        const int most = 3 * a.count * (d.K + 1);
        n_items = n_items < 0 ? 0 : (n_items < most ? n_items : most);
    }
    const int ci = (int)blockIdx.x * kModWaves + wave_id();
    if (ci >= n_items)
        return;
    const int lane = lane_id();
    const int M = d.M, F = d.F, E = d.E, K = d.K, H = d.H, dh = d.dh, dkv = d.dkv;
    const int q = p.mr_itq[ci], j = p.mr_itj[ci];
    const bool hop = MODE == kMrFirst && j < K;
    const QuerySet &tab = hop ? p.hop2 : a.qs;
    const size_t trow = hop ? (size_t)q * K + j : (size_t)q;
    int cnt = tab.cnt[trow];
    cnt = cnt < 0 ? 0 : (cnt > K ? K : cnt);
    float *kvb = p.mr_kvb + (size_t)ci * H * dkv;
    if (cnt == 0) {
        for (int i = lane; i < H * dkv; i += kWave)
            kvb[i] = 0.0f;
        return;
    }
    const double t_q = a.qs.t[q];
    // lane k < cnt: slot k of the item's table
    int32_t my_nbr = -1, my_eid = -1, my_src = 0;
    double my_dt = 0.0;
    if (lane < cnt) {
        my_nbr = tab.nbr[trow * K + lane];
        my_eid = tab.eid[trow * K + lane];
        my_dt = t_q - tab.ts[trow * K + lane];
        if (MODE == kMrSecond)  // (second layer: item ci is query row x = ci; its slot's first-layer row)
            my_src = mr_item_of(p, (size_t)ci * (K + 1) + lane);
    }
    // kvr[u][c] = column c * 64 + lane of the raw row [row of the neighbour | e | Phi(t - t_k)] of slot k0 + u
    auto load_chunk = [&](float (&kvr)[kMrCH][CC], int k0) {
#pragma unroll
        for (int u = 0; u < kMrCH; ++u) {
            const int k = k0 + u < cnt ? k0 + u : cnt - 1;  // (uniform; the shuffles are executed by every lane)
            const int32_t nb = __shfl(my_nbr, k), ee = __shfl(my_eid, k), sr = __shfl(my_src, k);
            const int dlo = __shfl(__double2loint(my_dt), k), dhi = __shfl(__double2hiint(my_dt), k);
            const double dt = __hiloint2double(dhi, dlo);
#pragma unroll
            for (int c = 0; c < CC; ++c) {
                const int i = c * kWave + lane;
                float v = 0.0f;
                if (c * kWave < dkv && i < dkv) {  // (the first test is uniform)
                    if (i < M)
                        v = MODE == kMrSecond ? p.h1[(size_t)sr * E + i] : repr_elem(a, p, M, nb, i);
                    else if (i < M + F)
                        v = ee >= 0 ? a.edge_feat[(size_t)ee * F + (i - M)] : 0.0f;
                    else
                        v = time_enc(p.time_w_rev[i - M - F], p.time_b_rev[i - M - F], dt);
                }
                kvr[u][c] = v;
            }
        }
    };
    const float scale = 1.0f / sqrtf((float)dh);
    float sc = -INFINITY;  // lane h * K + k: score of slot k under head h
    {
        float qtr[HT][CC];
        const float *qt = p.mr_qt + (size_t)ci * H * dkv;
#pragma unroll
        for (int h = 0; h < HT; ++h)
#pragma unroll
            for (int c = 0; c < CC; ++c) {
                const int i = c * kWave + lane;
                qtr[h][c] = h < H && c * kWave < dkv && i < dkv ? qt[(size_t)h * dkv + i] : 0.0f;
            }
        for (int k0 = 0; k0 < cnt; k0 += kMrCH) {
            float kvr[kMrCH][CC];
            load_chunk(kvr, k0);
#pragma unroll
            for (int u = 0; u < kMrCH; ++u)
#pragma unroll
                for (int h = 0; h < HT; ++h)
                    if (h < H && k0 + u < cnt) {  // (uniform)
                        float part = 0.0f;
#pragma unroll
                        for (int c = 0; c < CC; ++c)
                            part += qtr[h][c] * kvr[u][c];
                        const float sum = wave_sum_uniform(part) * scale;
                        if (lane == h * K + k0 + u)
                            sc = sum;
                    }
        }
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
    float acc[HT][CC];
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int c = 0; c < CC; ++c)
            acc[h][c] = 0.0f;
    for (int k0 = 0; k0 < cnt; k0 += kMrCH) {
        float kvr[kMrCH][CC];
        load_chunk(kvr, k0);
#pragma unroll
        for (int u = 0; u < kMrCH; ++u)
#pragma unroll
            for (int h = 0; h < HT; ++h)
                if (h < H && k0 + u < cnt) {  // (uniform: the shuffles are executed by every lane)
                    const float pk = __shfl(pr, h * K + k0 + u);
#pragma unroll
                    for (int c = 0; c < CC; ++c)
                        acc[h][c] += pk * kvr[u][c];
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
__device__ inline int mod_row_of_entry(const QuerySet &qs, int i, int entries)
{
    int s = qs.slot[i];
    if (s < 0) {
        const int rep = -s - 1;
        s = rep < entries ? qs.slot[rep] : 0;
    }
    return s >= 0 && s < entries ? s : 0;
}

// Both logits of kEV events.  from_rows: the embeddings are the distinct rows of the query set (and
// are copied out per query here); else they are already in the output, [sources | destinations |
// negatives].
__global__ void __launch_bounds__(kModThreads) k_mod_decode(StepArgs a, ModDims d, ModParams p, int from_rows)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int E = d.E, B = a.count, roles = a.roles;
    float *em = (float *)smem;            // [kEV][3][E]
    float *part = em + kEV * 3 * E;       // [kEV][2][waves]
    const int b0 = (int)blockIdx.x * kEV;
    const int nev = B - b0 < kEV ? B - b0 : kEV;
    for (int idx = threadIdx.x; idx < nev * roles * E; idx += kModThreads) {
        const int ev = idx / (roles * E), rem = idx - ev * roles * E;
        const int r = rem / E, j = rem - r * E;
        const int b = b0 + ev;
        float v;
        if (from_rows) {
            const int row = r < 2 ? mod_row_of_entry(a.qs, 2 * b + r, 2 * B) : 2 * B + b;
            v = a.emb_u[(size_t)row * E + j];
            a.emb[((size_t)r * B + b) * E + j] = v;
        } else {
            v = a.emb[((size_t)r * B + b) * E + j];
        }
        em[(ev * 3 + r) * E + j] = v;
    }
    __syncthreads();
    float sp[kEV], sn[kEV];
#pragma unroll
    for (int ev = 0; ev < kEV; ++ev)
        sp[ev] = sn[ev] = 0.0f;
    // (no condition inside the loops: events beyond the batch repeat event 0, a step without negatives
    // reads the destination row twice; both results are dropped below)
    const int noff = roles == 3 ? 2 * E : E;
    for (int j = threadIdx.x; j < E; j += kModThreads) {
        float ya[kEV], yb[kEV], yn[kEV];
#pragma unroll
        for (int ev = 0; ev < kEV; ++ev)
            ya[ev] = yb[ev] = yn[ev] = 0.0f;
#pragma unroll 10
        for (int i = 0; i < E; ++i) {  // (unrolled: the weight loads of ten steps are in flight together)
            const float wa = p.T_d1[(size_t)i * E + j], wb = p.T_d1[(size_t)(E + i) * E + j];
#pragma unroll
            for (int ev = 0; ev < kEV; ++ev) {
                const float *row = em + (ev < nev ? ev : 0) * 3 * E;
                ya[ev] = fmaf(wa, row[i], ya[ev]);
                yb[ev] = fmaf(wb, row[E + i], yb[ev]);
                yn[ev] = fmaf(wb, row[noff + i], yn[ev]);
            }
        }
        const float b1 = p.b_d1[j], w2 = p.w_d2[j];
#pragma unroll
        for (int ev = 0; ev < kEV; ++ev) {
            sp[ev] += w2 * fmaxf(ya[ev] + yb[ev] + b1, 0.0f);
            sn[ev] += w2 * fmaxf(ya[ev] + yn[ev] + b1, 0.0f);
        }
    }
#pragma unroll
    for (int ev = 0; ev < kEV; ++ev) {
        const float s1 = wave_sum_uniform(sp[ev]), s2 = wave_sum_uniform(sn[ev]);
        if (lane_id() == 0) {
            part[(ev * 2 + 0) * kModWaves + wave_id()] = s1;
            part[(ev * 2 + 1) * kModWaves + wave_id()] = s2;
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < nev * 2) {
        const int ev = threadIdx.x >> 1, pr = threadIdx.x & 1;
        float s = p.b_d2[0];
        for (int w = 0; w < kModWaves; ++w)
            s += part[(ev * 2 + pr) * kModWaves + w];
        if (pr == 0)
            a.score_pos[b0 + ev] = s;
        else if (roles == 3)
            a.score_neg[b0 + ev] = s;
    }
}

__global__ void k_mod_transpose(float *dst, const float *src, int rows, int cols)  // dst[c][r] = src[r][c]
{
    const size_t n = (size_t)rows * cols, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const size_t r = i / cols, c = i - r * cols;
        dst[c * rows + r] = src[i];
    }
}

__global__ void k_mod_revolutions(double *out, const float *in, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        out[i] = (double)in[i] / 6.283185307179586476925286766559;
}

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int update_lds(const ModDims &d) { return (d.Dmsg + d.M + 2 * d.G * d.M) * 4; }

int msgsum_lds(const ModDims &d) { return kMsgSlots * (d.M + d.T + d.F) * 8 + 2 * kMsgSlots * 4; }

int decode_lds(const ModDims &d) { return (kEV * 3 * d.E + kEV * 2 * kModWaves) * 4; }

// One matrix of the workspace: raw copy (kept for nothing but the transpose) and its transpose.
struct MatJob {
    const float *src;     // caller's [rows x cols]
    const float **dst_t;  // where the transposed copy's pointer goes
    int rows, cols;
};

struct VecJob {
    const float *src;
    const float **dst;
    size_t n;
};

}  // namespace

// Layout of the attached workspace: [vectors | transposed matrices | raw staging of one matrix |
// node features].  Fills `p` when base != NULL.
static size_t mod_layout(const Dims &d, int agg, int upd, int emb, int layers, bool node_feat, int64_t num_nodes, char *base,
                         ModParams *p, float **raw_stage, float **nf_dst)
{
    size_t off = 0;
    auto take = [&](size_t count, size_t elem) -> void * {
        void *q = base ? base + off : nullptr;
        off += align_up(count * elem);
        return q;
    };
    const size_t M = d.M, T = d.T, E = d.E, D = d.Dmsg, G = upd == TIG_UPD_GRU ? 3 : 1;
    const bool attn = emb == TIG_EMB_ATTENTION;
    ModParams q = {};
    q.agg = agg;
    q.upd = upd;
    q.emb = emb;
    q.layers = layers == 2 ? 2 : 1;
    q.time_w_rev = (const double *)take(T, 8);
    q.time_b_rev = (const double *)take(T, 8);
    q.b_i = (const float *)take(G * M, 4);
    q.b_h = (const float *)take(G * M, 4);
    q.T_i = (const float *)take(D * G * M, 4);
    q.T_h = (const float *)take(M * G * M, 4);
    size_t biggest = D * G * M;
    if (attn) {
        for (int l = 0; l < q.layers; ++l) {
            // layer l reads rows of width in_w: the state width, then the first layer's width
            const size_t in_w = l == 0 ? M : E, a_w = in_w + T, kv_w = in_w + d.F + T;
            AttnLayer &A = q.L[l];
            A.b_Q = (const float *)take(a_w, 4);
            A.b_K = (const float *)take(a_w, 4);
            A.b_V = (const float *)take(a_w, 4);
            A.b_O = (const float *)take(a_w, 4);
            A.b_m1 = (const float *)take(E, 4);
            A.b_m2 = (const float *)take(E, 4);
            A.T_Q = (const float *)take(a_w * a_w, 4);
            A.T_K = (const float *)take(kv_w * a_w, 4);
            A.T_V = (const float *)take(kv_w * a_w, 4);
            A.T_O = (const float *)take(a_w * a_w, 4);
            A.T_m1 = (const float *)take((a_w + in_w) * E, 4);
            A.T_m2 = (const float *)take(E * E, 4);
            A.N_Q = (const float *)take(a_w * a_w, 4);
            A.N_V = (const float *)take(a_w * kv_w, 4);
            A.N_O = (const float *)take(a_w * a_w, 4);
            A.N_m1 = (const float *)take(E * (a_w + in_w), 4);
            A.N_m2 = (const float *)take(E * E, 4);
            const size_t c[] = {a_w * a_w, kv_w * a_w, (a_w + in_w) * E, E * E};
            for (size_t v : c)
                biggest = v > biggest ? v : biggest;
        }
        if (q.layers == 2) {
            const size_t R2 = (size_t)3 * d.max_batch * d.K;  // rows of the second-hop tables
            q.hop2.node = (int32_t *)take(R2, 4);
            q.hop2.t = (double *)take(R2, 8);
            q.hop2.cnt = (int32_t *)take(R2, 4);
            q.hop2.nbr = (int32_t *)take(R2 * d.K, 4);
            q.hop2.eid = (int32_t *)take(R2 * d.K, 4);
            q.hop2.ts = (double *)take(R2 * d.K, 8);
            q.h1 = (float *)take((size_t)3 * d.max_batch * (d.K + 1) * E, 4);
            q.mr_ci = (int32_t *)take((size_t)3 * d.max_batch * (d.K + 1), 4);
            size_t slots = 1024;
            while (slots < (size_t)2 * 3 * d.max_batch * (d.K + 1))
                slots *= 2;
            q.mr_tab = (uint32_t *)take(slots, 4);
            q.mr_tab_mask = (uint32_t)(slots - 1);
        }
        {   // the items' matrices: widths of the wider layer
            const size_t items = (size_t)3 * d.max_batch * (q.layers == 2 ? d.K + 1 : 1);
            const size_t in_w = q.layers == 2 && E > M ? E : M, a_w = in_w + T, kv_w = in_w + d.F + T;
            q.mr_qin = (float *)take(items * a_w, 4);
            q.mr_qv = (float *)take(items * a_w, 4);
            q.mr_qt = (float *)take(items * d.H * kv_w, 4);
            q.mr_kvb = (float *)take(items * d.H * kv_w, 4);
            q.mr_o = (float *)take(items * a_w, 4);
            q.mr_x1 = (float *)take(items * (a_w + in_w), 4);
            q.mr_h1 = (float *)take(items * E, 4);
            q.mr_has = (int32_t *)take(items, 4);
            q.mr_itq = (int32_t *)take(items, 4);
            q.mr_itj = (int32_t *)take(items, 4);
            q.mr_n = (int32_t *)take(64, 4);
        }
    }
    q.b_d1 = (const float *)take(E, 4);
    q.w_d2 = (const float *)take(E, 4);
    q.b_d2 = (const float *)take(1, 4);
    q.T_d1 = (const float *)take(2 * E * E, 4);
    biggest = 2 * E * E > biggest ? 2 * E * E : biggest;
    if (emb == TIG_EMB_TIME_PROJECTION)
        q.time_proj_w = (const float *)take(M, 4);
    if (agg == TIG_AGG_MEAN) {
        q.acc = (double *)take((size_t)2 * d.max_batch * kAccCopies * (M + T + d.F), 8);
        q.acc_cnt = (int32_t *)take((size_t)2 * d.max_batch, 4);
    }
    float *stage = (float *)take(biggest > T ? biggest : T, 4);
    float *nf = node_feat ? (float *)take((size_t)num_nodes * M, 4) : nullptr;
    q.node_feat = nf;
    q.fused_embed = attn && !node_feat && q.layers == 1;
    if (p)
        *p = q;
    if (raw_stage)
        *raw_stage = stage;
    if (nf_dst)
        *nf_dst = nf;
    return off;
}

size_t modules_workspace_bytes(const Dims &d, const tig_modules &m, int64_t num_nodes)
{
    return mod_layout(d, m.aggregator, m.updater, m.embedding, m.num_layers, m.node_feat != nullptr, num_nodes, nullptr,
                      nullptr, nullptr, nullptr);
}

bool modules_supported(const Dims &d, const tig_modules &m)
{
    ModParams p = {};
    p.agg = m.aggregator;
    p.upd = m.updater;
    p.emb = m.embedding;
    const ModDims md = mod_dims(d, p);
    if (m.embedding != TIG_EMB_ATTENTION && d.E != d.M)
        return false;
    if (m.num_layers == 2 && (m.embedding != TIG_EMB_ATTENTION || (d.E + d.T) % d.H != 0 || d.K + 1 > kWave))
        return false;
    return d.prec == TIG_FP32 && update_lds(md) <= 160 * 1024 && msgsum_lds(md) <= 64 * 1024 && decode_lds(md) <= 160 * 1024 && d.K <= kModThreads &&
           (m.embedding != TIG_EMB_ATTENTION || (d.H <= kMrMaxHeads && d.H * d.K <= kWave && d.dkv <= kMrCC * kWave &&
                                                  d.E + d.F + d.T <= kMrCC * kWave));
}

hipError_t modules_attach(const Dims &d, const tig_modules &m, const tig_weights &w, int64_t num_nodes, void *workspace,
                          ModParams *out, hipStream_t s)
{
    ModParams p;
    float *stage = nullptr, *nf = nullptr;
    mod_layout(d, m.aggregator, m.updater, m.embedding, m.num_layers, m.node_feat != nullptr, num_nodes, (char *)workspace, &p,
               &stage, &nf);
    const ModDims md = mod_dims(d, p);
    const int M = d.M, T = d.T, E = d.E, D = d.Dmsg, GM = md.G * d.M;
    hipError_t e;
    auto vec = [&](const float *dst, const float *src, size_t n) -> hipError_t {
        return hipMemcpyAsync((void *)dst, src, 4 * n, hipMemcpyDefault, s);
    };
    // a matrix goes through the staging area (the source may be host memory) and is transposed from there
    auto mat = [&](const float *dst_t, const float *src, int rows, int cols) -> hipError_t {
        const size_t n = (size_t)rows * cols;
        hipError_t e2 = hipMemcpyAsync(stage, src, 4 * n, hipMemcpyDefault, s);
        if (e2 != hipSuccess)
            return e2;
        hipLaunchKernelGGL(k_mod_transpose, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (float *)dst_t, stage, rows, cols);
        return hipGetLastError();
    };
    auto rev = [&](const double *dst, const float *src) -> hipError_t {
        hipError_t e2 = hipMemcpyAsync(stage, src, 4 * (size_t)T, hipMemcpyDefault, s);
        if (e2 != hipSuccess)
            return e2;
        hipLaunchKernelGGL(k_mod_revolutions, dim3((T + 255) / 256), dim3(256), 0, s, (double *)dst, stage, T);
        return hipGetLastError();
    };
#define MOD_TRY(x)            \
    if ((e = (x)) != hipSuccess) \
        return e
    MOD_TRY(rev(p.time_w_rev, w.time_w));
    MOD_TRY(rev(p.time_b_rev, w.time_b));
    MOD_TRY(vec(p.b_i, w.b_i, GM));
    MOD_TRY(vec(p.b_h, w.b_h, GM));
    MOD_TRY(mat(p.T_i, w.W_i, GM, D));
    MOD_TRY(mat(p.T_h, w.W_h, GM, M));
    if (m.embedding == TIG_EMB_ATTENTION) {
        // the second layer's matrices have the first layer's roles with E-wide input rows
        tig_layer_weights first = {};
        first.W_Q = w.W_Q, first.b_Q = w.b_Q, first.W_K = w.W_K, first.b_K = w.b_K, first.W_V = w.W_V, first.b_V = w.b_V;
        first.W_O = w.W_O, first.b_O = w.b_O, first.W_m1 = w.W_m1, first.b_m1 = w.b_m1, first.W_m2 = w.W_m2, first.b_m2 = w.b_m2;
        for (int l = 0; l < p.layers; ++l) {
            const tig_layer_weights &src = l == 0 ? first : *m.layer2;
            const AttnLayer &A = p.L[l];
            const int in_w = l == 0 ? M : E, a_w = in_w + T, kv_w = in_w + d.F + T;
            MOD_TRY(vec(A.b_Q, src.b_Q, a_w));
            MOD_TRY(vec(A.b_K, src.b_K, a_w));
            MOD_TRY(vec(A.b_V, src.b_V, a_w));
            MOD_TRY(vec(A.b_O, src.b_O, a_w));
            MOD_TRY(vec(A.b_m1, src.b_m1, E));
            MOD_TRY(vec(A.b_m2, src.b_m2, E));
            MOD_TRY(mat(A.T_Q, src.W_Q, a_w, a_w));
            MOD_TRY(mat(A.T_K, src.W_K, a_w, kv_w));
            MOD_TRY(mat(A.T_V, src.W_V, a_w, kv_w));
            MOD_TRY(mat(A.T_O, src.W_O, a_w, a_w));
            MOD_TRY(mat(A.T_m1, src.W_m1, E, a_w + in_w));
            MOD_TRY(mat(A.T_m2, src.W_m2, E, E));
            MOD_TRY(vec(A.N_Q, src.W_Q, (size_t)a_w * a_w));
            MOD_TRY(vec(A.N_V, src.W_V, (size_t)a_w * kv_w));
            MOD_TRY(vec(A.N_O, src.W_O, (size_t)a_w * a_w));
            MOD_TRY(vec(A.N_m1, src.W_m1, (size_t)E * (a_w + in_w)));
            MOD_TRY(vec(A.N_m2, src.W_m2, (size_t)E * E));
        }
    }
    MOD_TRY(vec(p.b_d1, w.b_d1, E));
    MOD_TRY(vec(p.w_d2, w.w_d2, E));
    MOD_TRY(vec(p.b_d2, w.b_d2, 1));
    MOD_TRY(mat(p.T_d1, w.W_d1, E, 2 * E));
    if (m.embedding == TIG_EMB_TIME_PROJECTION)
        MOD_TRY(vec(p.time_proj_w, m.time_proj_w, M));
    if (nf)
        MOD_TRY(hipMemcpyAsync(nf, m.node_feat, 4 * (size_t)num_nodes * M, hipMemcpyDefault, s));
    if (p.acc) {
        MOD_TRY(launch_fill_zero(p.acc, (size_t)2 * d.max_batch * kAccCopies * (M + T + d.F) * 8, s));
        MOD_TRY(launch_fill_zero(p.acc_cnt, (size_t)2 * d.max_batch * 4, s));
    }
    MOD_TRY(hipFuncSetAttribute((const void *)k_mod_update, hipFuncAttributeMaxDynamicSharedMemorySize, update_lds(md)));
    MOD_TRY(hipFuncSetAttribute((const void *)k_mod_msgsum, hipFuncAttributeMaxDynamicSharedMemorySize, msgsum_lds(md)));
    MOD_TRY(hipFuncSetAttribute((const void *)k_mod_decode, hipFuncAttributeMaxDynamicSharedMemorySize, decode_lds(md)));
#undef MOD_TRY
    *out = p;
    return hipStreamSynchronize(s);
}

// Everything of a step after the selection (and, for the attention embedding, the query
// preparation): state update, memory overwrite, embedding, decoder, inspection outputs.
// `marks`: NULL, or two events recorded after the state update + overwrite and after the rest.
hipError_t launch_modules(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                          const ModParams &p, hipStream_t s, hipEvent_t *marks)
{
    const ModDims md = mod_dims(d, p);
    hipError_t e;
    if (a.msg_count > 0) {
        if (p.agg == TIG_AGG_MEAN)
            hipLaunchKernelGGL(k_mod_msgsum, dim3((2 * a.msg_count + kMsgEntries - 1) / kMsgEntries), dim3(kMsgThreads),
                               msgsum_lds(md), s, a, md, p);
        hipLaunchKernelGGL(k_mod_update, dim3(2 * a.msg_count), dim3(kModThreads), update_lds(md), s, a, md, p);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    if (p.fused_embed) {
        // attention without node features: the fused kernels of the headline instance embed and decode,
        // reading updated nodes' rows from the staged rows (the memory overwrite runs beside them)
        if (marks && (e = hipEventRecord(marks[0], s)) != hipSuccess)
            return e;
        StepArgs f = a;
        f.finish_here = 1;
        if ((e = launch_gru(d, plan, pw, f, s, false)) != hipSuccess || (e = launch_embed(d, plan, pw, f, s)) != hipSuccess ||
            (e = launch_closing(d, plan, pw, f, GruAhead{}, s)) != hipSuccess)
            return e;
        return marks ? hipEventRecord(marks[1], s) : hipSuccess;
    }
    if (a.msg_count > 0) {
        hipLaunchKernelGGL(k_mod_commit, dim3(64), dim3(kModThreads), 0, s, a, d.M);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    if (marks && (e = hipEventRecord(marks[0], s)) != hipSuccess)
        return e;
    // from here on every state row is read from the memory table: nothing is "applied" any more
    StepArgs b = a;
    b.msg_count = 0;
    const int B = a.count;
    if (p.emb == TIG_EMB_ATTENTION) {
        b.finish_here = 1;  // slots of the query set (its row references all name memory rows)
        if ((e = launch_gru(d, plan, pw, b, s)) != hipSuccess)
            return e;
        // one attention layer + merge MLP over all items of `mode`: item list and query rows, the layer's
        // products as contractions over the items, the attention core per item in between
        auto layer_pass = [&](const ModDims &ld, const AttnLayer &A, int mode) {
            const int items_max = 3 * B * (mode == kMrFirst ? d.K + 1 : 1);
            const RowCount rc = mode == kMrFirst ? RowCount{p.mr_n, 0, 1, items_max}
                                                 : RowCount{b.qs.n_u, b.roles == 3 ? B : 0, 1, items_max};
            const int da = ld.da, dh = ld.dh, dkv = ld.dkv, M_ = ld.M, E_ = ld.E, H = ld.H;
            const dim3 g_items((3 * B + kMrWaves - 1) / kMrWaves), g_attn((items_max + kModWaves - 1) / kModWaves);
            auto prod = [&](float *C, int ldc, const float *X, int lda, const float *W, int ldw, const float *bias, int N, int Kd) {
                RowGemm g = {};
                g.A = X, g.lda = lda, g.W = W, g.ldw = ldw, g.bias = bias, g.C = C, g.ldc = ldc, g.N = N, g.Kd = Kd, g.rc = rc;
                g.vecA = rowgemm_vec_ok(X, lda), g.vecW = rowgemm_vec_ok(W, ldw);
                return g;
            };
            if (mode == kMrSingle)
                hipLaunchKernelGGL(k_mr_items<kMrSingle>, g_items, dim3(kMrWaves * kWave), 0, s, b, ld, p);
            else if (mode == kMrFirst)
                hipLaunchKernelGGL(k_mr_items<kMrFirst>, g_items, dim3(kMrWaves * kWave), 0, s, b, ld, p);
            else
                hipLaunchKernelGGL(k_mr_items<kMrSecond>, g_items, dim3(kMrWaves * kWave), 0, s, b, ld, p);
            launch_rowgemm(prod(p.mr_qv, da, p.mr_qin, da, A.N_Q, da, A.b_Q, da, da), 1, s);
            {   // q~_h = W_K,h^T Qv_h, every head in one launch
                RowGemm g = prod(p.mr_qt, H * dkv, p.mr_qv, da, A.T_K, da, nullptr, dkv, dh);
                g.zA = dh, g.zW = dh, g.zC = dkv;
                g.vecA = g.vecA && dh % 4 == 0, g.vecW = g.vecW && dh % 4 == 0;
                launch_rowgemm(g, H, s);
            }
#define MR_ATTN(MODE)                                                                                             \
    do {                                                                                                          \
        if (H <= 2 && dkv <= 256)                                                                                 \
            hipLaunchKernelGGL((k_mr_attn<MODE, 2, 4>), g_attn, dim3(kModThreads), 0, s, b, ld, p);               \
        else if (H <= 2)                                                                                          \
            hipLaunchKernelGGL((k_mr_attn<MODE, 2, kMrCC>), g_attn, dim3(kModThreads), 0, s, b, ld, p);           \
        else                                                                                                      \
            hipLaunchKernelGGL((k_mr_attn<MODE, kMrMaxHeads, kMrCC>), g_attn, dim3(kModThreads), 0, s, b, ld, p); \
    } while (0)
            if (mode == kMrSingle)
                MR_ATTN(kMrSingle);
            else if (mode == kMrFirst)
                MR_ATTN(kMrFirst);
            else
                MR_ATTN(kMrSecond);
#undef MR_ATTN
            {   // o_h = W_V,h KVB_h + b_V,h
                RowGemm g = prod(p.mr_o, da, p.mr_kvb, H * dkv, A.N_V, dkv, A.b_V, dh, dkv);
                g.zA = dkv, g.zW = dh * dkv, g.zC = dh, g.zBias = dh;
                g.vecA = g.vecA && dkv % 4 == 0, g.vecW = g.vecW && (dh * dkv) % 4 == 0;
                launch_rowgemm(g, H, s);
            }
            {   // attn = W_O o + b_O into the head of the merge layer's input; the zero vector without neighbours
                RowGemm g = prod(p.mr_x1, da + M_, p.mr_o, da, A.N_O, da, A.b_O, da, da);
                g.rowmask = p.mr_has;
                launch_rowgemm(g, 1, s);
            }
            {
                RowGemm g = prod(p.mr_h1, E_, p.mr_x1, da + M_, A.N_m1, da + M_, A.b_m1, E_, da + M_);
                g.relu = 1;
                launch_rowgemm(g, 1, s);
            }
            if (mode == kMrFirst) {  // the first layer's rows, one per item
                launch_rowgemm(prod(p.h1, E_, p.mr_h1, E_, A.N_m2, E_, A.b_m2, E_, E_), 1, s);
            } else {                 // the embedding rows of the query set
                RowGemm g = prod(b.emb_u, E_, p.mr_h1, E_, A.N_m2, E_, A.b_m2, E_, E_);
                g.remap_nu = b.qs.n_u, g.remap_2b = 2 * B;
                launch_rowgemm(g, 1, s);
            }
        };
        if (p.layers == 2) {
            const ModDims md2 = second_layer_dims(md);
            if ((e = launch_fill_zero(p.mr_n, 4, s)) != hipSuccess ||
                (e = launch_fill_zero(p.mr_tab, ((size_t)p.mr_tab_mask + 1) * 4, s)) != hipSuccess)
                return e;
            hipLaunchKernelGGL(k_mod_hop2, dim3(3 * B), dim3(kModThreads), 0, s, b, md, p);
            layer_pass(md, p.L[0], kMrFirst);
            layer_pass(md2, p.L[1], kMrSecond);
        } else {
            layer_pass(md, p.L[0], kMrSingle);
        }
        hipLaunchKernelGGL(k_mod_decode, dim3((B + kEV - 1) / kEV), dim3(kModThreads), decode_lds(md), s, b, md, p, 1);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
        // inspection outputs; the query set's counter is cleared for its next preparation
        if ((e = launch_closing(d, plan, pw, b, GruAhead{}, s, false)) != hipSuccess)
            return e;
    } else {
        const size_t n = (size_t)a.roles * B * d.M;
        hipLaunchKernelGGL(k_mod_simple, dim3((unsigned)((n + kModThreads - 1) / kModThreads)), dim3(kModThreads), 0, s, b, md, p);
        hipLaunchKernelGGL(k_mod_decode, dim3((B + kEV - 1) / kEV), dim3(kModThreads), decode_lds(md), s, b, md, p, 0);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    if (marks && (e = hipEventRecord(marks[1], s)) != hipSuccess)
        return e;
    return hipSuccess;
}

}  // namespace tig
