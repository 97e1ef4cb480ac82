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
//   k_mod_rows     attention embedding in its direct form (separate query / key / value / output
//                  projections, merge MLP), one workgroup per distinct query, node features added
//                  wherever a state row is read; a negative's neighbours are looked up here
//   k_mod_hop2     two stacked attention layers (the embedding module's sum over the 2-hop temporal
//                  neighbourhood): the K most recent events, before the QUERY's time, of every
//                  neighbour of every distinct query; k_mod_rows then runs twice: the first layer for
//                  each (query, neighbour) pair and each query itself, the second layer over those rows
//   k_mod_decode   eight events per workgroup: both logits (and, for the attention embedding, the
//                  per-query embedding rows out of the distinct rows)
// Weight matrices are read through transposed copies ([in x out]) so that a thread that owns an
// output reads consecutive addresses.
#include <hip/hip_runtime.h>

#include "kernels_common.h"
#include "prepare.h"
#include "winners.h"

namespace tig {

namespace {

constexpr int kModThreads = 256;
constexpr int kModWaves = kModThreads / kWave;
constexpr int kKC = 8;   // neighbour slots per register chunk
constexpr int kEV = 8;   // events per decoder workgroup

struct ModDims {
    int M, T, F, E, K, H, da, dh, dkv, Dmsg;
    int G;  // gate blocks of the state update: 3 (GRU: r, z, n) or 1 (plain recurrent cell)
    int agg, upd, emb;
};

// What one launch of k_mod_rows computes.
enum RowsMode {
    kRowsSingle = 0,  // the one-layer embedding of every distinct query
    kRowsFirst = 1,   // first of two layers: item (q, j): neighbour j < cnt of query row q at the query's time, j == K: q itself
    kRowsSecond = 2,  // second of two layers, over the first layer's rows
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
#pragma unroll 8
        for (int i = 0; i < in; ++i)  // (unrolled: eight independent loads in flight, not one per step)
            acc += WT[(size_t)i * out + j] * x[i];
        y[j] = acc;
    }
}

// Y[k][j] = bias[j] + sum_i WT[i * out + j] * X[k][i] for k < cnt   (X [cnt x ldx], Y [cnt x out] in LDS)
__device__ inline void multivec_t(const float *WT, int in, int out, const float *X, int ldx, int cnt,
                                  const float *bias, float *Y)
{
    for (int k0 = 0; k0 < cnt; k0 += kKC) {
        for (int j = threadIdx.x; j < out; j += kModThreads) {
            float acc[kKC];
            const float b = bias ? bias[j] : 0.0f;
#pragma unroll
            for (int u = 0; u < kKC; ++u)
                acc[u] = b;
#pragma unroll 4
            for (int i = 0; i < in; ++i) {
                const float w = WT[(size_t)i * out + j];
#pragma unroll
                for (int u = 0; u < kKC; ++u)
                    acc[u] += w * X[(size_t)(k0 + u < cnt ? k0 + u : k0) * ldx + i];
            }
#pragma unroll
            for (int u = 0; u < kKC; ++u)
                if (k0 + u < cnt)
                    Y[(size_t)(k0 + u) * out + j] = acc[u];
        }
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
// One attention layer + merge MLP of one item, direct form.  d and L are the layer's own dimensions
// and weights (the second layer's input rows are E wide).
__global__ void __launch_bounds__(kModThreads) k_mod_rows(StepArgs a, ModDims d, ModParams p, AttnLayer L, int mode)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + (a.roles == 3 ? a.count : 0);
    const int M = d.M, F = d.F, E = d.E, K = d.K, H = d.H, da = d.da, dh = d.dh, dkv = d.dkv;
    const int x = mode == kRowsFirst ? (int)blockIdx.x / (K + 1) : (int)blockIdx.x;
    const int item = mode == kRowsFirst ? (int)blockIdx.x - x * (K + 1) : K;
    if (x >= n_rows)
        return;
    double *dts = (double *)smem;     // [K]
    int *nbrs = (int *)(dts + K);     // [K]
    int *eids = nbrs + K;             // [K]
    int *meta = eids + K;             // [2] cnt, node (+ 2 of padding)
    float *q_in = (float *)(meta + 4);  // [da]
    float *Qv = q_in + da;            // [da]
    float *kv = Qv + da;              // [K x dkv]
    float *KPs = kv + K * dkv;        // [K x da]
    float *VPs = KPs + K * da;        // [K x da]
    float *sc = VPs + K * da;         // [H x K]
    float *o = sc + H * K;            // [da]
    float *xcat = o + da;             // [da + M]: attn | own row
    float *h1 = xcat + da + M;        // [E]

    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    if (mode == kRowsSingle && x >= n_u && threadIdx.x < kWave) {  // a negative: the first wavefront looks up its neighbours
        int32_t rf, ee;
        double ts_k;
        (void)finish_negative(a, K, x - n_u, rf, ee, ts_k);
    }
    __syncthreads();
    // the item's neighbour table: the query's own, or (first of two layers, item < K) the one of its
    // neighbour `item` at the query's time
    const bool hop = mode == kRowsFirst && item < K;
    if (hop) {
        const int c = a.qs.cnt[q];
        if (item >= (c < 0 ? 0 : (c > K ? K : c)))
            return;  // (uniform over the workgroup) an unused slot
    }
    const QuerySet &tab = hop ? p.hop2 : a.qs;
    const int trow = hop ? q * K + item : q;
    if (threadIdx.x == 0) {
        const int c = tab.cnt[trow];
        meta[0] = c < 0 ? 0 : (c > K ? K : c);
        meta[1] = hop ? a.qs.nbr[(size_t)q * K + item] : a.qs.node[q];
    }
    const double t_q = a.qs.t[q];
    if ((int)threadIdx.x < K) {
        nbrs[threadIdx.x] = tab.nbr[(size_t)trow * K + threadIdx.x];
        eids[threadIdx.x] = tab.eid[(size_t)trow * K + threadIdx.x];
        dts[threadIdx.x] = t_q - tab.ts[(size_t)trow * K + threadIdx.x];
    }
    __syncthreads();
    const int cnt = meta[0];
    const int32_t u = meta[1];
    const float *rows1 = p.h1 + (size_t)q * (K + 1) * E;  // second layer: the first layer's rows of this query
    for (int j = threadIdx.x; j < da; j += kModThreads) {
        float v;
        if (j >= M)
            v = time_enc(p.time_w_rev[j - M], p.time_b_rev[j - M], 0.0);
        else if (mode == kRowsSecond)
            v = rows1[(size_t)K * E + j];
        else
            v = repr_elem(a, p, M, u, j);
        q_in[j] = v;
        if (j < M)
            xcat[da + j] = v;
    }
    // key / value rows [row of the neighbour | e | Phi(t - t_k)]
    for (int idx = threadIdx.x; idx < cnt * dkv; idx += kModThreads) {
        const int k = idx / dkv, i = idx - k * dkv;
        float v;
        if (i < M)
            v = mode == kRowsSecond ? rows1[(size_t)k * E + i] : repr_elem(a, p, M, nbrs[k], i);
        else if (i < M + F)
            v = eids[k] >= 0 ? a.edge_feat[(size_t)eids[k] * F + (i - M)] : 0.0f;
        else
            v = time_enc(p.time_w_rev[i - M - F], p.time_b_rev[i - M - F], dts[k]);
        kv[idx] = v;
    }
    __syncthreads();
    if (cnt > 0) {
        matvec_t(L.T_Q, da, da, q_in, L.b_Q, Qv);
        multivec_t(L.T_K, dkv, da, kv, dkv, cnt, L.b_K, KPs);
        multivec_t(L.T_V, dkv, da, kv, dkv, cnt, L.b_V, VPs);
        __syncthreads();
        const float scale = 1.0f / sqrtf((float)dh);
        for (int idx = threadIdx.x; idx < H * cnt; idx += kModThreads) {
            const int hh = idx / cnt, k = idx - hh * cnt;
            float s = 0.0f;
            for (int e = 0; e < dh; ++e)
                s += Qv[hh * dh + e] * KPs[(size_t)k * da + hh * dh + e];
            sc[hh * K + k] = s * scale;
        }
        __syncthreads();
        if ((int)threadIdx.x < H) {
            const int hh = threadIdx.x;
            float mx = -INFINITY, sum = 0.0f;
            for (int k = 0; k < cnt; ++k)
                mx = fmaxf(mx, sc[hh * K + k]);
            for (int k = 0; k < cnt; ++k) {
                const float e = expf(sc[hh * K + k] - mx);
                sc[hh * K + k] = e;
                sum += e;
            }
            for (int k = 0; k < cnt; ++k)
                sc[hh * K + k] /= sum;
        }
        __syncthreads();
        for (int j = threadIdx.x; j < da; j += kModThreads) {
            const int hh = j / dh;
            float acc = 0.0f;
            for (int k = 0; k < cnt; ++k)
                acc += sc[hh * K + k] * VPs[(size_t)k * da + j];
            o[j] = acc;
        }
        __syncthreads();
        matvec_t(L.T_O, da, da, o, L.b_O, xcat);
    } else {
        for (int j = threadIdx.x; j < da; j += kModThreads)
            xcat[j] = 0.0f;  // an empty neighbourhood gives the zero vector (no bias)
    }
    __syncthreads();
    matvec_t(L.T_m1, da + M, E, xcat, L.b_m1, h1);
    __syncthreads();
    for (int j = threadIdx.x; j < E; j += kModThreads)
        h1[j] = fmaxf(h1[j], 0.0f);
    __syncthreads();
    float *out = mode == kRowsFirst ? p.h1 + ((size_t)q * (K + 1) + item) * E : a.emb_u + (size_t)q * E;
    for (int j = threadIdx.x; j < E; j += kModThreads) {
        float acc = L.b_m2[j];
        for (int i = 0; i < E; ++i)
            acc += L.T_m2[(size_t)i * E + j] * h1[i];
        out[j] = acc;
    }
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
#pragma unroll 4
        for (int i = 0; i < E; ++i) {  // (unrolled: the weight loads of four steps are in flight together)
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

int rows_lds(const ModDims &d)
{
    return d.K * 8 + (2 * d.K + 4) * 4 +
           (2 * d.da + d.K * d.dkv + 2 * d.K * d.da + d.H * d.K + d.da + d.da + d.M + d.E) * 4;
}

// the larger of the two layers' needs (the second layer's rows are E wide)
int rows_lds_all(const ModDims &d, int layers)
{
    const int a = rows_lds(d), b = layers == 2 ? rows_lds(second_layer_dims(d)) : 0;
    return a > b ? a : b;
}

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
    if (m.num_layers == 2 && (m.embedding != TIG_EMB_ATTENTION || (d.E + d.T) % d.H != 0))
        return false;
    return d.prec == TIG_FP32 && update_lds(md) <= 160 * 1024 && msgsum_lds(md) <= 64 * 1024 && rows_lds_all(md, m.num_layers) <= 160 * 1024 &&
           decode_lds(md) <= 160 * 1024 && d.K <= kModThreads;
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
    MOD_TRY(hipFuncSetAttribute((const void *)k_mod_rows, hipFuncAttributeMaxDynamicSharedMemorySize, rows_lds_all(md, p.layers)));
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
        if (p.layers == 2) {
            const ModDims md2 = second_layer_dims(md);
            hipLaunchKernelGGL(k_mod_hop2, dim3(3 * B), dim3(kModThreads), 0, s, b, md, p);
            hipLaunchKernelGGL(k_mod_rows, dim3(3 * B * (d.K + 1)), dim3(kModThreads), rows_lds(md), s, b, md, p, p.L[0], (int)kRowsFirst);
            hipLaunchKernelGGL(k_mod_rows, dim3(3 * B), dim3(kModThreads), rows_lds(md2), s, b, md2, p, p.L[1], (int)kRowsSecond);
        } else {
            hipLaunchKernelGGL(k_mod_rows, dim3(3 * B), dim3(kModThreads), rows_lds(md), s, b, md, p, p.L[0], (int)kRowsSingle);
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
