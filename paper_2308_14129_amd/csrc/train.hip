// Training step (paper Sec. II-C: the decoder's edge probabilities "provide the self-supervised
// signals for training"; Alg. 2: "Training and compute loss", "Backward and Optimize"), device side.
// gfx950 only, fp32.
//
// The step's forward pass is recomputed here in its DIRECT form (separate query / key / value /
// output projections, the intermediates a backward pass needs kept in memory), then the loss
// (binary cross-entropy on the logits of each event against one negative), the hand-written
// backward pass and a plain SGD update of the fp32 master weights; the folded, lane-ordered
// weights that the inference kernels read are rebuilt from the masters afterwards (pack.hip).
//   k_tr_rows_fwd   one workgroup per distinct query: attention and merge MLP from the step's
//                   state rows (a negative's neighbours are looked up here)
//   k_tr_decoder    one workgroup per event: both logits, loss terms, embedding rows out, and the
//                   decoder's backward down to the embeddings (added into the rows' gradients)
//   k_tr_rows_bwd   one workgroup per distinct query: merge MLP and attention backward; the
//                   gradient w.r.t. state rows that this step's GRU wrote goes to those rows
//   k_tr_gru_bwd    one workgroup per applied winner: message and GRU gates recomputed from the
//                   memory as the step found it, backward to the gate pre-activations
//   k_gemm_tn       every weight gradient is dW = D^T X over the rows' stored (delta, input) pairs:
//                   a [out x in] contraction over thousands of rows on the matrix cores (fp32
//                   16x16x4), split over the row range, partial results added with atomics
//   k_colsum        bias and time-encoding gradients: column sums of stored per-row values
// Weight matrices are kept twice, [out x in] and transposed: a thread that owns an output reads
// the transposed copy, a thread that owns an input the native one, so both directions are
// coalesced.
#include <hip/hip_runtime.h>

#include <cstring>

#include "kernels_common.h"
#include "prepare.h"
#include "winners.h"

namespace tig {

namespace {

constexpr int kTrThreads = 256;
constexpr int kKC = 8;  // neighbour slots per register chunk

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

// y[j] = bias[j] + sum_i WT[i * out + j] * x[i]   (x, y in LDS)
__device__ inline void matvec_t(const float *WT, int in, int out, const float *x, const float *bias, float *y)
{
    for (int j = threadIdx.x; j < out; j += kTrThreads) {
        float acc = bias ? bias[j] : 0.0f;
#pragma unroll 8
        for (int i = 0; i < in; ++i)  // (unrolled: eight independent weight loads in flight, not one per step)
            acc += WT[(size_t)i * out + j] * x[i];
        y[j] = acc;
    }
}

// dx[i] = sum_o W[o * in + i] * dy[o]  for i in [0, in)   (dy, dx in LDS)
__device__ inline void matvec_n(const float *W, int out, int in, const float *dy, float *dx)
{
    for (int i = threadIdx.x; i < in; i += kTrThreads) {
        float acc = 0.0f;
#pragma unroll 8
        for (int o = 0; o < out; ++o)
            acc += W[(size_t)o * in + i] * dy[o];
        dx[i] = acc;
    }
}

// Y[k][j] = bias[j] + sum_i WT[i * out + j] * X[k][i] for k < cnt   (X [cnt x ldx], Y [cnt x out] in LDS)
__device__ inline void multivec_t(const float *WT, int in, int out, const float *X, int ldx, int cnt,
                                  const float *bias, float *Y)
{
    for (int k0 = 0; k0 < cnt; k0 += kKC) {
        for (int j = threadIdx.x; j < out; j += kTrThreads) {
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
    // per neighbour slot (row x * K + k)
    float *KV, *KP, *VP, *DKP, *DVP;
    // per (pair, event): pair 0 = (source, destination), pair 1 = (source, negative); row p * count + b
    float *CAT, *DY, *G_, *DLOGIT, *LOSS;
    // per applied winner r, and per entry of the applied batch
    float *MSG, *DGI, *DGH, *TGG, *D_STAG;
    int32_t *n_rows;  // [1] distinct queries of the step (written by the forward kernel's block 0)
    int32_t *live;    // [3B x K] the filled neighbour slots (row x * K + k) of the step, in no particular order
    int32_t *n_live;  // [1] their number (cleared with the gradients)
};

// compact row of query-set row q
__device__ inline int compact_row(int q, int n_u, int count) { return q < 2 * count ? q : n_u + (q - 2 * count); }

// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kTrThreads) k_tr_rows_fwd(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + a.count;
    if (blockIdx.x == 0 && threadIdx.x == 0)
        *t.n_rows = n_rows;
    const int x = (int)blockIdx.x;
    if (x >= n_rows)
        return;
    const int M = d.M, F = d.F, E = d.E, K = d.K, H = d.H, da = d.da, dh = d.dh, dkv = d.dkv;
    double *dts = (double *)smem;     // [K]
    int *refs = (int *)(dts + K);     // [K]
    int *eids = refs + K;             // [K]
    int *meta = eids + K;             // [2] cnt, self_ref (+ 2 of padding)
    float *s_u = (float *)(meta + 4); // [M]
    float *q_in = s_u + M;            // [da]
    float *Qv = q_in + da;            // [da]
    float *kv = Qv + da;              // [K x dkv]
    float *KPs = kv + K * dkv;        // [K x da]
    float *VPs = KPs + K * da;        // [K x da]
    float *sc = VPs + K * da;         // [H x K]
    float *o = sc + H * K;            // [da]
    float *xcat = o + da;             // [da + M]: attn | s_u
    float *h1 = xcat + da + M;        // [E]

    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    if (x >= n_u && threadIdx.x < kWave) {  // a negative: the first wavefront looks up its neighbours
        int32_t rf, ee;
        double ts_k;
        (void)finish_negative(a, K, x - n_u, rf, ee, ts_k);
        if (threadIdx.x == 0)
            a.qs.self_ref[q] = resolve_ref(ref_ctx(a), a.neg[x - n_u]);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int c = a.qs.cnt[q];
        meta[0] = c < 0 ? 0 : (c > K ? K : c);
        meta[1] = a.qs.self_ref[q];
    }
    const double t_q = a.qs.t[q];
    if ((int)threadIdx.x < K) {
        refs[threadIdx.x] = a.qs.ref[(size_t)q * K + threadIdx.x];
        eids[threadIdx.x] = a.qs.eid[(size_t)q * K + threadIdx.x];
        dts[threadIdx.x] = t_q - a.qs.ts[(size_t)q * K + threadIdx.x];
    }
    __syncthreads();
    const int cnt = meta[0];
    const float *self = state_row(a, M, meta[1]);
    if (threadIdx.x < kWave && cnt > 0) {
        // the filled slots go on the list that the key / value weight gradients run over (most rows of
        // a step are negatives without history: their K slots are zero rows)
        int base = 0;
        if (threadIdx.x == 0)
            base = atomicAdd(t.n_live, cnt);
        base = __shfl(base, 0);
        if ((int)threadIdx.x < cnt && base >= 0 && base + (int)threadIdx.x < 3 * a.count * K)
            t.live[base + threadIdx.x] = x * K + (int)threadIdx.x;
    }
    for (int j = threadIdx.x; j < da; j += kTrThreads) {
        const float v = j < M ? (self ? self[j] : 0.0f) : time_enc(pw.time_w_rev[j - M], pw.time_b_rev[j - M], 0.0);
        q_in[j] = v;
        if (j < M)
            s_u[j] = v;
        t.QIN[(size_t)x * da + j] = v;
    }
    // key / value rows [s_v | e | Phi(t - t_k)]; unused slots are zero rows
    for (int idx = threadIdx.x; idx < K * dkv; idx += kTrThreads) {
        const int k = idx / dkv, i = idx - k * dkv;
        float v = 0.0f;
        if (k < cnt) {
            if (i < M) {
                const float *row = state_row(a, M, refs[k]);
                v = row ? row[i] : 0.0f;
            } else if (i < M + F) {
                v = eids[k] >= 0 ? a.edge_feat[(size_t)eids[k] * F + (i - M)] : 0.0f;
            } else {
                v = time_enc(pw.time_w_rev[i - M - F], pw.time_b_rev[i - M - F], dts[k]);
            }
        }
        kv[idx] = v;
        t.KV[((size_t)x * K) * dkv + idx] = v;
    }
    __syncthreads();
    if (cnt > 0) {
        matvec_t(t.T_Q, da, da, q_in, t.b_Q, Qv);
        multivec_t(t.T_K, dkv, da, kv, dkv, cnt, t.b_K, KPs);
        multivec_t(t.T_V, dkv, da, kv, dkv, cnt, t.b_V, VPs);
        __syncthreads();
        const float scale = 1.0f / sqrtf((float)dh);
        for (int idx = threadIdx.x; idx < H * cnt; idx += kTrThreads) {
            const int h = idx / cnt, k = idx - h * cnt;
            float s = 0.0f;
            for (int e = 0; e < dh; ++e)
                s += Qv[h * dh + e] * KPs[(size_t)k * da + h * dh + e];
            sc[h * K + k] = s * scale;
        }
        __syncthreads();
        if ((int)threadIdx.x < H) {
            const int h = threadIdx.x;
            float mx = -INFINITY, sum = 0.0f;
            for (int k = 0; k < cnt; ++k)
                mx = fmaxf(mx, sc[h * K + k]);
            for (int k = 0; k < cnt; ++k) {
                const float e = expf(sc[h * K + k] - mx);
                sc[h * K + k] = e;
                sum += e;
            }
            for (int k = 0; k < cnt; ++k)
                sc[h * K + k] /= sum;
            for (int k = cnt; k < K; ++k)
                sc[h * K + k] = 0.0f;
        }
        __syncthreads();
        for (int j = threadIdx.x; j < da; j += kTrThreads) {
            const int h = j / dh;
            float acc = 0.0f;
            for (int k = 0; k < cnt; ++k)
                acc += sc[h * K + k] * VPs[(size_t)k * da + j];
            o[j] = acc;
        }
        __syncthreads();
        matvec_t(t.T_O, da, da, o, t.b_O, xcat);
    } else {
        for (int j = threadIdx.x; j < da; j += kTrThreads) {
            Qv[j] = 0.0f;
            o[j] = 0.0f;
            xcat[j] = 0.0f;
        }
        for (int idx = threadIdx.x; idx < H * K; idx += kTrThreads)
            sc[idx] = 0.0f;
    }
    for (int j = threadIdx.x; j < M; j += kTrThreads)
        xcat[da + j] = s_u[j];
    __syncthreads();
    matvec_t(t.T_m1, da + M, E, xcat, t.b_m1, h1);
    __syncthreads();
    for (int j = threadIdx.x; j < E; j += kTrThreads)
        h1[j] = fmaxf(h1[j], 0.0f);
    __syncthreads();
    // emb = W_m2 h1 + b_m2 straight to the row of the query set
    for (int j = threadIdx.x; j < E; j += kTrThreads) {
        float acc = t.b_m2[j];
        for (int i = 0; i < E; ++i)
            acc += t.T_m2[(size_t)i * E + j] * h1[i];
        a.emb_u[(size_t)q * E + j] = acc;
        t.H1[(size_t)x * E + j] = h1[j];
    }
    for (int j = threadIdx.x; j < da; j += kTrThreads) {
        t.QV[(size_t)x * da + j] = Qv[j];
        t.O_[(size_t)x * da + j] = o[j];
    }
    for (int j = threadIdx.x; j < da + M; j += kTrThreads)
        t.X1[(size_t)x * (da + M) + j] = xcat[j];
    for (int idx = threadIdx.x; idx < H * K; idx += kTrThreads)
        t.PROB[(size_t)x * H * K + idx] = sc[idx];
    for (int idx = threadIdx.x; idx < K * da; idx += kTrThreads) {
        const bool live = idx / da < cnt;
        t.KP[((size_t)x * K) * da + idx] = live ? KPs[idx] : 0.0f;
        t.VP[((size_t)x * K) * da + idx] = live ? VPs[idx] : 0.0f;
    }
}

// ------------------------------------------------------------------------------------------
__device__ inline float block_sum(float v, float *red)
{
    v = wave_sum_uniform(v);
    if ((threadIdx.x & (kWave - 1)) == 0)
        red[threadIdx.x / kWave] = v;
    __syncthreads();
    float s = 0.0f;
    for (int w = 0; w < kTrThreads / kWave; ++w)
        s += red[w];
    __syncthreads();
    return s;
}

__device__ inline int row_of_entry_tr(const QuerySet &qs, int i, int entries)
{
    int s = qs.slot[i];
    if (s < 0) {
        const int rep = -s - 1;
        s = rep < entries ? qs.slot[rep] : 0;
    }
    return s >= 0 && s < entries ? s : 0;
}

__global__ void __launch_bounds__(kTrThreads) k_tr_decoder(StepArgs a, TrainDims d, TrainBufs t)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int E = d.E, b = (int)blockIdx.x, B = a.count;
    float *em = (float *)smem;  // [3 x E]: source, destination, negative
    float *y = em + 3 * E;      // [E]
    float *dy = y + E;          // [E]
    float *red = dy + E;        // [waves]
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * B ? n_u : 2 * B;
    int row[3];
    row[0] = row_of_entry_tr(a.qs, 2 * b, 2 * B);
    row[1] = row_of_entry_tr(a.qs, 2 * b + 1, 2 * B);
    row[2] = 2 * B + b;
    for (int idx = threadIdx.x; idx < 3 * E; idx += kTrThreads) {
        const int r = idx / E, j = idx - r * E;
        const float v = a.emb_u[(size_t)row[r] * E + j];
        em[idx] = v;
        a.emb[((size_t)r * B + b) * E + j] = v;
    }
    __syncthreads();
    for (int p = 0; p < 2; ++p) {
        const float *ea = em, *eb = em + (1 + p) * E;
        const size_t pr = (size_t)p * B + b;
        for (int j = threadIdx.x; j < E; j += kTrThreads) {
            float acc = t.b_d1[j];
            for (int i = 0; i < E; ++i)
                acc += t.T_d1[(size_t)i * E + j] * ea[i] + t.T_d1[(size_t)(E + i) * E + j] * eb[i];
            y[j] = acc;
        }
        __syncthreads();
        float part = 0.0f;
        for (int j = threadIdx.x; j < E; j += kTrThreads)
            part += t.w_d2[j] * fmaxf(y[j], 0.0f);
        const float logit = block_sum(part, red) + t.b_d2[0];
        // d softplus(sign * logit) / d logit = sign * sigmoid(sign * logit), averaged over the batch
        const float sign = p == 0 ? -1.0f : 1.0f;
        const float z = sign * logit;
        const float dlogit = sign / (1.0f + expf(-z)) / (float)B;
        if (threadIdx.x == 0) {
            (p == 0 ? a.score_pos : a.score_neg)[b] = logit;
            t.DLOGIT[pr] = dlogit;
            t.LOSS[pr] = (z > 0.0f ? z + log1pf(expf(-z)) : log1pf(expf(z))) / (float)B;
        }
        for (int j = threadIdx.x; j < E; j += kTrThreads) {
            const float g = fmaxf(y[j], 0.0f);
            const float v = y[j] > 0.0f ? dlogit * t.w_d2[j] : 0.0f;
            dy[j] = v;
            t.DY[pr * E + j] = v;
            t.G_[pr * E + j] = g;
            t.CAT[pr * 2 * E + j] = ea[j];
            t.CAT[pr * 2 * E + E + j] = eb[j];
        }
        __syncthreads();
        const int xa = compact_row(row[0], n_u, B), xb = compact_row(row[1 + p], n_u, B);
        for (int i = threadIdx.x; i < 2 * E; i += kTrThreads) {
            float acc = 0.0f;
            for (int o2 = 0; o2 < E; ++o2)
                acc += t.W_d1[(size_t)o2 * 2 * E + i] * dy[o2];
            atomicAdd(&t.D_EMB[(size_t)(i < E ? xa : xb) * E + (i < E ? i : i - E)], acc);
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kTrThreads) k_tr_rows_bwd(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int n_u = *a.qs.n_u;
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int n_rows = n_u + a.count;
    const int x = (int)blockIdx.x;
    if (x >= n_rows)
        return;
    const int M = d.M, T = d.T, F = d.F, E = d.E, K = d.K, H = d.H, da = d.da, dh = d.dh, dkv = d.dkv;
    double *dts = (double *)smem;     // [K]
    int *refs = (int *)(dts + K);     // [K]
    int *meta = refs + K;             // [2] (+ K + 2 of padding)
    float *de = (float *)(meta + K + 4);  // [E]
    float *dz1 = de + E;              // [E]
    float *dx = dz1 + E;              // [da + M]
    float *dout = dx + da + M;        // [da]  gradient of the heads' outputs
    float *Qv = dout + da;            // [da]
    float *KPs = Qv + da;             // [K x da]
    float *VPs = KPs + K * da;        // [K x da]
    float *dKP = VPs + K * da;        // [K x da]
    float *dVP = dKP + K * da;        // [K x da]
    float *pr = dVP + K * da;         // [H x K]
    float *dav = pr + H * K;          // [H x K]
    float *dsv = dav + H * K;         // [H x K]
    float *dQv = dsv + H * K;         // [da]
    float *dqin = dQv + da;           // [da]
    float *tg = dqin + da;            // [2T]

    const int q = x < n_u ? x : 2 * a.count + (x - n_u);
    if (threadIdx.x == 0) {
        int c = a.qs.cnt[q];
        meta[0] = c < 0 ? 0 : (c > K ? K : c);
        meta[1] = a.qs.self_ref[q];
    }
    const double t_q = a.qs.t[q];
    if ((int)threadIdx.x < K) {
        refs[threadIdx.x] = a.qs.ref[(size_t)q * K + threadIdx.x];
        dts[threadIdx.x] = t_q - a.qs.ts[(size_t)q * K + threadIdx.x];
    }
    for (int j = threadIdx.x; j < E; j += kTrThreads)
        de[j] = t.D_EMB[(size_t)x * E + j];
    for (int j = threadIdx.x; j < 2 * T; j += kTrThreads)
        tg[j] = 0.0f;
    __syncthreads();
    const int cnt = meta[0];
    // merge MLP: dz1 = (W_m2^T d_emb) where z1 > 0;  dx = W_m1^T dz1 = [d_attn | d s_u]
    for (int i = threadIdx.x; i < E; i += kTrThreads) {
        float acc = 0.0f;
        for (int o2 = 0; o2 < E; ++o2)
            acc += t.W_m2[(size_t)o2 * E + i] * de[o2];
        const float v = t.H1[(size_t)x * E + i] > 0.0f ? acc : 0.0f;
        dz1[i] = v;
        t.DZ1[(size_t)x * E + i] = v;
    }
    __syncthreads();
    matvec_n(t.W_m1, E, da + M, dz1, dx);
    __syncthreads();
    for (int j = threadIdx.x; j < da; j += kTrThreads)
        t.D_ATTN[(size_t)x * da + j] = cnt > 0 ? dx[j] : 0.0f;  // no neighbours: attn is the constant 0
    if (cnt > 0) {
        matvec_n(t.W_O, da, da, dx, dout);
        for (int j = threadIdx.x; j < da; j += kTrThreads)
            Qv[j] = t.QV[(size_t)x * da + j];
        for (int idx = threadIdx.x; idx < cnt * da; idx += kTrThreads) {
            KPs[idx] = t.KP[((size_t)x * K) * da + idx];
            VPs[idx] = t.VP[((size_t)x * K) * da + idx];
        }
        for (int idx = threadIdx.x; idx < H * K; idx += kTrThreads)
            pr[idx] = t.PROB[(size_t)x * H * K + idx];
        __syncthreads();
        for (int idx = threadIdx.x; idx < H * cnt; idx += kTrThreads) {
            const int h = idx / cnt, k = idx - h * cnt;
            float s = 0.0f;
            for (int e = 0; e < dh; ++e)
                s += VPs[(size_t)k * da + h * dh + e] * dout[h * dh + e];
            dav[h * K + k] = s;
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < H * cnt; idx += kTrThreads) {
            const int h = idx / cnt, k = idx - h * cnt;
            float dot = 0.0f;
            for (int k2 = 0; k2 < cnt; ++k2)
                dot += pr[h * K + k2] * dav[h * K + k2];
            dsv[h * K + k] = pr[h * K + k] * (dav[h * K + k] - dot);
        }
        __syncthreads();
        const float scale = 1.0f / sqrtf((float)dh);
        for (int j = threadIdx.x; j < da; j += kTrThreads) {
            const int h = j / dh;
            float acc = 0.0f;
            for (int k = 0; k < cnt; ++k) {
                acc += dsv[h * K + k] * KPs[(size_t)k * da + j];
                dKP[(size_t)k * da + j] = dsv[h * K + k] * Qv[j] * scale;
                dVP[(size_t)k * da + j] = pr[h * K + k] * dout[j];
            }
            dQv[j] = acc * scale;
        }
        __syncthreads();
        matvec_n(t.W_Q, da, da, dQv, dqin);
        __syncthreads();
        // Phi(0)_j = cos(b_j): only the phase takes a gradient from the query row
        for (int j = threadIdx.x; j < T; j += kTrThreads)
            tg[T + j] += -time_enc_sin(pw.time_w_rev[j], pw.time_b_rev[j], 0.0) * dqin[M + j];
        __syncthreads();
        // d kv[k][i] = sum_o W_K[o][i] dKP[k][o] + W_V[o][i] dVP[k][o]; the thread that owns column i
        // sends the state part to the staged rows and keeps the time-encoding part
        for (int i = threadIdx.x; i < dkv; i += kTrThreads) {
            if (i >= M && i < M + F)
                continue;  // edge features are constants
            float gw = 0.0f, gb = 0.0f;
            for (int k0 = 0; k0 < cnt; k0 += kKC) {
                float acc[kKC];
#pragma unroll
                for (int u = 0; u < kKC; ++u)
                    acc[u] = 0.0f;
                for (int o2 = 0; o2 < da; ++o2) {
                    const float wk = t.W_K[(size_t)o2 * dkv + i], wv = t.W_V[(size_t)o2 * dkv + i];
#pragma unroll
                    for (int u = 0; u < kKC; ++u) {
                        const int k = k0 + u < cnt ? k0 + u : k0;
                        acc[u] += wk * dKP[(size_t)k * da + o2] + wv * dVP[(size_t)k * da + o2];
                    }
                }
#pragma unroll
                for (int u = 0; u < kKC; ++u) {
                    const int k = k0 + u;
                    if (k >= cnt)
                        continue;
                    if (i < M) {
                        const int32_t rf = refs[k];
                        if (rf < 0 && rf != kRefNone && ~rf < 2 * a.msg_count)
                            atomicAdd(&t.D_STAG[(size_t)(~rf) * M + i], acc[u]);
                    } else {
                        const int j = i - M - F;
                        const float sn = time_enc_sin(pw.time_w_rev[j], pw.time_b_rev[j], dts[k]);
                        gw += -sn * (float)dts[k] * acc[u];
                        gb += -sn * acc[u];
                    }
                }
            }
            if (i >= M + F) {
                tg[i - M - F] += gw;
                tg[T + i - M - F] += gb;
            }
        }
        for (int j = threadIdx.x; j < da; j += kTrThreads)
            t.DQV[(size_t)x * da + j] = dQv[j];
    } else {
        for (int j = threadIdx.x; j < da; j += kTrThreads) {
            t.DQV[(size_t)x * da + j] = 0.0f;
            dqin[j] = 0.0f;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < K * da; idx += kTrThreads) {
        const bool live = idx / da < cnt;
        t.DKP[((size_t)x * K) * da + idx] = live ? dKP[idx] : 0.0f;
        t.DVP[((size_t)x * K) * da + idx] = live ? dVP[idx] : 0.0f;
    }
    // own state row: from the merge layer and (with neighbours) from the query projection
    const int32_t sr = meta[1];
    if (sr < 0 && sr != kRefNone && ~sr < 2 * a.msg_count)
        for (int i = threadIdx.x; i < M; i += kTrThreads)
            atomicAdd(&t.D_STAG[(size_t)(~sr) * M + i], dx[da + i] + dqin[i]);
    for (int j = threadIdx.x; j < 2 * T; j += kTrThreads)
        t.TG[(size_t)x * 2 * T + j] = tg[j];
}

// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kTrThreads) k_tr_gru_bwd(StepArgs a, PackedWeights pw, TrainDims d, TrainBufs t)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int n_win = *a.n_win;
    n_win = n_win < 2 * a.msg_count ? n_win : 2 * a.msg_count;
    const int r = (int)blockIdx.x;
    if (r >= n_win)
        return;
    const int M = d.M, T = d.T, F = d.F, D = d.Dmsg;
    float *m = (float *)smem;     // [Dmsg]
    float *gi = m + D;            // [3M]
    float *gh = gi + 3 * M;       // [3M]
    float *dgi = gh + 3 * M;      // [3M]
    float *dgh = dgi + 3 * M;     // [3M]
    const WinDesc w = a.win[r];
    const bool ok = w.node >= 0 && (int64_t)w.node < a.num_nodes && w.other >= 0 && (int64_t)w.other < a.num_nodes &&
                    w.entry >= 0 && w.entry < 2 * a.msg_count && w.b >= 0 && w.b < a.msg_count;
    const double dt = ok ? w.t - a.lu[w.node] : 0.0;
    for (int j = threadIdx.x; j < D; j += kTrThreads) {
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
        m[j] = v;
        t.MSG[(size_t)r * D + j] = v;
    }
    __syncthreads();
    matvec_t(t.T_i, D, 3 * M, m, t.b_i, gi);
    matvec_t(t.T_h, M, 3 * M, m, t.b_h, gh);  // h = s_self = the first M entries of the message
    __syncthreads();
    for (int j = threadIdx.x; j < M; j += kTrThreads) {
        const float rg = 1.0f / (1.0f + expf(-(gi[j] + gh[j])));
        const float zg = 1.0f / (1.0f + expf(-(gi[M + j] + gh[M + j])));
        const float ng = tanhf(gi[2 * M + j] + rg * gh[2 * M + j]);
        const float dh = ok ? t.D_STAG[(size_t)w.entry * M + j] : 0.0f;
        const float dn = dh * (1.0f - zg);
        const float dz = dh * (m[j] - ng);
        const float dpre_n = dn * (1.0f - ng * ng);
        const float dpre_r = dpre_n * gh[2 * M + j] * rg * (1.0f - rg);
        const float dpre_z = dz * zg * (1.0f - zg);
        dgi[j] = dpre_r;
        dgi[M + j] = dpre_z;
        dgi[2 * M + j] = dpre_n;
        dgh[j] = dpre_r;
        dgh[M + j] = dpre_z;
        dgh[2 * M + j] = dpre_n * rg;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < 3 * M; j += kTrThreads) {
        t.DGI[(size_t)r * 3 * M + j] = dgi[j];
        t.DGH[(size_t)r * 3 * M + j] = dgh[j];
    }
    // the message's time encoding: d m[2M + j] = sum_o W_i[o][2M + j] dgi[o]
    for (int j = threadIdx.x; j < T; j += kTrThreads) {
        float acc = 0.0f;
        for (int o2 = 0; o2 < 3 * M; ++o2)
            acc += t.W_i[(size_t)o2 * D + 2 * M + j] * dgi[o2];
        const float sn = time_enc_sin(pw.time_w_rev[j], pw.time_b_rev[j], dt);
        t.TGG[(size_t)r * 2 * T + j] = -sn * (float)dt * acc;
        t.TGG[(size_t)r * 2 * T + T + j] = -sn * acc;
    }
}

// ------------------------------------------------------------------------------------------
struct RowCount {  // rows = min(rows_max, (*dev + add) * mul), or rows_max if dev is NULL
    const int32_t *dev;
    int add, mul, rows_max;
};
__device__ inline int row_count(const RowCount &rc)
{
    if (!rc.dev)
        return rc.rows_max;
    const long long r = ((long long)*rc.dev + rc.add) * rc.mul;
    return r < 0 ? 0 : (r < rc.rows_max ? (int)r : rc.rows_max);
}

// C[Mo x No] += A[rows x Mo]^T B[rows x No]; one wavefront per 32 x 32 block of C and slice of the rows.
// csum != NULL: also csum[Mo] += the column sums of A (the bias gradient that goes with the weight
// gradient: A^T times a column of ones), by the wavefronts of the first block column.
// ridx != NULL: the contraction runs over the rows ridx[0 .. rows) of A and B (each below ridx_max).
__global__ void __launch_bounds__(256) k_gemm_tn(float *C, int ldc, const float *A, int lda, const float *B, int ldb,
                                                 int Mo, int No, RowCount rc, int n_slices, float *csum, const int32_t *ridx,
                                                 int ridx_max)
{
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int tiles_n = (No + 31) / 32, tiles_m = (Mo + 31) / 32;
    const int slice = wave % n_slices;
    const int tile = wave / n_slices;
    if (tile >= tiles_m * tiles_n)
        return;
    const int m0 = (tile / tiles_n) * 32, n0 = (tile % tiles_n) * 32;
    const int rows = row_count(rc);
    const int per = ((rows + n_slices - 1) / n_slices + 3) / 4 * 4;
    const int k_lo = slice * per, k_hi = k_lo + per < rows ? k_lo + per : rows;
    if (k_lo >= k_hi)
        return;
    const bool with_sum = csum != nullptr && n0 == 0;  // (uniform over the wavefront)
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
            bool kin = kk < k_hi;
            int row = kk;
            if (ridx) {
                row = kin ? ridx[kk] : 0;
                kin = kin && row >= 0 && row < ridx_max;
            }
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
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int mm = m0 + 16 * i + 4 * g + v, nn = n0 + 16 * j + c;
                if (mm < Mo && nn < No)
                    atomicAdd(&C[(size_t)mm * ldc + nn], acc[i][j][v]);
            }
    if (with_sum && c == 0) {  // every column of the sum block holds the same value: column 0 adds it
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int mm = m0 + 16 * i + 4 * g + v;
                if (mm < Mo)
                    atomicAdd(&csum[mm], accs[i][v]);
            }
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

__global__ void k_loss_sum(const float *terms, int n, float *loss_out)
{
    __shared__ float red[256];
    float acc = 0.0f;
    for (int i = threadIdx.x; i < n; i += 256)
        acc += terms[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s)
            red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0)
        *loss_out = red[0];
}

__global__ void k_sgd(float *P, const float *G, size_t n, float lr)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        P[i] -= lr * G[i];
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

__global__ void __launch_bounds__(256) k_tr_commit(StepArgs a, int M)
{
    overwrite_memory(a, M, (int)(blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave),
                     (int)(gridDim.x * (blockDim.x / kWave)));
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
    b.KV = take(S * dkv);
    b.KP = take(S * da);
    b.VP = take(S * da);
    b.DKP = take(S * da);
    b.DVP = take(S * da);
    b.CAT = take(U * 2 * E);
    b.DY = take(U * E);
    b.G_ = take(U * E);
    b.DLOGIT = take(U);
    b.LOSS = take(U);
    b.MSG = take(U * D);
    b.DGI = take(U * 3 * M);
    b.DGH = take(U * 3 * M);
    b.TGG = take(U * 2 * T);
    b.n_rows = (int32_t *)take(64);
    b.live = (int32_t *)take(S);
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

static int fwd_lds(const Dims &d)
{
    // doubles [K], ints [2K + 4], floats: s_u, q_in, Qv, kv, KP, VP, sc, o, xcat, h1
    return 8 * d.K + 4 * (2 * d.K + 4) +
           4 * (d.M + 2 * d.da + d.K * d.dkv + 2 * d.K * d.da + d.H * d.K + d.da + d.da + d.M + d.E) + 64;
}
static int bwd_lds(const Dims &d)
{
    // doubles [K], ints [2K + 4], floats: de, dz1, dx, dout, Qv, KP, VP, dKP, dVP, pr, dav, dsv, dQv, dqin, tg
    return 8 * d.K + 4 * (2 * d.K + 4) +
           4 * (2 * d.E + d.da + d.M + 2 * d.da + 4 * d.K * d.da + 3 * d.H * d.K + 2 * d.da + 2 * d.T) + 64;
}
static int gru_bwd_lds(const Dims &d) { return 4 * (d.Dmsg + 12 * d.M); }
static int dec_lds(const Dims &d) { return 4 * (5 * d.E + 8); }

size_t train_workspace_bytes(const Dims &d) { return train_layout(d, nullptr).bytes; }

hipError_t prepare_train(const Dims &d)
{
    hipError_t e = hipFuncSetAttribute((const void *)k_tr_rows_fwd, hipFuncAttributeMaxDynamicSharedMemorySize, fwd_lds(d));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)k_tr_rows_bwd, hipFuncAttributeMaxDynamicSharedMemorySize, bwd_lds(d));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)k_tr_gru_bwd, hipFuncAttributeMaxDynamicSharedMemorySize, gru_bwd_lds(d));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)k_tr_decoder, hipFuncAttributeMaxDynamicSharedMemorySize, dec_lds(d));
    return e;
}

bool train_supported(const Dims &d)
{
    return d.prec == TIG_FP32 && fwd_lds(d) <= 160 * 1024 && bwd_lds(d) <= 160 * 1024 && gru_bwd_lds(d) <= 160 * 1024 &&
           d.K <= kTrThreads;
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
                        float *loss_out, hipStream_t s)
{
    const TrainLayout L = train_layout(d, workspace);
    const TrainDims td = train_dims(d);
    const TrainBufs &b = L.b;
    const PackedWeights pwv = *pw;
    hipError_t e = launch_fill_zero((char *)workspace + L.zero_lo, L.zero_hi - L.zero_lo, s);
    if (e != hipSuccess)
        return e;
    const int B = a.count, R = 3 * B, K = d.K;
    hipLaunchKernelGGL(k_tr_rows_fwd, dim3(R), dim3(kTrThreads), fwd_lds(d), s, a, pwv, td, b);
    hipLaunchKernelGGL(k_tr_decoder, dim3(B), dim3(kTrThreads), dec_lds(d), s, a, td, b);
    hipLaunchKernelGGL(k_tr_rows_bwd, dim3(R), dim3(kTrThreads), bwd_lds(d), s, a, pwv, td, b);
    if (a.msg_count > 0)
        hipLaunchKernelGGL(k_tr_gru_bwd, dim3(2 * a.msg_count), dim3(kTrThreads), gru_bwd_lds(d), s, a, pwv, td, b);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;

    const RowCount rows{b.n_rows, 0, 1, R}, live{b.n_live, 0, 1, R * K}, pairs{nullptr, 0, 1, 2 * B},
        wins{a.n_win, 0, 1, 2 * a.msg_count};
    // weight gradient C += A^T B together with the bias gradient csum += column sums of A
    auto gemm = [&](const float *C, const float *csum, int Mo, int No, const float *A, const float *Bm, const RowCount &rc,
                    int ldb = 0, const int32_t *ridx = nullptr, int ridx_max = 0) {
        const int tiles = ((Mo + 31) / 32) * ((No + 31) / 32);
        // about 3072 wavefronts per contraction: every slice ends in one atomic add per element of its
        // block, so few slices; a slice keeps at least 64 rows
        int n_slices = 3072 / tiles;
        const int most = rc.rows_max / 64;
        n_slices = n_slices > most ? most : n_slices;
        n_slices = n_slices < 1 ? 1 : n_slices;
        const int waves = tiles * n_slices;
        hipLaunchKernelGGL(k_gemm_tn, dim3((waves + 3) / 4), dim3(256), 0, s, (float *)C, No, A, Mo, Bm, ldb ? ldb : No, Mo, No,
                           rc, n_slices, (float *)csum, ridx, ridx_max);
    };
    auto colsum = [&](const float *out, const float *A, int lda, int cols, const RowCount &rc) {
        int n_slices = rc.rows_max / 512;
        n_slices = n_slices < 1 ? 1 : (n_slices > 256 ? 256 : n_slices);
        hipLaunchKernelGGL(k_colsum, dim3((cols + 255) / 256, n_slices), dim3(256), 0, s, (float *)out, A, lda, cols, rc,
                           n_slices);
    };
    const int M = d.M, T = d.T, E = d.E, da = d.da, dkv = d.dkv, D = d.Dmsg;
    // decoder
    gemm(L.g.W_d1, L.g.b_d1, E, 2 * E, b.DY, b.CAT, pairs);
    gemm(L.g.w_d2, L.g.b_d2, 1, E, b.DLOGIT, b.G_, pairs);
    // merge MLP
    gemm(L.g.W_m2, L.g.b_m2, E, E, b.D_EMB, b.H1, rows);
    gemm(L.g.W_m1, L.g.b_m1, E, da + M, b.DZ1, b.X1, rows);
    // attention
    gemm(L.g.W_O, L.g.b_O, da, da, b.D_ATTN, b.O_, rows);
    gemm(L.g.W_Q, L.g.b_Q, da, da, b.DQV, b.QIN, rows);
    gemm(L.g.W_K, L.g.b_K, da, dkv, b.DKP, b.KV, live, 0, b.live, R * K);
    gemm(L.g.W_V, L.g.b_V, da, dkv, b.DVP, b.KV, live, 0, b.live, R * K);
    // time encoding: per-row partial sums [gw | gb]; the two gradients are neighbours in the gradient buffer
    colsum(L.g.time_w, b.TG, 2 * T, 2 * T, rows);
    if (a.msg_count > 0) {
        gemm(L.g.W_i, L.g.b_i, 3 * M, D, b.DGI, b.MSG, wins);
        gemm(L.g.W_h, L.g.b_h, 3 * M, M, b.DGH, b.MSG, wins, D);  // h = the first M columns of the message rows
        colsum(L.g.time_w, b.TGG, 2 * T, 2 * T, wins);
    }
    if (loss_out)
        hipLaunchKernelGGL(k_loss_sum, dim3(1), dim3(256), 0, s, b.LOSS, 2 * B, loss_out);
    // the memory overwrite comes last: the GRU's backward read the memory as the step found it
    if (a.msg_count > 0)
        hipLaunchKernelGGL(k_tr_commit, dim3(32), dim3(256), 0, s, a, M);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    if (lr != 0.0f) {
        hipLaunchKernelGGL(k_sgd, dim3((unsigned)((L.n_params + 255) / 256)), dim3(256), 0, s, L.P, L.G, L.n_params, lr);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
        if ((e = transpose_all(d, L, s)) != hipSuccess)
            return e;
        // the step's own forward pass reads the masters and their transposes; of the prepared weights
        // only the state update's (and the time encoding's) are read by a training step, so only they
        // follow every update; the rest is re-folded when an inference step next needs it
        e = pack_weights(d, L.w, packed, L.pack_scratch, pw, s, kPackGru);
    }
    return e;
}

hipError_t train_refold_embed(const Dims &d, void *workspace, void *packed, PackedWeights *pw, hipStream_t s)
{
    const TrainLayout L = train_layout(d, workspace);
    return pack_weights(d, L.w, packed, L.pack_scratch, pw, s, kPackEmbed);
}

}  // namespace tig
