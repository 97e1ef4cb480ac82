// k_gru: message build and GRU state update (message module, state-update module and memory
// fetch of the paper's Sec. II-C) for the compacted winners of one batch.  gfx950 only.
// The same grid carries, in extra workgroups, work that depends on nothing the GRU produces:
//   - ahead of the embedding launch (a step whose batch was not prepared by the step before):
//     what is left of the query preparation (prepare.h), slots and row references;
//   - as the closing launch of a step (decode.h): the decoder scores and embedding rows of the
//     step's events and the finishing pass of the batch prepared for the next step -- and then
//     the GRU workgroups run for the batch the NEXT step applies (its winners were selected
//     beside the embedding launch), so that step starts with its embedding launch.
// All of these are chains of dependent memory round trips, so they hide each other.
//
// The number of winners is only known on the device (hub nodes make it a small fraction of the
// 2B entries), so the GRU workgroups are a fixed grid that divides the work itself: 16-row tiles
// of winners x slices of the gate columns, as many column slices per tile as keep the grid busy
// (every workgroup streams only its slice of the gate weights; all slices of a tile gather the
// same rows).  One work item (8 wavefronts):
//   1  row descriptors: node, partner, event, event time (dt = t - last_update[node] in step 2)
//   2  message rows [s_self | s_other | Phi(dt) | e] gathered from the batch-START memory into an
//      LDS tile (every element of every row is an independent load: one round of latency)
//   3  gate pre-activations on the matrix cores: the 8 wavefronts are 4 pairs, one wavefront of
//      a pair for the r and z gates, the other for the two halves of the n gate (input part over
//      the whole message, hidden part over s_self); the pairs split the item's column tiles and,
//      when there are fewer column tiles than pairs, the k range of each; partial sums meet in LDS
//   4  h' = (1 - z) n + z h  -> staging rows (memory is overwritten beside the embedding)
// W_hr and W_hz are folded onto the s_self columns of W_ir / W_iz at init (pack.hip).
#include <hip/hip_runtime.h>

#include "decode.h"
#include "kernels_common.h"
#include "prepare.h"

namespace tig {

#ifdef TIG_PHASE_CLOCKS
static __device__ unsigned long long g_phase_clocks[8192 * 8];
extern "C" __attribute__((visibility("default"))) int tig_debug_phase_clocks_gru(unsigned long long *out, int n)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_clocks), sizeof(unsigned long long) * (size_t)n);
}
#endif

namespace {

constexpr int kGruThreads = 512;  // two workgroups per compute unit: the finishing pass runs beside the GRU
constexpr int kGruWaves = kGruThreads / kWave;
constexpr int kPairs = kGruWaves / 2;  // wavefront pairs: (r, z) | n
constexpr int EC = 16;                 // winners per tile

struct GruParams {
    int M, T, F, Dmsg;
    int Kg, Khn, Ng;
    int ldx;       // LDS row stride of the message tile, bytes
    int off_part;  // byte offset of the partial-sum buffer in LDS
    int n_gru;     // GRU workgroups (the first blocks of the grid)
    int cs;        // column slices per tile (any value from 1 to the number of column tiles is correct)
    int n_row_blocks;   // then: blocks that fix row references of this step's queries (grid-stride over the rows)
    int n_slot_blocks;  // then: blocks that fix their slots, one entry per thread
                        // then: the blocks of the closing work (decode.h)
    int32_t *clear;     // a counter block 0 sets to 0, or NULL
};

// The batch whose winners the GRU workgroups apply.
struct GruJob {
    int64_t first_eid;
    int32_t count;      // 0: nothing to apply
    const WinDesc *win;
    const int32_t *n_win;
};

// acc1 += A x W1[nt]^T over W1's k-blocks [kb_lo, kb_hi) and acc2 += A x W2[nt]^T over W2's
// k-blocks [kb_lo, min(kb_hi, w2_kblocks)): both weight streams are loaded DEPTH blocks ahead and
// share the A operand.
template <int PREC, int DEPTH>
__device__ inline void tile_gemm2(floatx4 &acc1, floatx4 &acc2, const char *A, int lda, const void *W1,
                                  const void *W2, int w1_kblocks, int w2_kblocks, int kb_lo, int kb_hi, int nt)
{
    using P = Prec<PREC>;
    using frag = typename P::frag;
    const int lane = lane_id();
    const size_t w1 = (size_t)nt * w1_kblocks * kWave + lane;
    const size_t w2 = (size_t)nt * w2_kblocks * kWave + lane;
    const char *ap = A + (size_t)(lane & 15) * lda;
    const int g = lane >> 4;
    const int kb_hi2 = kb_hi < w2_kblocks ? kb_hi : w2_kblocks;
    for (int kb = kb_lo; kb < kb_hi; kb += DEPTH) {
        frag b1[DEPTH], b2[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            if (kb + u < kb_hi)
                b1[u] = P::load_w(W1, w1 + (size_t)(kb + u) * kWave);
            if (kb + u < kb_hi2)
                b2[u] = P::load_w(W2, w2 + (size_t)(kb + u) * kWave);
        }
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kb_hi) {
                const frag afrag = P::load_a(ap, kb + u, g);
                P::mma(acc1, afrag, b1[u]);
                if (kb + u < kb_hi2)
                    P::mma(acc2, afrag, b2[u]);
            }
    }
}

template <int PREC>
__global__ void __launch_bounds__(kGruThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))  // 128 registers: two workgroups per unit
k_gru(StepArgs a, GruJob gj, PackedWeights w, GruParams g, DecodeParams dp)
{
    TIG_MARK(0);
    if (blockIdx.x == 0 && threadIdx.x == 0 && g.clear)
        *g.clear = 0;
    if ((int)blockIdx.x >= g.n_gru) {
        int x = (int)blockIdx.x - g.n_gru;
        if (x < g.n_row_blocks) {  // finishing pass of this step's query preparation
            int n_u = *a.qs.n_u;
            n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
            for (int row = x * kGruWaves + wave_id(); row < n_u; row += g.n_row_blocks * kGruWaves)
                finish_row(ref_ctx(a), a.qs, dp.K, row);
        } else if ((x -= g.n_row_blocks) < g.n_slot_blocks) {
            const int i = x * kGruThreads + (int)threadIdx.x;
            if (i < 2 * a.count)
                finish_slots(a.qs, i, 2 * a.count);
        } else {
            closing_block(a, w, dp, x - g.n_slot_blocks, kGruWaves);
        }
        TIG_MARK(1);
        return;
    }
    using P = Prec<PREC>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *row_i = (int *)smem;                  // [EC] entry 2b + role
    int *row_u = row_i + EC;                   // [EC] node
    int *row_o = row_u + EC;                   // [EC] partner
    int *row_e = row_o + EC;                   // [EC] event id - first_eid
    double *row_t = (double *)(row_e + EC);    // [EC] event time
    char *X = smem + EC * 24;                  // [EC rows x ldx bytes]
    float *part = (float *)(smem + g.off_part);  // [2 halves][kPairs][2 streams][16 x 16]
    double *tw_tab = (double *)(part + 2 * kPairs * 2 * 256);  // [T][2] time-encoding (w_rev, b_rev)

    const int lane = lane_id();
    const int wave = wave_id();

    // the work: tiles x column slices.  The slice count comes with the launch, so the first item's
    // descriptors are requested together with the winner count (slots beyond the count hold stale
    // descriptors of earlier batches or nothing: they are only used below the count).
    const int n_ct = g.Ng / 16;
    const int cs = g.cs;
    const int tpp = (n_ct + cs - 1) / cs;  // column tiles per item
    WinDesc d_first;
    {
        const int r = ((int)blockIdx.x / cs) * EC + (int)threadIdx.x;
        if (threadIdx.x < EC && r < 2 * gj.count)
            d_first = gj.win[r];
    }
    int n_win = *gj.n_win;
    n_win = n_win < 2 * gj.count ? n_win : 2 * gj.count;  // (a list never holds more than the batch's entries)
    const int tiles = (n_win + EC - 1) / EC;
    if (tiles == 0)
        return;
    const int items = tiles * cs;
    const int kblocks = g.Kg / P::KB;
    const int kblocks_hn = g.Khn / P::KB;
    for (int j = threadIdx.x; j < g.T; j += kGruThreads) {  // (visible after the first barrier below)
        tw_tab[2 * j] = w.time_w_rev[j];
        tw_tab[2 * j + 1] = w.time_b_rev[j];
    }

    for (int item = (int)blockIdx.x; item < items; item += g.n_gru) {
        // 1. this item's slice of the compacted winner list
        const int r0 = (item / cs) * EC;
        const int ct_lo = (item % cs) * tpp;
        const int ct_hi = n_ct < ct_lo + tpp ? n_ct : ct_lo + tpp;
        const int n_rows = n_win - r0 < EC ? n_win - r0 : EC;
        if (threadIdx.x < EC) {
            const int r = threadIdx.x;
            int i = 0, u = 0, o = 0, b = 0;
            double t = 0.0;
            if (r < n_rows) {
                const WinDesc d0 = item == (int)blockIdx.x ? d_first : gj.win[r0 + r];
                i = d0.entry;
                u = d0.node;
                o = d0.other;
                b = d0.b;
                t = d0.t;
            }
            row_i[r] = i;
            row_u[r] = u;
            row_o[r] = o;
            row_e[r] = b;
            row_t[r] = t;
        }
        __syncthreads();
        TIG_MARK(1);

        // 2. message rows from batch-start memory; rows beyond n_rows are zero.  One wavefront per
        //    row, lanes along the row (no index arithmetic per element); the loads of both rows of a
        //    wavefront are requested before the first element is converted and stored.
        {
            constexpr int kRowsPerWave = EC / kGruWaves;
            constexpr int kAhead = 6;  // 384 elements of a message row per pass
            for (int base = 0; base < g.Kg; base += kWave * kAhead) {
                float v[kRowsPerWave][kAhead];
                double dt[kRowsPerWave];
#pragma unroll
                for (int i = 0; i < kRowsPerWave; ++i) {
                    const int r = wave + i * kGruWaves;
                    const bool live = r < n_rows;
                    const int u = row_u[r], o = row_o[r];
                    const float *self = a.mem + (size_t)u * g.M;
                    const float *other = a.mem + (size_t)o * g.M;
                    const float *feat = a.edge_feat + (size_t)(gj.first_eid + row_e[r]) * g.F;
                    dt[i] = live ? row_t[r] - a.lu[u] : 0.0;  // since the node's last update
#pragma unroll
                    for (int k = 0; k < kAhead; ++k) {
                        const int j = base + lane + kWave * k;
                        v[i][k] = 0.0f;
                        if (live && j < g.Dmsg) {
                            if (j < g.M)
                                v[i][k] = self[j];
                            else if (j < 2 * g.M)
                                v[i][k] = other[j - g.M];
                            else if (j >= 2 * g.M + g.T)
                                v[i][k] = feat[j - 2 * g.M - g.T];
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < kRowsPerWave; ++i) {
                    const int r = wave + i * kGruWaves;
                    const bool live = r < n_rows;
#pragma unroll
                    for (int k = 0; k < kAhead; ++k) {
                        const int j = base + lane + kWave * k;
                        if (j < g.Kg) {
                            float x = v[i][k];
                            if (live && j >= 2 * g.M && j < 2 * g.M + g.T)
                                x = time_enc(tw_tab[2 * (j - 2 * g.M)], tw_tab[2 * (j - 2 * g.M) + 1], dt[i]);
                            P::store_a(X + (size_t)r * g.ldx, j, x);
                        }
                    }
                }
            }
        }
        __syncthreads();
        TIG_MARK(2);

        // 3. + 4. gates.  A round covers up to kPairs column tiles; with fewer, the pairs also split k.
        for (int base = ct_lo; base < ct_hi; base += kPairs) {
            const int cts = ct_hi - base < kPairs ? ct_hi - base : kPairs;  // column tiles of this round
            const int ksplit = cts == 1 ? 4 : (cts == 2 ? 2 : 1);
            const int pair = wave % kPairs;
            const int half = wave / kPairs;  // 0: r and z gates, 1: n gate
            const int ctl = pair / ksplit;   // column tile of the round
            const int ks = pair % ksplit;    // k slice
            const bool on = ctl < cts;
            // gate biases of the element this thread finishes below, requested with the weights
            float pb[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if ((int)threadIdx.x < cts * 256) {
                const int col = (base + ((int)threadIdx.x >> 8)) * 16 + ((int)threadIdx.x & 15);
                pb[0] = w.gru_br[col];
                pb[1] = w.gru_bz[col];
                pb[2] = w.gru_bin[col];
                pb[3] = w.gru_bhn[col];
            }
            floatx4 acc1 = floatx4{0, 0, 0, 0}, acc2 = floatx4{0, 0, 0, 0};
            if (on) {
                const int ct = base + ctl;
                const int per = (kblocks + ksplit - 1) / ksplit;
                const int kb_lo = ks * per;
                const int kb_hi = kblocks < kb_lo + per ? kblocks : kb_lo + per;
                if (half == 0)
                    tile_gemm2<PREC, 3>(acc1, acc2, X, g.ldx, w.gru_Wr, w.gru_Wz, kblocks, kblocks, kb_lo, kb_hi, ct);
                else  // input part over the whole message, hidden part over s_self (the first Khn k's)
                    tile_gemm2<PREC, 3>(acc1, acc2, X, g.ldx, w.gru_Win, w.gru_Whn, kblocks, kblocks_hn, kb_lo,
                                        kb_hi, ct);
            }
            {
                float *p1 = part + (size_t)((half * kPairs + pair) * 2) * 256;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = (4 * (lane >> 4) + v) * 16 + (lane & 15);
                    p1[e] = acc1[v];
                    p1[256 + e] = acc2[v];
                }
            }
            __syncthreads();
            TIG_MARK(3);
            for (int idx = threadIdx.x; idx < cts * 256; idx += kGruThreads) {
                const int ctl2 = idx >> 8, e = idx & 255;
                const int row = e >> 4, col = (base + ctl2) * 16 + (e & 15);
                if (row < n_rows && col < g.M) {
                    float sr = 0.0f, sz = 0.0f, sin_ = 0.0f, shn = 0.0f;
                    for (int k2 = 0; k2 < ksplit; ++k2) {
                        const float *q0 = part + (size_t)((ctl2 * ksplit + k2) * 2) * 256;
                        const float *q1 = part + (size_t)((kPairs + ctl2 * ksplit + k2) * 2) * 256;
                        sr += q0[e];
                        sz += q0[256 + e];
                        sin_ += q1[e];
                        shn += q1[256 + e];
                    }
                    const bool pre = idx < kGruThreads;  // the preloaded biases are this element's
                    const float br = pre ? pb[0] : w.gru_br[col], bz = pre ? pb[1] : w.gru_bz[col];
                    const float bin = pre ? pb[2] : w.gru_bin[col], bhn = pre ? pb[3] : w.gru_bhn[col];
                    const float r = 1.0f / (1.0f + __expf(-(sr + br)));
                    const float z = 1.0f / (1.0f + __expf(-(sz + bz)));
                    const float h = P::load_elem(X + (size_t)row * g.ldx, col);  // s_self
                    const float x = sin_ + bin + r * (shn + bhn);
                    const float e2 = __expf(2.0f * x);          // tanh(x) = 1 - 2 / (e^{2x} + 1)
                    const float n = 1.0f - 2.0f / (e2 + 1.0f);
                    a.staging[(size_t)row_i[row] * g.M + col] = (1.0f - z) * n + z * h;
                    if (a.gru_gates) {  // (uniform) a training step keeps the gates for its backward pass
                        float *go = a.gru_gates + (size_t)(r0 + row) * 4 * g.M + col;
                        go[0] = r;
                        go[g.M] = z;
                        go[2 * g.M] = n;
                        go[3 * g.M] = shn + bhn;
                    }
                }
            }
            __syncthreads();  // the partial sums (and, after the last round, the tile) are reused
        }
    }
    TIG_MARK(4);
}

GruParams gru_params(const Dims &d)
{
    GruParams g;
    g.M = d.M;
    g.T = d.T;
    g.F = d.F;
    g.Dmsg = d.Dmsg;
    g.Kg = d.Kg;
    g.Khn = d.Khn;
    g.Ng = d.Ng;
    g.ldx = lds_row_bytes(d.Kg);
    g.off_part = (EC * 24 + EC * g.ldx + 15) / 16 * 16;
    g.n_gru = 0;
    g.cs = 1;
    g.n_row_blocks = 0;
    g.n_slot_blocks = 0;
    g.clear = nullptr;
    return g;
}

const void *gru_kernel(const Dims &d)
{
    return d.prec == TIG_BF16_MFMA ? (const void *)k_gru<TIG_BF16_MFMA> : (const void *)k_gru<TIG_FP32>;
}

// GRU workgroups and column slices for a batch of `count` events with about `wins_est` winners.
void size_gru(const Dims &d, const LaunchPlan &plan, int count, int wins_est, GruParams *g)
{
    // one workgroup per compute unit, but no more than the work of the largest possible winner
    // count (every entry a winner, every column tile its own item); none if nothing is applied
    const int cus = plan.num_cus > 0 ? plan.num_cus : 256;
    const int max_items = (2 * count + EC - 1) / EC * (d.Ng / 16);
    g->n_gru = max_items < cus ? max_items : cus;
    // as many column slices per tile as keep the GRU workgroups busy at the winner count recent
    // steps had (hub nodes make it a small share of the 2 * count entries)
    const int most = 2 * count;
    const int wins = wins_est > 0 && wins_est < most ? wins_est : most;
    const int tiles = (wins + EC - 1) / EC > 0 ? (wins + EC - 1) / EC : 1;
    const int n_ct = d.Ng / 16;
    int cs = g->n_gru / tiles;
    cs = cs < 1 ? 1 : (cs > n_ct ? n_ct : cs);
    const int tpp = (n_ct + cs - 1) / cs;
    g->cs = (n_ct + tpp - 1) / tpp;
}

DecodeParams no_closing(const Dims &d)
{
    DecodeParams p;
    p.M = d.M;
    p.E = d.E;
    p.Ep = d.Ep;
    p.K = d.K;
    p.n_event_blocks = p.n_expand_blocks = p.n_fin_row_blocks = p.n_fin_slot_blocks = 0;
    return p;
}

}  // namespace

int gru_lds_bytes(const Dims &d)
{
    return gru_params(d).off_part + 2 * kPairs * 2 * 256 * 4 + d.T * 16;
}

hipError_t prepare_gru(const Dims &d, const LaunchPlan &plan)
{
    return hipFuncSetAttribute(gru_kernel(d), hipFuncAttributeMaxDynamicSharedMemorySize, gru_lds_bytes(d));
}

// Ahead of the embedding launch: the GRU of the batch this step applies and, if asked for, the
// finishing pass of this step's queries.
hipError_t launch_gru(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                      hipStream_t s, bool gru_work)
{
    StepArgs aa = a;
    PackedWeights ww = pw;
    GruParams g = gru_params(d);
    GruJob gj = {a.msg_first_eid, gru_work ? a.msg_count : 0, a.win, a.n_win};
    DecodeParams dp = no_closing(d);
    size_gru(d, plan, gj.count, a.wins_est, &g);
    if (a.finish_here) {
        const int cus = plan.num_cus > 0 ? plan.num_cus : 256;
        const int rows = 2 * a.count;  // at most; a wavefront takes several rows if there are many
        g.n_row_blocks = (rows + kGruWaves - 1) / kGruWaves;
        if (g.n_row_blocks > 2 * cus)
            g.n_row_blocks = 2 * cus;
        g.n_slot_blocks = (2 * a.count + kGruThreads - 1) / kGruThreads;
    }
    const int blocks = g.n_gru + g.n_row_blocks + g.n_slot_blocks;
    if (blocks == 0)
        return hipSuccess;  // nothing to apply, nothing to finish
    void *args[] = {&aa, &gj, &ww, &g, &dp};
    return hipLaunchKernel(gru_kernel(d), dim3(blocks), dim3(kGruThreads), args, (size_t)gru_lds_bytes(d), s);
}

// The closing launch of a step: scores and embedding rows of its events, inspection outputs, the
// finishing pass of the batch prepared ahead; its own query set's counter is cleared for the
// set's next preparation; and, if ahead.count > 0, the GRU of the batch the next step applies.
hipError_t launch_closing(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                          const GruAhead &ahead, hipStream_t s, bool events)
{
    StepArgs aa = a;
    PackedWeights ww = pw;
    GruParams g = gru_params(d);
    GruJob gj = {ahead.first_eid, ahead.count, ahead.win, ahead.n_win};
    if (ahead.count > 0)
        size_gru(d, plan, ahead.count, a.wins_est, &g);
    g.clear = a.qs.n_u;
    DecodeParams p = no_closing(d);
    p.n_event_blocks = events ? (a.count + kGruWaves - 1) / kGruWaves : 0;  // (a training step decodes itself)
    const bool expand = wants_inspection(a);
    p.n_expand_blocks = expand ? (a.roles * a.count + kGruWaves - 1) / kGruWaves : 0;
    if (a.fin_count > 0) {
        p.n_fin_row_blocks = (2 * a.fin_count + kGruWaves - 1) / kGruWaves;
        if (p.n_fin_row_blocks > 128)
            p.n_fin_row_blocks = 128;
        p.n_fin_slot_blocks = (2 * a.fin_count + kGruThreads - 1) / kGruThreads;
    }
    int blocks = g.n_gru + p.n_event_blocks + p.n_expand_blocks + p.n_fin_row_blocks + p.n_fin_slot_blocks;
    blocks = blocks > 0 ? blocks : 1;  // (block 0 clears the counter whatever else there is to do)
    void *args[] = {&aa, &gj, &ww, &g, &p};
    return hipLaunchKernel(gru_kernel(d), dim3(blocks), dim3(kGruThreads), args, (size_t)gru_lds_bytes(d), s);
}

}  // namespace tig
