// k_gru: message build and GRU state update (message module, state-update module and memory
// fetch of the paper's Sec. II-C) for the compacted winners of one batch.  gfx950 only.
// The same launch carries the neighbour lookup of every query in extra workgroups (lookup.h):
// it depends on nothing the GRU produces, and both are chains of dependent memory round trips,
// so they hide each other's latency.
//
// One workgroup (16 wavefronts) takes 16*MT winners:
//   1  row descriptors: node, partner, event, event time (dt = t - last_update[node] in step 2)
//   2  message rows [s_self | s_other | Phi(dt) | e] gathered from the batch-START memory into an
//      LDS tile (every element of every row is an independent load: one round of latency)
//   3  gate pre-activations on the matrix cores.  Per 16-column tile two wavefronts work side by
//      side: one computes the r and z gates, the other the two halves of the n gate (input part
//      over the whole message, hidden part over s_self); r and z cross over through LDS
//   4  h' = (1 - z) n + z h  -> staging rows (memory is overwritten by k_commit afterwards)
// W_hr and W_hz are folded onto the s_self columns of W_ir / W_iz at init (pack.hip).
#include <hip/hip_runtime.h>

#include "kernels_common.h"
#include "lookup.h"

namespace tig {

#ifdef TIG_PHASE_CLOCKS
static __device__ unsigned long long g_phase_clocks[8192 * 8];
extern "C" __attribute__((visibility("default"))) int tig_debug_phase_clocks_gru(unsigned long long *out, int n)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_clocks), sizeof(unsigned long long) * (size_t)n);
}
#endif

namespace {

constexpr int kGruThreads = 1024;
constexpr int kGruWaves = kGruThreads / kWave;

struct GruParams {
    int M, T, F, Dmsg;
    int Kg, Khn, Ng;
    int ldx;     // LDS row stride of the message tile, bytes
    int off_rz;  // byte offset of the r/z exchange buffer in LDS
    int cs;      // workgroups per row tile: each takes `tpp` consecutive 16-column tiles of the gates
    int tpp;
};

// acc1 += A x W1[nt]^T and acc2 += A x W2[nt]^T over k-blocks [0, kblocks): both weight streams
// are loaded DEPTH blocks ahead and share the A operand.
template <int PREC, int MT, int DEPTH>
__device__ inline void tile_gemm2(floatx4 (&acc1)[MT], floatx4 (&acc2)[MT], const char *A, int lda,
                                  const void *W1, const void *W2, int w1_kblocks, int w2_kblocks,
                                  int kblocks, int nt)
{
    using P = Prec<PREC>;
    using frag = typename P::frag;
    const int lane = lane_id();
    const size_t w1 = (size_t)nt * w1_kblocks * kWave + lane;
    const size_t w2 = (size_t)nt * w2_kblocks * kWave + lane;
    const char *ap = A + (size_t)(lane & 15) * lda;
    const int g = lane >> 4;
    for (int kb = 0; kb < kblocks; kb += DEPTH) {
        frag b1[DEPTH], b2[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks) {
                b1[u] = P::load_w(W1, w1 + (size_t)(kb + u) * kWave);
                b2[u] = P::load_w(W2, w2 + (size_t)(kb + u) * kWave);
            }
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, kb + u, g);
                    P::mma(acc1[mt], afrag, b1[u]);
                    P::mma(acc2[mt], afrag, b2[u]);
                }
            }
    }
}

template <int PREC, int MT>
__global__ void __launch_bounds__(kGruThreads)
k_gru(StepArgs a, PackedWeights w, GruParams g, int n_gru_blocks, int K)
{
    TIG_MARK(0);
    if ((int)blockIdx.x >= n_gru_blocks) {  // lookup workgroup: one query per wavefront
        const int q = ((int)blockIdx.x - n_gru_blocks) * kGruWaves + wave_id();
        if (q < a.roles * a.count)
            nbr_lookup_wave(a, K, q);
        TIG_MARK(1);
        return;
    }
    using P = Prec<PREC>;
    constexpr int EC = 16 * MT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *row_i = (int *)smem;                  // [EC] entry 2b + role
    int *row_u = row_i + EC;                   // [EC] node
    int *row_o = row_u + EC;                   // [EC] partner
    int *row_e = row_o + EC;                   // [EC] event id - first_eid
    double *row_t = (double *)(row_e + EC);    // [EC] event time
    char *X = smem + EC * 24;                  // [EC rows x ldx bytes]
    float *rz = (float *)(smem + g.off_rz);    // [EC][Ng][2]

    const int lane = lane_id();
    const int wave = wave_id();

    // 1. this block's slice of the compacted winner list (descriptor and count are read in the
    //    same round trip; slots beyond the count hold stale but in-range descriptors).  The g.cs
    //    workgroups of a row tile gather the same rows and split the gate columns: each streams
    //    only its share of the gate weights.
    const int r0 = ((int)blockIdx.x / g.cs) * EC;
    const int ct_lo = ((int)blockIdx.x % g.cs) * g.tpp;
    WinDesc d0;
    if (threadIdx.x < EC)
        d0 = a.win[r0 + threadIdx.x];
    const int n_win = *a.n_win;
    if (r0 >= n_win)
        return;
    const int n_rows = n_win - r0 < EC ? n_win - r0 : EC;
    if (threadIdx.x < EC) {
        const int r = threadIdx.x;
        int i = 0, u = 0, o = 0, b = 0;
        double t = 0.0;
        if (r < n_rows) {
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
    //    row, lanes along the row (no index arithmetic per element); all loads of a row are
    //    requested before its first element is converted and stored.
    for (int r = wave; r < EC; r += kGruWaves) {
        const bool live = r < n_rows;
        const int u = row_u[r], o = row_o[r];
        const float *self = a.mem + (size_t)u * g.M;
        const float *other = a.mem + (size_t)o * g.M;
        const float *feat = a.edge_feat + (size_t)(a.msg_first_eid + row_e[r]) * g.F;
        const double lu = live ? a.lu[u] : 0.0;
        constexpr int kAhead = 8;  // 512 elements of a message row per pass
        for (int base = 0; base < g.Kg; base += kWave * kAhead) {
            float v[kAhead];
            double tw[kAhead], tb[kAhead];
#pragma unroll
            for (int k = 0; k < kAhead; ++k) {
                const int j = base + lane + kWave * k;
                v[k] = 0.0f;
                tw[k] = tb[k] = 0.0;
                if (live && j < g.Dmsg) {
                    if (j < g.M)
                        v[k] = self[j];
                    else if (j < 2 * g.M)
                        v[k] = other[j - g.M];
                    else if (j < 2 * g.M + g.T) {
                        tw[k] = w.time_w_rev[j - 2 * g.M];
                        tb[k] = w.time_b_rev[j - 2 * g.M];
                    } else
                        v[k] = feat[j - 2 * g.M - g.T];
                }
            }
            const double dt = row_t[r] - lu;  // since the node's last update
#pragma unroll
            for (int k = 0; k < kAhead; ++k) {
                const int j = base + lane + kWave * k;
                if (j < g.Kg) {
                    float x = v[k];
                    if (live && j >= 2 * g.M && j < 2 * g.M + g.T)
                        x = time_enc(tw[k], tb[k], dt);
                    P::store_a(X + (size_t)r * g.ldx, j, x);
                }
            }
        }
    }
    __syncthreads();
    TIG_MARK(2);

    // 3. + 4. gates
    const int kblocks = g.Kg / P::KB;
    const int kblocks_hn = g.Khn / P::KB;
    const int n_ct = g.Ng / 16 < ct_lo + g.tpp ? g.Ng / 16 : ct_lo + g.tpp;  // end of this block's tiles
    constexpr int kPairs = kGruWaves / 2;  // column tiles per round
    for (int base = ct_lo; base < n_ct; base += kPairs) {
        const int ct = base + (wave % kPairs);
        const int half = wave / kPairs;  // 0: r and z gates, 1: n gate
        const bool on = ct < n_ct;
        floatx4 acc1[MT], acc2[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc1[mt] = floatx4{0, 0, 0, 0};
            acc2[mt] = floatx4{0, 0, 0, 0};
        }
        const int col = ct * 16 + (lane & 15);
        if (on) {
            if (half == 0) {
                tile_gemm2<PREC, MT, 5>(acc1, acc2, X, g.ldx, w.gru_Wr, w.gru_Wz, kblocks, kblocks, kblocks, ct);
                const float br = w.gru_br[col], bz = w.gru_bz[col];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = mt * 16 + 4 * (lane >> 4) + v;
                        float *o2 = rz + ((size_t)row * g.Ng + col) * 2;
                        o2[0] = 1.0f / (1.0f + __expf(-(acc1[mt][v] + br)));
                        o2[1] = 1.0f / (1.0f + __expf(-(acc2[mt][v] + bz)));
                    }
            } else {
                // input part over the whole message, hidden part over s_self (the first Khn k's)
                tile_gemm2<PREC, MT, 5>(acc1, acc2, X, g.ldx, w.gru_Win, w.gru_Whn, kblocks, kblocks_hn,
                                        kblocks_hn, ct);
                tile_gemm<PREC, MT, 6>(acc1, X, g.ldx, kblocks_hn, w.gru_Win, kblocks, kblocks_hn,
                                       kblocks - kblocks_hn, ct);
            }
        }
        __syncthreads();
        TIG_MARK(3);
        if (on && half == 1 && col < g.M) {
            const float bin = w.gru_bin[col], bhn = w.gru_bhn[col];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = mt * 16 + 4 * (lane >> 4) + v;
                    if (row < n_rows) {
                        const float *i2 = rz + ((size_t)row * g.Ng + col) * 2;
                        const float r = i2[0], z = i2[1];
                        const float h = P::load_elem(X + (size_t)row * g.ldx, col);  // s_self
                        const float x = acc1[mt][v] + bin + r * (acc2[mt][v] + bhn);
                        const float e2 = __expf(2.0f * x);          // tanh(x) = 1 - 2 / (e^{2x} + 1)
                        const float n = 1.0f - 2.0f / (e2 + 1.0f);
                        a.staging[(size_t)row_i[row] * g.M + col] = (1.0f - z) * n + z * h;
                    }
                }
        }
        __syncthreads();  // rz is reused by the next round
    }
    TIG_MARK(4);
}

GruParams gru_params(const Dims &d, int mt)
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
    g.off_rz = (16 * mt * 24 + 16 * mt * g.ldx + 15) / 16 * 16;
    g.cs = 1;
    g.tpp = d.Ng / 16;
    return g;
}

template <int PREC>
const void *pick_mt(int mt)
{
    return mt == 1 ? (const void *)k_gru<PREC, 1> : (const void *)k_gru<PREC, 2>;
}

const void *gru_kernel(const Dims &d, int mt)
{
    return d.prec == TIG_BF16_MFMA ? pick_mt<TIG_BF16_MFMA>(mt) : pick_mt<TIG_FP32>(mt);
}

}  // namespace

int gru_lds_bytes(const Dims &d, int mt)
{
    const GruParams g = gru_params(d, mt);
    return g.off_rz + 16 * mt * d.Ng * 2 * 4;
}

hipError_t prepare_gru(const Dims &d, const LaunchPlan &plan)
{
    for (int mt = 1; mt <= plan.gru_mt; ++mt) {
        const hipError_t e = hipFuncSetAttribute(gru_kernel(d, mt), hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 gru_lds_bytes(d, mt));
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

hipError_t launch_gru(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                      hipStream_t s)
{
    StepArgs aa = a;
    PackedWeights ww = pw;
    const int entries = 2 * a.msg_count;  // 0 in a deferred step with nothing to apply: lookup only
    // Column split.  Every workgroup streams the gate weights of its columns from L2, which bounds
    // its run time, so when the 16-row tiles do not fill the device the columns of a tile are
    // split over as many workgroups as it takes at once.  Only the tiles below the winner count
    // do any work.  (32-row tiles with halved columns measured slower at large batches.)
    const int cus = plan.num_cus > 0 ? plan.num_cus : 256;
    const int mt = 1;
    GruParams g = gru_params(d, mt);
    const int tiles = (entries + 16 * mt - 1) / (16 * mt);
    const int n_ct = d.Ng / 16;
    int cs = tiles > 0 ? 2 * cus / tiles : 1;
    cs = cs < 1 ? 1 : (cs > n_ct ? n_ct : cs);
    g.tpp = (n_ct + cs - 1) / cs;
    g.cs = (n_ct + g.tpp - 1) / g.tpp;
    int n_gru_blocks = tiles * g.cs;
    int K = d.K;
    const int n_lookup_blocks = (a.roles * a.count + kGruWaves - 1) / kGruWaves;
    void *args[] = {&aa, &ww, &g, &n_gru_blocks, &K};
    return hipLaunchKernel(gru_kernel(d, mt), dim3(n_gru_blocks + n_lookup_blocks), dim3(kGruThreads), args,
                           (size_t)gru_lds_bytes(d, mt), s);
}

}  // namespace tig
