// k_embed: temporal attention embedding and merge MLP of one batch step (embedding module f of
// the paper's Sec. II-C) and the first decoder layer (decoder g), fused in one kernel, for the
// DISTINCT queries (node, t) of the batch (prepare.h).  gfx950 only.
//
// One workgroup (16 wavefronts) takes 16*MT rows of the query set at a time and keeps every
// intermediate of those rows in LDS:
//   A  row descriptors: row reference of the node's state, neighbour count, time; s_u
//   B  folded query  q~ = A1 s_u + a1                        (matrix cores; fp32 result)
//   C  per row: gather the K neighbour rows [Phi(t - t_k) | s_v | e], scores <q~_h, kv_k>,
//      softmax over the filled slots, kvbar_h = sum_k a_k kv_k   (vector ALU, one wavefront/row)
//   D  h1 = relu(P kvbar + R s_u + c)                         (matrix cores, k split over 2 waves)
//   E  from h1 in one pass: emb = W_m2 h1 + b_m2 and both halves of decoder layer 1,
//      W_d1[:, :E] emb and W_d1[:, E:] emb (merge layer 2 folded into the decoder weights)
//      -> per-row arrays in global memory; the decode kernel pairs them up per event
// State rows are read through row references: the memory table, or the staged GRU output for a
// node this step updates -- so the memory overwrite M <- s_i(t) itself runs in a few extra
// workgroups of this launch.
// The negatives of the batch arrive with the call; the wavefront that takes a negative's row in
// phase C looks up its neighbours first (a chain of dependent reads that hides behind the other
// wavefronts' rows).
// The projections W_Q, W_K, W_V, W_O and the first merge layer are folded into A1 and P at init
// (pack.hip), which removes the per-neighbour key/value projections.
// The number of rows is known on the device only: the grid has a tile for every 16*MT rows the
// batch could have, and the tiles beyond the actual row count return at once.  Row r of tile p is
// query row p + (number of tiles in use) * r, which spreads the heavy rows (sources /
// destinations, first in the set) over all tiles.  Workgroups beyond the tiles and the memory
// overwrite prepare the batch expected next: one selects its last-message winners, the others
// merge and look up its queries.
#include <type_traits>
#include <hip/hip_runtime.h>

#include "kernels_common.h"
#include "prepare.h"
#include "winners.h"

namespace tig {

#ifdef TIG_PHASE_CLOCKS
__device__ unsigned long long g_phase_clocks[8192 * 8];
extern "C" __attribute__((visibility("default"))) int tig_debug_phase_clocks(unsigned long long *out, int n)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_clocks), sizeof(unsigned long long) * (size_t)n);
}
#endif

namespace {

// Wavefronts per workgroup: 16 (128 registers per lane) unless the query and accumulator rows of
// all heads need 64 registers per lane or more, then 8 (256 registers per lane).
template <int NPL, int H>
struct EmbedShape {
    static constexpr int kThreads = (NPL >= 8 && H >= 4) ? 512 : 1024;
    static constexpr int kWaves = kThreads / kWave;
};

struct EmbedParams {
    int M, T, F, E, K;
    int dkv, dkvp, Mq, N1, K2, Ep, Ek;
    int row_bytes;  // LDS bytes per query row of the main buffer: [q~ / kvbar (N1) | s_u (Mq)]
    int ld1;        // row stride of the E-wide buffers, bytes
    int off_h1, off_meta;  // byte offsets in LDS
    int n_tiles;    // workgroups that take row tiles
    int n_commit;   // then: workgroups of the memory overwrite; the ones beyond prepare the next batch
    // bit n set: register n of a key/value row (dims 64 n .. 64 n + 63 of [Phi | s_v | e]) holds
    // at least one dim of the time encoding / of the neighbour's memory / of the edge feature
    int phi_regs, mem_regs, feat_regs;
};

// Key/value row shapes compiled in (0: taken from the launch parameters).  With a fixed shape
// every "which register holds which segment" decision of phase C is made by the compiler.
template <int SHAPE>
struct RowShape {
    static constexpr bool kFixed = false;
    static constexpr int T = 0, M = 0, F = 0, H = 0;
};
template <>
struct RowShape<1> {  // memory, time encoding and embedding of 100 dims, 8-dim edge features
    static constexpr bool kFixed = true;
    static constexpr int T = 100, M = 100, F = 8, H = 2;
};
template <>
struct RowShape<2> {  // 172-dim memory and edge features, 100-dim time encoding
    static constexpr bool kFixed = true;
    static constexpr int T = 100, M = 172, F = 172, H = 2;
};

template <>
struct RowShape<3> {  // 100-dim memory and time encoding, 16-dim edge features
    static constexpr bool kFixed = true;
    static constexpr int T = 100, M = 100, F = 16, H = 2;
};

// bit n set: register n (dims 64 n .. 64 n + 63) holds at least one dim of [lo, hi)
constexpr int regs_touching(int lo, int hi, int dims)
{
    int m = 0;
    for (int n = 0; n * kWave < dims; ++n)
        if (n * kWave + kWave > lo && n * kWave < hi)
            m |= 1 << n;
    return m;
}

template <int PREC, int MT, int NPL, int H, int SHAPE>
__global__ void __launch_bounds__((EmbedShape<NPL, H>::kThreads))
k_embed(StepArgs a, PackedWeights w, EmbedParams p)
{
    using P = Prec<PREC>;
    using SH = RowShape<SHAPE>;
    // segment sizes and segment-to-register maps of a key/value row, as phase C uses them
    const int cT = SH::kFixed ? SH::T : p.T, cM = SH::kFixed ? SH::M : p.M, cF = SH::kFixed ? SH::F : p.F;
    // d_kv padded to whole k-blocks of the precision's matrix-core operand
    const int cDkvp = SH::kFixed ? (SH::T + SH::M + SH::F + P::KB - 1) / P::KB * P::KB : p.dkvp;
    const int phi_regs = SH::kFixed ? regs_touching(0, SH::T, kWave * NPL) : p.phi_regs;
    const int mem_regs = SH::kFixed ? regs_touching(SH::T, SH::T + SH::M, kWave * NPL) : p.mem_regs;
    const int feat_regs =
        SH::kFixed ? regs_touching(SH::T + SH::M, SH::T + SH::M + SH::F, kWave * NPL) : p.feat_regs;
    constexpr int kEmbedThreads = EmbedShape<NPL, H>::kThreads;
    constexpr int kEmbedWaves = EmbedShape<NPL, H>::kWaves;
    constexpr int ROWS = 16 * MT;
    constexpr int KC = NPL >= 8 ? 5 : (NPL == 4 ? 10 : 16);      // neighbour rows in flight
    constexpr int NPHI = NPL;  // registers that may hold time-encoding dims (T <= 64 * NPL)
    extern __shared__ __attribute__((aligned(16))) char smem[];
    if ((int)blockIdx.x >= p.n_tiles) {
        int x = (int)blockIdx.x - p.n_tiles;
        if (x < p.n_commit) {
            overwrite_memory(a, p.M, x * kEmbedWaves + wave_id(), p.n_commit * kEmbedWaves);
            return;
        }
        x -= p.n_commit;
        // The workgroups beyond, on compute units this launch leaves idle (launched only with
        // 1024 threads): last-message selection and query preparation for a later step.
        if constexpr (kEmbedThreads == kScatterThreads) {
            TIG_MARK(0);
            if (x == 0 && threadIdx.x == 0 && a.rows_seen) {
                // hints for the host (stores to its memory take a while: from a workgroup that ends
                // long before the launch does)
                a.rows_seen[0] = *a.qs.n_u + (a.roles == 3 ? a.count : 0);  // (a hint: not clamped)
                if (a.msg_count > 0)
                    a.rows_seen[1] = *a.n_win;
            }
            if (a.sel.count > 0) {
                if (x == 0) {
                    winners_block(a, a.sel, smem);
                    TIG_MARK(7);
                    return;
                }
                --x;
            }
            if (a.ded.count > 0 && x < a.ded.n_wgs)
                dedup_block(a, a.ded, p.K, x, smem);
            TIG_MARK(7);
        }
        return;
    }
    char *rowbuf = smem;
    char *h1buf = smem + p.off_h1;
    int *row_q = (int *)(smem + p.off_meta);  // [ROWS] row of the query set or -1
    int *row_cnt = row_q + ROWS;              // [ROWS]
    int *row_ref = row_cnt + ROWS;            // [ROWS] row reference of the node's own state
    double *row_t = (double *)(row_ref + ROWS);   // [ROWS] query time
    double *tw_tab = row_t + ROWS;                // [T][2] time-encoding (w_rev, b_rev)
    int *next_row = (int *)(tw_tab + 2 * p.T);    // [1] row counter of phase C
    int *row_todo = next_row + 4;                 // [ROWS] 1: a negative whose neighbours phase C looks up

    const int lane = lane_id();
    const int wave = wave_id();
    const int mem_off = 4 * p.N1;
    int n_u = *a.qs.n_u;  // distinct source / destination queries; the negatives' rows follow at 2 * count
    n_u = n_u < 2 * a.count ? n_u : 2 * a.count;
    const int neg_row0 = 2 * a.count;
    const int n_rows = n_u + (a.roles == 3 ? a.count : 0);
    const int n_passes = (n_rows + ROWS - 1) / ROWS;
    // a row reference that is neither a memory row nor a staged row of the applied batch reads as none
    auto checked_ref = [&](int32_t ref) -> int32_t {
        const bool ok = ref >= 0 ? (int64_t)ref < a.num_nodes : (ref != kRefNone && ~ref < 2 * a.msg_count);
        return ok ? ref : kRefNone;
    };

    const int pass = (int)blockIdx.x;
    if (pass >= n_passes)
        return;  // fewer distinct queries than the grid was sized for
    TIG_MARK(0);
    // ---- A. query rows ------------------------------------------------------------------------
    // Every load of this phase is unconditional (an index that does not apply is replaced by one that
    // is valid, and the value dropped): a load inside a branch is waited for at the end of the branch,
    // and the phase would be a chain of round trips instead of two.
    double tw_w = 0.0, tw_b = 0.0;
    if ((int)threadIdx.x < p.T) {  // (T <= 512 <= the threads of the workgroup)
        tw_w = w.time_w_rev[threadIdx.x];
        tw_b = w.time_b_rev[threadIdx.x];
    }
    if (threadIdx.x < ROWS) {
        const int r = threadIdx.x;
        const int x = pass + n_passes * r;
        const bool is_rep = x < n_u, is_neg = !is_rep && x < n_rows;
        // a negative: node and time from the call.  For now the reference is the node's own memory
        // row; the gather below checks whether this step updates the node.
        const int b = is_neg ? x - n_u : 0, qq = is_rep ? x : 0;
        const int32_t *ref_p = is_neg ? a.neg + b : a.qs.self_ref + qq;
        const double *t_p = is_neg ? a.ts + a.first_eid + b : a.qs.t + qq;
        int32_t ref = *ref_p;
        double t = *t_p;
        int cnt = a.qs.cnt[qq];
        int q = is_rep ? x : neg_row0 + b;
        if (is_neg) {
            ref = ref >= 0 ? ref : kRefNone;
            cnt = 0;
        }
        if (!is_rep && !is_neg) {
            q = -1;
            ref = kRefNone;
            cnt = 0;
            t = 0.0;
        }
        row_q[r] = q;
        row_ref[r] = checked_ref(ref);
        row_cnt[r] = cnt < p.K ? cnt : p.K;
        row_t[r] = t;
        row_todo[r] = 0;
    }
    if (threadIdx.x == 0)
        *next_row = 0;
    if ((int)threadIdx.x < p.T) {
        tw_tab[2 * threadIdx.x] = tw_w;
        tw_tab[2 * threadIdx.x + 1] = tw_b;
    }
    __syncthreads();
    {
        // one wavefront per row, lanes along the row (no index arithmetic per element); the loads
        // of all of a wavefront's rows are requested before the first is stored.  For a negative
        // the same round trip fetches the node's key (is its state row a staged one?) and the
        // bounds of its adjacency list: a node without history, the usual case in a large graph,
        // needs no lookup; the others are looked up by the wavefront that takes the row in phase C.
        constexpr int kRowsPerWave = (ROWS + kEmbedWaves - 1) / kEmbedWaves;
        constexpr int kAhead = 2;  // 128 floats of a row per lane pair of loads
        // A row is read through a buffer descriptor in scalar registers (base = the row, extent = the
        // row, or nothing for a missing reference): lanes beyond the row read 0, no load sits inside a
        // branch (the compiler waits for such a load at the end of its branch: a round trip per load),
        // and a wavefront's rows are all in flight together.
        float v[kRowsPerWave][kAhead];
        __amdgpu_buffer_rsrc_t src_row[kRowsPerWave];
        int32_t neg_u[kRowsPerWave], neg_ref[kRowsPerWave];  // node / checked row reference of a negative, else kRefNone
        unsigned long long neg_key[kRowsPerWave];
        int64_t deg_lo[kRowsPerWave], deg_hi[kRowsPerWave];
        const RefCtx rc = ref_ctx(a);
        auto row_rsrc = [&](int32_t ref) -> __amdgpu_buffer_rsrc_t {  // ref: the same in every lane
            const float *row = ref >= 0 ? a.mem + (size_t)ref * p.M : a.staging + (size_t)(ref == kRefNone ? 0 : ~ref) * p.M;
            return __builtin_amdgcn_make_buffer_rsrc((void *)row, 0, ref == kRefNone ? 0 : p.M * 4, kBufferFlags);
        };
        // (with no batch applied the key array may not exist: any readable 8 bytes stand in)
        const unsigned long long *key_tab = rc.count > 0 ? rc.key : (const unsigned long long *)a.indptr;
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            const int r = wave + i * kEmbedWaves;
            const int ref = __builtin_amdgcn_readfirstlane(r < ROWS ? row_ref[r] : kRefNone);
            const bool is_neg = r < ROWS && __builtin_amdgcn_readfirstlane(row_q[r < ROWS ? r : 0]) >= neg_row0;
            src_row[i] = row_rsrc(ref);
#pragma unroll
            for (int u = 0; u < kAhead; ++u)
                v[i][u] = buffer_load_f32(src_row[i], (uint32_t)(lane + kWave * u) * 4u);
            neg_u[i] = is_neg ? ref : kRefNone;
            const int32_t nu = neg_u[i] != kRefNone ? neg_u[i] : 0;  // (a valid node id: checked above)
            const unsigned long long got_key = key_tab[nu];
            const int64_t got_lo = a.indptr[nu], got_hi = a.indptr[nu + 1];
            neg_key[i] = neg_u[i] != kRefNone && rc.count > 0 ? got_key : 0ull;
            deg_lo[i] = neg_u[i] != kRefNone ? got_lo : 0;
            deg_hi[i] = neg_u[i] != kRefNone ? got_hi : 0;
        }
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i)
            neg_ref[i] = neg_u[i] != kRefNone ? checked_ref(ref_of_key(rc, neg_u[i], neg_key[i])) : kRefNone;
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            const int r = wave + i * kEmbedWaves;
            if (r < ROWS) {
                if (neg_ref[i] != neg_u[i]) {  // a negative this step updates: the staged row instead (uniform)
                    src_row[i] = row_rsrc(__builtin_amdgcn_readfirstlane(neg_ref[i]));
#pragma unroll
                    for (int u = 0; u < kAhead; ++u)
                        v[i][u] = buffer_load_f32(src_row[i], (uint32_t)(lane + kWave * u) * 4u);
                    if (lane == 0)
                        row_ref[r] = neg_ref[i];
                }
                if (deg_hi[i] > deg_lo[i] && lane == 0)
                    row_todo[r] = 1;  // (a negative: only those have a degree here)
                char *dst = rowbuf + (size_t)r * p.row_bytes + mem_off;
#pragma unroll
                for (int u = 0; u < kAhead; ++u)
                    if (lane + kWave * u < p.Mq)
                        P::store_a(dst, lane + kWave * u, v[i][u]);
                for (int j = lane + kWave * kAhead; j < p.Mq; j += kWave)  // rows beyond 128 floats
                    P::store_a(dst, j, buffer_load_f32(src_row[i], (uint32_t)j * 4u));
            }
        }
    }
    __syncthreads();

    // Phase C hands its rows out through an LDS counter, heaviest first (sources / destinations come
    // first in the set), so that wavefronts with short rows take more of them.  The neighbour table
    // of a row (slot k lives in lane k) is fetched when the row before it is started; the first
    // row's table is requested here, a phase early.
    // Order: the negatives that still need their lookup first (the longest chain of dependent
    // reads), then the other rows by index.
    static_assert(ROWS < 64, "one mask bit per row");
    const unsigned long long todo_mask = __ballot(lane < ROWS && row_todo[lane < ROWS ? lane : 0] != 0);
    const unsigned long long rest_mask = ~todo_mask & ((1ull << ROWS) - 1ull);
    const int n_todo = __popcll(todo_mask);
    auto grab = [&]() -> int {
        int pos = 0;
        if (lane == 0)
            pos = atomicAdd(next_row, 1);
        pos = __builtin_amdgcn_readfirstlane(pos);
        if (pos >= ROWS)
            return ROWS;
        const unsigned long long m = pos < n_todo ? todo_mask : rest_mask;
        const int k = pos < n_todo ? pos : pos - n_todo;
        const bool hit = ((m >> lane) & 1ull) != 0ull && __popcll(m & ((1ull << lane) - 1ull)) == k;
        const unsigned long long h = __ballot(hit);  // exactly one lane: the k-th set bit of m
        return h != 0ull ? __ffsll((long long)h) - 1 : ROWS;
    };
    auto load_nb = [&](int r, int32_t &v, int32_t &e, double &dt) {
        v = 0;
        e = 0;
        dt = 0.0;
        if (r < ROWS) {
            const int q = row_q[r];
            if (q >= 0 && q < neg_row0 && lane < row_cnt[r]) {
                v = a.qs.ref[(size_t)q * p.K + lane];  // row reference of the neighbour's state
                e = a.qs.eid[(size_t)q * p.K + lane];
                dt = row_t[r] - a.qs.ts[(size_t)q * p.K + lane];
            }
        }
    };
    // what a gather can safely be pointed at: a valid row reference and event id (anything else, which
    // only a corrupted table could hold, reads row 0)
    auto safe_slot = [&](int32_t &v, int32_t &e) {
        v = checked_ref(v) == kRefNone ? 0 : v;
        e = e >= 0 ? e : 0;
    };
    int r = grab();
    int32_t nb_v2, nb_e2;
    double nb_dt2;
    load_nb(r, nb_v2, nb_e2, nb_dt2);

    TIG_MARK(1);
    // ---- B. folded query: q~ = A1 s_u + a1  (fp32, [H x dkvp] per row) -----------------------
    {
        const int ntB = p.N1 / 16, kbB = p.Mq / P::KB, a_kb0 = p.N1 / P::KB;
        auto put = [&](const floatx4 (&acc)[MT], int nt, float bias) {
            const int col = nt * 16 + (lane & 15);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = mt * 16 + 4 * (lane >> 4) + v;
                    ((float *)(rowbuf + (size_t)row * p.row_bytes))[col] = acc[mt][v] + bias;
                }
        };
        // two output tiles per pass where the wavefront has two: they share the reads of s_u
        for (int nt = wave; nt < ntB; nt += 2 * kEmbedWaves) {
            const int nt2 = nt + kEmbedWaves;
            floatx4 acc1[MT], acc2[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc1[mt] = floatx4{0, 0, 0, 0};
                acc2[mt] = floatx4{0, 0, 0, 0};
            }
            const float bias1 = w.emb_a1[nt * 16 + (lane & 15)];
            if (nt2 < ntB) {
                const float bias2 = w.emb_a1[nt2 * 16 + (lane & 15)];
                tile_gemm_two<PREC, MT, 2>(acc1, acc2, rowbuf, p.row_bytes, a_kb0, w.emb_A1, kbB, kbB, nt, nt2);
                put(acc1, nt, bias1);
                put(acc2, nt2, bias2);
            } else {
                tile_gemm<PREC, MT, 4>(acc1, rowbuf, p.row_bytes, a_kb0, w.emb_A1, kbB, 0, kbB, nt);
                put(acc1, nt, bias1);
            }
        }
    }
    __syncthreads();

    TIG_MARK(2);
    // ---- C. attention over the neighbours ------------------------------------------------------
    {
        // Per-lane view of a key/value row, kernel order [Phi (T) | s_v (M) | e (F) | 0]: the lane
        // owns dims j = lane + 64 n.  (Time encoding first: its lanes are densely packed.)
        // Neighbour rows are read through buffer descriptors built per row in scalar registers
        // (base = the row, extent = the row): a lane whose dim lies outside the row reads 0, so
        // the gathers need no per-lane predication and no per-lane 64-bit address.
        uint32_t offm[NPL];  // byte offset of the lane's dim inside the memory row, or out of range
#pragma unroll
        for (int n = 0; n < NPL; ++n) {
            const int jj = lane + kWave * n - cT;
            offm[n] = jj < 0 ? 0xffffffffu : (uint32_t)jj * 4u;
        }
        const uint32_t m_bytes = (uint32_t)cM * 4u, f_bytes = (uint32_t)cF * 4u;
        // time-encoding parameters of the lane's Phi dims, kept in registers for compiled-in shapes
        double tw_reg[NPHI], tb_reg[NPHI];
#pragma unroll
        for (int n = 0; n < NPHI; ++n) {
            tw_reg[n] = 0.0;
            tb_reg[n] = 0.0;
            if (SH::kFixed && ((phi_regs >> n) & 1)) {
                const int j = lane + kWave * n < cT ? lane + kWave * n : 0;
                tw_reg[n] = tw_tab[2 * j];
                tb_reg[n] = tw_tab[2 * j + 1];
            }
        }
        int32_t nb_v1, nb_e1;
        double nb_dt1;
#pragma unroll 1
        while (r < ROWS) {
            int32_t nb_vc = nb_v2, nb_ec = nb_e2;
            double nb_dtc = nb_dt2;
            const int r_next = grab();
            load_nb(r_next, nb_v1, nb_e1, nb_dt1);
            const int r_cur = r;
            r = r_next;
            nb_v2 = nb_v1;
            nb_e2 = nb_e1;
            nb_dt2 = nb_dt1;
            const int q_cur = __builtin_amdgcn_readfirstlane(row_q[r_cur]);
            if (q_cur < 0)
                continue;
            int cnt;
            if (q_cur >= neg_row0 && !__builtin_amdgcn_readfirstlane(row_todo[r_cur])) {
                // a negative without history: its (empty) row of the query set is written here, where
                // nothing waits for the stores
                if (lane < p.K) {
                    const size_t o = (size_t)q_cur * p.K + lane;
                    a.qs.nbr[o] = -1;
                    a.qs.eid[o] = -1;
                    a.qs.ts[o] = 0.0;
                    a.qs.ref[o] = kRefNone;
                }
                if (lane == 0) {
                    const int32_t u = a.neg[q_cur - neg_row0];
                    a.qs.cnt[q_cur] = 0;
                    a.qs.node[q_cur] = u >= 0 && (int64_t)u < a.num_nodes ? u : -1;
                    a.qs.t[q_cur] = row_t[r_cur];
                }
                cnt = 0;
            } else if (q_cur >= neg_row0) {
                // a negative: its neighbours are looked up now (slot k lands in lane k)
                double ts_k;
                cnt = finish_negative(a, p.K, q_cur - neg_row0, nb_vc, nb_ec, ts_k);
                cnt = __builtin_amdgcn_readfirstlane(cnt);
                nb_dtc = row_t[r_cur] - ts_k;
                if (lane == 0)
                    row_cnt[r_cur] = cnt;  // phase D picks the bias by it
            } else {
                cnt = __builtin_amdgcn_readfirstlane(row_cnt[r_cur]);
            }
            safe_slot(nb_vc, nb_ec);
            const float *qrow = (const float *)(rowbuf + (size_t)r_cur * p.row_bytes);
            char *arow = rowbuf + (size_t)r_cur * p.row_bytes;
            float qv[H][NPL], accv[H][NPL];
            float mx[H], den[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                mx[h] = -INFINITY;
                den[h] = 0.0f;
#pragma unroll
                for (int n = 0; n < NPL; ++n) {
                    const int j = lane + kWave * n;
                    qv[h][n] = j < cDkvp ? qrow[h * cDkvp + j] : 0.0f;
                    accv[h][n] = 0.0f;
                }
            }
            // One chunk of up to KC neighbour slots starting at slot c0.  FULL: the row has exactly
            // KC neighbours (the usual case once the adjacency is deep), so no slot is conditional
            // and there is no earlier chunk to merge with.
            auto chunk = [&](const int c0, auto full_tag) {
                constexpr bool FULL = decltype(full_tag)::value;
                constexpr bool VEC = FULL && H % 2 == 0 && KC % 2 == 0 && KC <= 32;  // softmax across lanes
                float S[H / 2 > 0 ? H / 2 : 1];
#pragma unroll
                for (int h = 0; h < H / 2; ++h)
                    S[h] = -INFINITY;
                float raw[KC][NPL];
                float mix[KC];  // edge-feature lanes of the one register that also holds s_v dims
                // issue every gather of the chunk before using any of them
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
                    const int k = c0 + kk;
                    mix[kk] = 0.0f;
                    if (FULL || k < cnt) {  // scalar
                        const int32_t v = __builtin_amdgcn_readlane(nb_vc, k & 63);
                        const int32_t e = __builtin_amdgcn_readlane(nb_ec, k & 63);
                        const float *vrow = v >= 0 ? a.mem + (size_t)v * cM : a.staging + (size_t)(~v) * cM;
                        const __amdgpu_buffer_rsrc_t rm =
                            __builtin_amdgcn_make_buffer_rsrc((void *)vrow, 0, (int)m_bytes, kBufferFlags);
                        const __amdgpu_buffer_rsrc_t re = __builtin_amdgcn_make_buffer_rsrc(
                            (void *)(a.edge_feat + (size_t)e * cF), 0, (int)f_bytes, kBufferFlags);
#pragma unroll
                        for (int n = 0; n < NPL; ++n) {
                            const bool has_m = (mem_regs >> n) & 1, has_e = (feat_regs >> n) & 1;  // scalar
                            float x = 0.0f;
                            if (has_m)
                                x = buffer_load_f32(rm, offm[n]);
                            else if (has_e)
                                x = buffer_load_f32(re, offm[n] - m_bytes);
                            if (has_m && has_e)  // at most one register: the one with dim T + M inside
                                mix[kk] = buffer_load_f32(re, offm[n] - m_bytes);
                            raw[kk][n] = x;
                        }
                    }
                }
                // time encoding of t - t_k and the lane's share of every score; slots in pairs so
                // that the wavefront sums of a pair interleave
                float sc[KC][H];
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
#pragma unroll
                    for (int h = 0; h < H; ++h)
                        sc[kk][h] = -INFINITY;
                }
#pragma unroll
                for (int k2 = 0; k2 < KC; k2 += 2) {
                    if (FULL || c0 + k2 < cnt) {  // scalar
                        float part[2][H];
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const int kk = k2 + u < KC ? k2 + u : KC - 1;
                            const int k = c0 + kk;
#pragma unroll
                            for (int h = 0; h < H; ++h)
                                part[u][h] = 0.0f;
                            if (k2 + u < KC && (FULL || k < cnt)) {  // scalar
                                const double dt = readlane_f64(nb_dtc, k & 63);
#pragma unroll
                                for (int n = 0; n < NPL; ++n) {
                                    if ((mem_regs & feat_regs) >> n & 1)  // scalar
                                        raw[kk][n] += mix[kk];  // disjoint lanes; the other side read 0
                                }
#pragma unroll
                                for (int n = 0; n < NPHI; ++n) {
                                    if ((phi_regs >> n) & 1) {  // scalar: this register holds Phi dims
                                        const int j = lane + kWave * n < cT ? lane + kWave * n : 0;
                                        float ph = SH::kFixed ? time_enc(tw_reg[n], tb_reg[n], dt)
                                                              : time_enc(tw_tab[2 * j], tw_tab[2 * j + 1], dt);
                                        if (SH::kFixed && kWave * n + kWave > cT) {
                                            // every lane evaluates, the others keep their dim: no
                                            // branch, so the whole chunk stays one scheduling region
                                            asm volatile("" : "+v"(ph));
                                            raw[kk][n] = lane + kWave * n < cT ? ph : raw[kk][n];
                                        } else if (lane + kWave * n < cT) {
                                            raw[kk][n] = ph;
                                        }
                                    }
                                }
#pragma unroll
                                for (int h = 0; h < H; ++h) {
#pragma unroll
                                    for (int n = 0; n < NPL; ++n)
                                        part[u][h] += qv[h][n] * raw[kk][n];
                                }
                            }
                        }
                        if constexpr (H % 2 == 0) {
                            // four wavefront sums (2 slots x 2 heads) for the price of one: the
                            // half- and quarter-wave swaps fold them into the four 16-lane rows of
                            // one register, which the row shifts then sum
#pragma unroll
                            for (int h = 0; h < H; h += 2) {
                                const float z = wave_sum_four(part[0][h], part[1][h], part[0][h + 1], part[1][h + 1]);
                                if constexpr (VEC) {
                                    // lane 15 - (pair index) of each row collects the row's sum: pair
                                    // i shifts in from the right and leaves the i lanes before it
                                    // alone (the lanes to the left are cleared after the last pair)
                                    S[h / 2] = row_shl_keep(S[h / 2], z, k2 / 2);
                                    continue;
                                }
#pragma unroll
                                for (int u = 0; u < 2; ++u) {
                                    if (k2 + u < KC && (FULL || c0 + k2 + u < cnt)) {  // scalar
                                        const int kk = k2 + u < KC ? k2 + u : KC - 1;
                                        sc[kk][h] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(z), 15 + 16 * u));
                                        sc[kk][h + 1] =
                                            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(z), 47 + 16 * u));
                                    }
                                }
                            }
                        } else {
                            // wavefront sums of the pair, one DPP step at a time across its 2H values
                            // (see wave_sum_uniform for the step sequence)
#define TIG_DPP_STEP(CTRL, ROWS_)                                          \
    _Pragma("unroll") for (int u = 0; u < 2; ++u)                          \
        _Pragma("unroll") for (int h = 0; h < H; ++h)                      \
            part[u][h] += dpp_or_zero<CTRL, ROWS_, 0xf>(part[u][h]);
                            TIG_DPP_STEP(0x111, 0xf)
                            TIG_DPP_STEP(0x112, 0xf)
                            TIG_DPP_STEP(0x114, 0xf)
                            TIG_DPP_STEP(0x118, 0xf)
#undef TIG_DPP_STEP
#pragma unroll
                            for (int h = 0; h < H; ++h)
                                add_row_bcasts(part[0][h], part[1][h]);
#pragma unroll
                            for (int u = 0; u < 2; ++u) {
                                if (k2 + u < KC && (FULL || c0 + k2 + u < cnt)) {  // scalar
#pragma unroll
                                    for (int h = 0; h < H; ++h)
                                        sc[k2 + u < KC ? k2 + u : KC - 1][h] =
                                            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(part[u][h]), 63));
                                }
                            }
                        }
                    }
                }
                if constexpr (VEC) {
                    // softmax with one score per lane: register S[h/2] holds, in its rows 0..3, the
                    // scores of (even slots, head h), (odd slots, head h), (even, h+1), (odd, h+1);
                    // slot pair i sits in lane 15 - i of the row, every other lane is -inf
#pragma unroll
                    for (int h = 0; h < H; h += 2) {
                        S[h / 2] = (lane & 15) >= 16 - KC / 2 ? S[h / 2] : -INFINITY;
                        float m = row_max_all(S[h / 2]);
                        max_row_bcast15(m);  // rows 1 and 3 now hold the maximum of their head
                        const float m0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 31));
                        const float m1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 63));
                        const float e = __expf(S[h / 2] - (lane < 32 ? m0 : m1));
                        float sum = row_sum_all(e);
                        add_row_bcast15(sum);
                        den[h] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sum), 31));
                        den[h + 1] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sum), 63));
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk) {
                            const int src = 16 * (kk & 1) + 15 - kk / 2;
                            const float p0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(e), src));
                            const float p1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(e), 32 + src));
#pragma unroll
                            for (int n = 0; n < NPL; ++n) {
                                accv[h][n] += p0 * raw[kk][n];
                                accv[h + 1][n] += p1 * raw[kk][n];
                            }
                        }
                    }
                    return;
                }
                // softmax across the chunk, merged with earlier chunks by rescaling
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    float mnew = mx[h];
#pragma unroll
                    for (int kk = 0; kk < KC; ++kk)
                        mnew = fmaxf(mnew, sc[kk][h]);
                    float dsum = 0.0f;
                    if constexpr (!FULL) {
                        const float corr = __expf(mx[h] - mnew);  // first chunk: exp(-inf) = 0
                        dsum = den[h] * corr;
#pragma unroll
                        for (int n = 0; n < NPL; ++n)
                            accv[h][n] *= corr;
                    }
#pragma unroll
                    for (int kk = 0; kk < KC; ++kk) {
                        if (FULL || c0 + kk < cnt) {  // scalar
                            const float pk = __expf(sc[kk][h] - mnew);
                            dsum += pk;
#pragma unroll
                            for (int n = 0; n < NPL; ++n)
                                accv[h][n] += pk * raw[kk][n];
                        }
                    }
                    den[h] = dsum;
                    mx[h] = mnew;
                }
            };
            if (cnt == KC) {
                chunk(0, std::true_type{});
            } else {
                for (int c0 = 0; c0 < cnt; c0 += KC)
                    chunk(c0, std::false_type{});
            }
            // kvbar overwrites q~ in place (as matrix-core operand elements)
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float inv = cnt > 0 ? __builtin_amdgcn_rcpf(den[h]) : 0.0f;  // den >= 1; 1 ulp
#pragma unroll
                for (int n = 0; n < NPL; ++n) {
                    const int j = lane + kWave * n;
                    if (j < cDkvp)
                        P::store_a(arow, h * cDkvp + j, accv[h][n] * inv);
                }
            }
        }
    }
    __syncthreads();

    TIG_MARK(3);
    // ---- D. merge layer 1: h1 = relu(P kvbar + R s_u + c)   (c0 when there is no neighbour) ---
    // The row [kvbar | s_u] is one contiguous K2-deep operand.  The k range is split over two
    // wavefronts per output tile when that fills more of the workgroup; the upper half hands its
    // partial sums over through LDS (the h1 buffer, not yet written).
    {
        const int n_tiles = p.Ep / 16;
        const int kbT = p.K2 / P::KB;
        const int ksplit = (2 * n_tiles <= kEmbedWaves && kbT >= 8) ? 2 : 1;
        const int kb_half = (kbT + ksplit - 1) / ksplit;
        float *red = (float *)h1buf;  // [ROWS][ld1/4] partial sums of the upper k half
        floatx4 acc[MT];
        int my_nt = -1, my_ks = 0;
        for (int base = 0; base < n_tiles * ksplit; base += kEmbedWaves) {  // at most one round if split
            const int unit = base + wave;
            const bool on = unit < n_tiles * ksplit;
            my_nt = on ? unit % n_tiles : -1;
            my_ks = on ? unit / n_tiles : 0;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = floatx4{0, 0, 0, 0};
            float c = 0.0f, c0 = 0.0f;  // requested with the first weight operands, used in the epilogue
            if (on) {
                if (my_ks == 0) {
                    c = w.emb_c[my_nt * 16 + (lane & 15)];
                    c0 = w.emb_c0[my_nt * 16 + (lane & 15)];
                }
                const int kb0 = my_ks * kb_half;
                const int nkb = (kbT - kb0) < kb_half ? (kbT - kb0) : kb_half;
                tile_gemm<PREC, MT, (MT <= 2 ? 5 : 4)>(acc, rowbuf, p.row_bytes, kb0, w.emb_PR, kbT, kb0, nkb, my_nt);
            }
            if (ksplit == 2) {
                if (on && my_ks == 1) {
                    const int col = my_nt * 16 + (lane & 15);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int row = mt * 16 + 4 * (lane >> 4) + v;
                            red[(size_t)row * (p.ld1 / 4) + col] = acc[mt][v];
                        }
                }
                __syncthreads();
            }
            if (on && my_ks == 0) {
                const int col = my_nt * 16 + (lane & 15);
                float part[MT][4];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = mt * 16 + 4 * (lane >> 4) + v;
                        part[mt][v] = ksplit == 2 ? red[(size_t)row * (p.ld1 / 4) + col] : 0.0f;
                    }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = mt * 16 + 4 * (lane >> 4) + v;
                        const float x = acc[mt][v] + part[mt][v] + (row_cnt[row] > 0 ? c : c0);
                        P::store_a(h1buf + (size_t)row * p.ld1, col, fmaxf(x, 0.0f));
                    }
            }
        }
    }
    // k-depth padding of the E-wide buffers (columns Ep..Ek-1)
    for (int idx = threadIdx.x; idx < ROWS * (p.Ek - p.Ep); idx += kEmbedThreads) {
        const int row = idx / (p.Ek - p.Ep), col = p.Ep + idx % (p.Ek - p.Ep);
        P::store_a(h1buf + (size_t)row * p.ld1, col, 0.0f);
    }
    __syncthreads();

    TIG_MARK(4);
    // ---- E. from h1: emb = W_m2 h1 + b_m2, and decoder layer 1 split by operand, W_a emb and
    // W_b emb, through the decoder weights folded with merge layer 2 -> per-row arrays in global
    // memory.  3 * Ep / 16 output tiles; a wavefront takes two at a time where it has two, which
    // share the reads of h1.
    {
        const int nE = p.Ep / 16, kbE = p.Ek / P::KB;
        const int n_out = 3 * nE;
        auto put = [&](const floatx4 (&acc)[MT], int ot) {
            const int grp = ot / nE;  // 0: embedding, 1: source half, 2: second-operand half
            const int col = (ot - grp * nE) * 16 + (lane & 15);
            const float bias = grp == 0 ? w.emb_bm2[col] : 0.0f;
            float *dst = grp == 0 ? a.emb_u : (grp == 1 ? a.dec_a : a.dec_b);
            const int ld = grp == 0 ? p.E : p.Ep;
            if (grp == 0 && col >= p.E)
                return;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = mt * 16 + 4 * (lane >> 4) + v;
                    const int q = row_q[row];
                    if (q >= 0)
                        dst[(size_t)q * ld + col] = acc[mt][v] + bias;
                }
        };
        auto weights_of = [&](int ot) -> const void * { return ot < nE ? w.emb_Wm2 : w.dec_WF; };
        auto tile_of = [&](int ot) -> int { return ot < nE ? ot : ot - nE; };
        for (int ot = wave; ot < n_out; ot += 2 * kEmbedWaves) {
            const int ot2 = ot + kEmbedWaves;
            floatx4 acc1[MT], acc2[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc1[mt] = floatx4{0, 0, 0, 0};
                acc2[mt] = floatx4{0, 0, 0, 0};
            }
            if (ot2 < n_out) {
                tile_gemm_pair<PREC, MT, 4>(acc1, acc2, h1buf, p.ld1, weights_of(ot), weights_of(ot2), kbE,
                                            tile_of(ot), tile_of(ot2));
                put(acc1, ot);
                put(acc2, ot2);
            } else {
                tile_gemm<PREC, MT, 4>(acc1, h1buf, p.ld1, 0, weights_of(ot), kbE, 0, kbE, tile_of(ot));
                put(acc1, ot);
            }
        }
    }
    TIG_MARK(5);
}

// ------------------------------------------------------------------------------------------
// host side

EmbedParams embed_params(const Dims &d, int mt)
{
    EmbedParams p;
    p.M = d.M;
    p.T = d.T;
    p.F = d.F;
    p.E = d.E;
    p.K = d.K;
    p.dkv = d.dkv;
    p.dkvp = d.dkvp;
    p.Mq = d.Mq;
    p.N1 = d.N1;
    p.K2 = d.K2;
    p.Ep = d.Ep;
    p.Ek = d.Ek;
    const int rows = 16 * mt;
    p.row_bytes = lds_row_bytes(d.N1 + d.Mq);
    p.ld1 = lds_row_bytes(d.Ek);
    p.off_h1 = (rows * p.row_bytes + 15) / 16 * 16;
    p.off_meta = p.off_h1 + rows * p.ld1;
    p.n_tiles = 0;
    p.n_commit = 0;
    p.phi_regs = p.mem_regs = p.feat_regs = 0;
    for (int n = 0; n * kWave < d.dkvp; ++n) {
        const int lo = n * kWave, hi = lo + kWave;
        if (lo < d.T)
            p.phi_regs |= 1 << n;
        if (hi > d.T && lo < d.T + d.M)
            p.mem_regs |= 1 << n;
        if (hi > d.T + d.M && lo < d.T + d.M + d.F)
            p.feat_regs |= 1 << n;
    }
    return p;
}

int npl_for(const Dims &d)
{
    const int need = (d.dkvp + 63) / 64;
    int npl = 1;
    while (npl < need)
        npl *= 2;
    return npl;
}

// must agree with EmbedShape (heads other than 1 and 2 run the 4-head kernels)
int embed_threads(const Dims &d) { return npl_for(d) >= 8 && d.H > 2 ? 512 : 1024; }

template <int PREC, int MT, int NPL>
const void *pick_h(int H)
{
    switch (H) {
    case 1: return (const void *)k_embed<PREC, MT, NPL, 1, 0>;
    case 2: return (const void *)k_embed<PREC, MT, NPL, 2, 0>;
    default: return (const void *)k_embed<PREC, MT, NPL, 4, 0>;
    }
}

constexpr int npl_of_dims(int dims)
{
    int npl = 1;
    while (npl * kWave < dims)
        npl *= 2;
    return npl;
}

template <int PREC, int SHAPE>
const void *pick_fixed(int mt)
{
    using SH = RowShape<SHAPE>;
    constexpr int NPL = npl_of_dims(SH::T + SH::M + SH::F);
    switch (mt) {
    case 1: return (const void *)k_embed<PREC, 1, NPL, SH::H, SHAPE>;
    case 2: return (const void *)k_embed<PREC, 2, NPL, SH::H, SHAPE>;
    default: return (const void *)k_embed<PREC, 3, NPL, SH::H, SHAPE>;
    }
}

template <int SHAPE>
bool shape_is(const Dims &d)
{
    using SH = RowShape<SHAPE>;
    return d.T == SH::T && d.M == SH::M && d.F == SH::F && d.H == SH::H;
}

template <int PREC, int MT>
const void *pick_npl(int npl, int H)
{
    switch (npl) {
    case 1: return pick_h<PREC, MT, 1>(H);
    case 2: return pick_h<PREC, MT, 2>(H);
    case 4: return pick_h<PREC, MT, 4>(H);
    default: return pick_h<PREC, MT, 8>(H);
    }
}

template <int PREC>
const void *pick_mt(int mt, int npl, int H)
{
    switch (mt) {
    case 1: return pick_npl<PREC, 1>(npl, H);
    case 2: return pick_npl<PREC, 2>(npl, H);
    default: return pick_npl<PREC, 3>(npl, H);
    }
}

const void *embed_kernel(const Dims &d, int mt)
{
    const int npl = npl_for(d);
    const bool bf16 = d.prec == TIG_BF16_MFMA;
    if (shape_is<1>(d))
        return bf16 ? pick_fixed<TIG_BF16_MFMA, 1>(mt) : pick_fixed<TIG_FP32, 1>(mt);
    if (shape_is<2>(d))
        return bf16 ? pick_fixed<TIG_BF16_MFMA, 2>(mt) : pick_fixed<TIG_FP32, 2>(mt);
    if (shape_is<3>(d))
        return bf16 ? pick_fixed<TIG_BF16_MFMA, 3>(mt) : pick_fixed<TIG_FP32, 3>(mt);
    return bf16 ? pick_mt<TIG_BF16_MFMA>(mt, npl, d.H) : pick_mt<TIG_FP32>(mt, npl, d.H);
}

}  // namespace

int embed_lds_bytes(const Dims &d, int mt)
{
    const EmbedParams p = embed_params(d, mt);
    return p.off_meta + 16 * mt * (4 * 4 + 8) + d.T * 16 + 16;
}

// 16-row tiles per workgroup for `rows` query rows.  A workgroup's latency grows with its rows,
// so the smallest tile count is taken whose tiles, one per workgroup, fit the compute units at hand.
static int embed_tiles(const LaunchPlan &plan, int rows, int units)
{
    for (int mt = 1; mt < plan.emb_mt; ++mt)
        if ((rows + 16 * mt - 1) / (16 * mt) <= units)
            return mt;
    return plan.emb_mt;
}

hipError_t prepare_embed(const Dims &d, const LaunchPlan &plan)
{
    for (int mt = 1; mt <= plan.emb_mt; ++mt) {
        const int own = embed_lds_bytes(d, mt);
        const int lds = embed_threads(d) == kScatterThreads && own < kOneLds ? kOneLds : own;
        const hipError_t e =
            hipFuncSetAttribute(embed_kernel(d, mt), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

// Workgroups of the preparation of a batch of `count` events.  When it shares a launch, every
// workgroup occupies a compute unit (the launch's LDS size applies to all of its workgroups), so
// there are few, each wavefront with several entries; on its own, four entries per wavefront.
int prepare_workgroups(int count, bool shared)
{
    const int entries = 2 * count;
    int n = shared ? (entries + kPrepWaves - 1) / kPrepWaves : (entries + 4 * kPrepWaves - 1) / (4 * kPrepWaves);
    if (shared && n > 31)
        n = 31;
    const int least = (entries + kPrepThreads - 1) / kPrepThreads;  // one entry per thread at most
    return n < least ? least : n;
}

int embed_spare_workgroups(const Dims &d, const LaunchPlan &plan, int roles, int count)
{
    if (embed_threads(d) != kScatterThreads)
        return 0;
    // the selection workgroup and the preparation workgroups of a batch of the same size; the row
    // tiles keep at least three quarters of the compute units
    const int want = 1 + prepare_workgroups(count, true);
    return want <= plan.num_cus / 4 ? want : 0;
}

hipError_t launch_embed(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                        hipStream_t s)
{
    StepArgs aa = a;
    PackedWeights ww = pw;
    const int threads = embed_threads(d);
    // memory overwrite: about four winners per wavefront at the winner count recent steps had
    int n_commit = 0;
    if (a.msg_count > 0) {
        const int most = 2 * a.msg_count;
        const int wins = a.wins_est > 0 && a.wins_est < most ? a.wins_est : most;
        const int per_block = 4 * (threads / kWave);
        n_commit = (wins + per_block - 1) / per_block;
        n_commit = n_commit < 1 ? 1 : (n_commit > 16 ? 16 : n_commit);
    }
    const int extra = n_commit + (a.sel.count > 0 ? 1 : 0) + (a.ded.count > 0 ? a.ded.n_wgs : 0);
    const int cus = plan.num_cus > 0 ? plan.num_cus : 256;
    const int units = cus - extra > 16 ? cus - extra : 16;
    // The tile height follows the number of distinct rows recent steps had (any height is correct:
    // the grid covers the most rows the batch can have, and tiles beyond the actual count return).
    const int most = a.roles * a.count;
    const int rows = a.rows_est > 0 && a.rows_est < most ? a.rows_est : most;
    const int mt = embed_tiles(plan, rows, units);
    EmbedParams p = embed_params(d, mt);
    p.n_tiles = (a.roles * a.count + 16 * mt - 1) / (16 * mt);  // tiles in use if no query repeats
    p.n_commit = n_commit;
    void *args[] = {&aa, &ww, &p};
    const int own = embed_lds_bytes(d, mt);
    const int lds = a.sel.count > 0 && own < kOneLds ? kOneLds : (own < kPrepLds ? kPrepLds : own);
    return hipLaunchKernel(embed_kernel(d, mt), dim3(p.n_tiles + extra), dim3(threads), args, (size_t)lds, s);
}

}  // namespace tig
