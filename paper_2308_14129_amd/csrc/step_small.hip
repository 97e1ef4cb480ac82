// The small kernels of one batch step (paper Sec. II-C), gfx950 only.
//
// Last-message aggregation (all messages of a node within a batch are aggregated; this build
// keeps the last one): per node, the (event, role) entry with the greatest 64-bit
// (time, event id) key wins, found with atomicMax.
//   k_prepare  a step whose batch was not prepared during the previous step's embedding launch:
//              one workgroup selects the winners of a batch of up to 4096 events (winners.h: the
//              keys of the whole batch in an LDS hash table, no global atomics), the others merge
//              equal queries and look up the neighbours of the distinct ones (prepare.h)
//   k_scatter + k_select  larger batches: keys go to the per-node array in memory, pre-reduced per
//              wavefront and per workgroup; a second launch selects and compacts the winners
//   k_decode   per event, from the rows of the distinct queries: the two logits and the three
//              embedding rows; in the same launch the memory overwrite M <- s_i(t), last_update,
//              and the optional inspection outputs
#include <hip/hip_runtime.h>

#include "kernels_common.h"
#include "prepare.h"
#include "winners.h"

namespace tig {

namespace {

constexpr int kHashSlots = 2048;       // k_scatter: power of two, 2 x entries per workgroup

__global__ void __launch_bounds__(kScatterThreads) k_prepare(StepArgs a, SelectJob sel, DedupJob ded, int K)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int x = (int)blockIdx.x;
    if (sel.count > 0) {
        if (x == 0) {
            winners_block(a, sel, smem);
            return;
        }
        --x;
    }
    if (ded.count > 0 && x < ded.n_wgs)
        dedup_block(a, ded, K, x, smem);
}

// Larger batches, part 1: keys to the per-node array in memory.  Lanes of a wavefront that hit
// the same node are merged first, then the workgroup merges across wavefronts in an LDS hash
// table (hub nodes take thousands of entries per batch, and same-address device atomics
// serialise), and finally one atomicMax per distinct node of the workgroup goes to memory.
// Keys left in the array by earlier batches are smaller than any key of this one.
__global__ void __launch_bounds__(kScatterThreads) k_scatter(StepArgs a, SelectJob j)
{
    __shared__ int32_t t_node[kHashSlots];
    __shared__ unsigned long long t_key[kHashSlots];
    for (int sidx = threadIdx.x; sidx < kHashSlots; sidx += kScatterThreads) {
        t_node[sidx] = -1;
        t_key[sidx] = 0ull;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        *j.n_win = 0;  // counter of k_select, which follows
    __syncthreads();
    const int i = blockIdx.x * kScatterThreads + threadIdx.x;
    const bool active = i < 2 * j.count;
    Entry e;
    e.node = -1;
    e.key = 0ull;
    if (active)
        e = load_entry(a.src, a.dst, a.ts, j.first_eid, i);
    if (wave_leader_of_node(active, e.node))
        table_insert_max<kHashSlots>(t_node, t_key, e.node, e.key);
    __syncthreads();
    for (int sidx = threadIdx.x; sidx < kHashSlots; sidx += kScatterThreads)
        if (t_node[sidx] >= 0)
            atomicMax(j.key + t_node[sidx], t_key[sidx]);
}

// Larger batches, part 2: an entry supplies its node's message iff the node's key is the entry's
// own.  Winners are compacted through an atomic counter; their order is irrelevant (rows are
// independent).
__global__ void __launch_bounds__(256) k_select(StepArgs a, SelectJob j)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    bool win = false;
    Entry e;
    e.node = 0;
    e.other = 0;
    e.t = 0.0;
    e.key = 0ull;
    if (i < 2 * j.count) {
        e = load_entry(a.src, a.dst, a.ts, j.first_eid, i);
        win = j.key[e.node] == e.key;
        if (j.flags)
            j.flags[i] = win ? 1 : 0;
    }
    const unsigned long long mask = __ballot(win);
    if (mask == 0ull)
        return;
    const int lane = lane_id();
    int base = 0;
    if (lane == 0)
        base = atomicAdd(j.n_win, __popcll(mask));
    base = __shfl(base, 0, kWave);
    if (win) {
        WinDesc d;
        d.entry = i;
        d.node = e.node;
        d.other = e.other;
        d.b = i >> 1;
        d.t = e.t;
        j.win[base + __popcll(mask & ((1ull << lane) - 1ull))] = d;
    }
}

struct DecodeParams {
    int M, E, Ep, K;
    int n_event_blocks;   // blocks of 4 wavefronts, one event each
    int n_commit_blocks;  // one winner each
    int n_expand_blocks;  // one query each (inspection outputs), 0 if none is wanted
    int n_fin_row_blocks; // row references of the batch prepared ahead, grid-stride over its rows
    int n_fin_slot_blocks; // its slots, one entry per thread
};

__device__ inline int row_of_entry(const QuerySet &qs, int i)
{
    const int s = qs.slot[i];
    return s >= 0 ? s : qs.slot[-s - 1];
}

// score(a, b) = w_d2 . relu(W_d1 [emb_a | emb_b] + b_d1) + b_d2 (decoder g of Sec. II-C) from the
// per-row halves of layer 1 that the embedding kernel left; the embedding rows of the event's
// three queries are copies of their distinct rows.
__global__ void __launch_bounds__(256) k_decode(StepArgs a, PackedWeights w, DecodeParams p)
{
    const int lane = lane_id();
    int blk = (int)blockIdx.x;
    if (blk < p.n_event_blocks) {
        const int b = blk * 4 + wave_id();
        if (b >= a.count)
            return;
        const int n_u = *a.qs.n_u;
        int row[3];
        row[0] = row_of_entry(a.qs, 2 * b);
        row[1] = row_of_entry(a.qs, 2 * b + 1);
        row[2] = a.roles == 3 ? n_u + b : row[1];
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
        return;
    }
    blk -= p.n_event_blocks;
    if (blk < p.n_commit_blocks) {
        // Memory overwrite M <- s_i(t) for the winners of the applied batch (every reader of this
        // step took the staged rows instead), and last_update.  One wavefront per winner at a time.
        const int n_win = *a.n_win;
        for (int r = blk * 4 + wave_id(); r < n_win; r += p.n_commit_blocks * 4) {
            const WinDesc d = a.win[r];
            for (int j = lane; j < p.M; j += kWave)
                a.mem[(size_t)d.node * p.M + j] = a.staging[(size_t)d.entry * p.M + j];
            if (lane == 0)
                a.lu[d.node] = d.t;
        }
        return;
    }
    blk -= p.n_commit_blocks;
    if (blk >= p.n_expand_blocks) {
        // Finishing pass for the batch that the embedding launch has just prepared (prepare.h): its
        // row references against the batch the NEXT step will apply, and its slots.
        blk -= p.n_expand_blocks;
        const QuerySet &nq = a.ded.qs;
        if (blk < p.n_fin_row_blocks) {
            const RefCtx c{a.num_nodes, a.fin_msg_key, a.fin_msg_first_eid, a.fin_msg_count};
            const int n_u = *nq.n_u;
            for (int row = blk * 4 + wave_id(); row < n_u; row += p.n_fin_row_blocks * 4)
                finish_row(c, nq, p.K, row);
        } else {
            const int i = (blk - p.n_fin_row_blocks) * 256 + (int)threadIdx.x;
            if (i < 2 * a.fin_count)
                finish_slots(nq, i);
        }
        return;
    }
    // inspection outputs, per query in the order [sources | destinations | negatives]
    const int q = blk * 4 + wave_id();
    if (q >= a.roles * a.count)
        return;
    const int role = q / a.count, b = q - role * a.count;
    const int row = role < 2 ? row_of_entry(a.qs, 2 * b + role) : *a.qs.n_u + b;
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

__global__ void k_fill_zero(uint32_t *p, size_t words)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride)
        p[i] = 0u;
}

}  // namespace

hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t s)
{
    if (bytes == 0)
        return hipSuccess;
    const size_t words = bytes / 4;  // every buffer of the library is a multiple of 4 bytes
    size_t blocks = (words + 255) / 256;
    if (blocks > 16384)
        blocks = 16384;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, (uint32_t *)ptr, words);
    return hipGetLastError();
}

hipError_t prepare_small()
{
    return hipFuncSetAttribute((const void *)k_prepare, hipFuncAttributeMaxDynamicSharedMemorySize, kOneLds);
}

bool winners_in_one_launch(int count) { return 2 * count <= kOneMaxEntries; }

hipError_t launch_scatter(const StepArgs &a, const SelectJob &j, hipStream_t s)
{
    const int entries = 2 * j.count;
    hipLaunchKernelGGL(k_scatter, dim3((entries + kScatterThreads - 1) / kScatterThreads),
                       dim3(kScatterThreads), 0, s, a, j);
    return hipGetLastError();
}

hipError_t launch_select(const StepArgs &a, const SelectJob &j, hipStream_t s)
{
    hipLaunchKernelGGL(k_select, dim3((2 * j.count + 255) / 256), dim3(256), 0, s, a, j);
    return hipGetLastError();
}

hipError_t launch_prepare(const StepArgs &a, const SelectJob &sel, const DedupJob &ded, int K, hipStream_t s)
{
    const int blocks = (sel.count > 0 ? 1 : 0) + (ded.count > 0 ? ded.n_wgs : 0);
    if (blocks == 0)
        return hipSuccess;
    const int lds = sel.count > 0 ? kOneLds : kPrepLds;
    hipLaunchKernelGGL(k_prepare, dim3(blocks), dim3(kScatterThreads), lds, s, a, sel, ded, K);
    return hipGetLastError();
}

hipError_t launch_decode(const Dims &d, const PackedWeights &pw, const StepArgs &a, hipStream_t s)
{
    DecodeParams p;
    p.M = d.M;
    p.E = d.E;
    p.Ep = d.Ep;
    p.K = d.K;
    p.n_event_blocks = (a.count + 3) / 4;
    // the winners are usually a small share of the 2 * msg_count entries: a modest number of
    // wavefronts, each taking winner after winner
    p.n_commit_blocks = a.msg_count > 0 ? (2 * a.msg_count + 3) / 4 : 0;
    if (p.n_commit_blocks > 128)
        p.n_commit_blocks = 128;
    const bool expand = a.out_nbr_node || a.out_nbr_eid || a.out_nbr_ts || a.out_nbr_cnt || a.out_is_winner;
    p.n_expand_blocks = expand ? (a.roles * a.count + 3) / 4 : 0;
    p.n_fin_row_blocks = p.n_fin_slot_blocks = 0;
    if (a.fin_count > 0) {
        p.n_fin_row_blocks = (2 * a.fin_count + 3) / 4;
        if (p.n_fin_row_blocks > 256)
            p.n_fin_row_blocks = 256;
        p.n_fin_slot_blocks = (2 * a.fin_count + 255) / 256;
    }
    hipLaunchKernelGGL(k_decode, dim3(p.n_event_blocks + p.n_commit_blocks + p.n_expand_blocks + p.n_fin_row_blocks +
                                      p.n_fin_slot_blocks),
                       dim3(256), 0, s, a, pw, p);
    return hipGetLastError();
}

}  // namespace tig
