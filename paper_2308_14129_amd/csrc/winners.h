// Last-message selection of a whole batch inside ONE workgroup of 1024 threads (paper Sec. II-C:
// the messages of a node within a batch are aggregated; this build keeps the last one).
// The result depends on the event stream only, not on the model state, so the embedding kernel
// of one step can run it for the FOLLOWING batch in one extra workgroup; the same code also runs
// in the preparation launch of a step whose batch was not anticipated.  gfx950 only.
#pragma once

#include "kernels_common.h"

namespace tig {

constexpr int kScatterThreads = 1024;  // one (event, role) entry per thread and iteration
constexpr int kScatterWaves = kScatterThreads / kWave;
constexpr int kOneIters = 8;           // up to 8 entries per thread
constexpr int kOneMaxEntries = kOneIters * kScatterThreads;
constexpr int kOneSlots = 12288;       // 1.5 x the most distinct nodes, never fills up
constexpr int kOneLds = kOneSlots * 12 + (kOneIters * kScatterWaves + 1) * 4;

struct Entry {
    int32_t node, other;
    double t;
    unsigned long long key;
};

__device__ inline Entry load_entry(const int32_t *src, const int32_t *dst, const double *ts, int64_t first_eid, int i)
{
    Entry e;
    const int64_t eid = first_eid + (i >> 1);
    const int role = i & 1;
    const int32_t s = src[eid], d = dst[eid];
    e.node = role ? d : s;
    e.other = role ? s : d;
    e.t = ts[eid];
    e.key = winner_key(e.t, (int32_t)eid, role);
    return e;
}

// Among the active lanes of the wavefront, true for the one lane per distinct node that holds
// that node's greatest key.  Keys grow with the entry index (time-sorted events), and entries
// grow with the lane, so that is the highest lane of each group.
// Only the first kRounds distinct nodes of the wavefront are merged this way (heavy hitters show
// up early); lanes of any other node all answer true and meet in the hash table instead.
__device__ inline bool wave_leader_of_node(bool active, int32_t node)
{
    constexpr int kRounds = 4;
    const int lane = lane_id();
    unsigned long long todo = __ballot(active);
    bool leader = active;
#pragma unroll
    for (int round = 0; round < kRounds; ++round) {
        if (todo == 0ull)
            break;
        const int first = __ffsll((long long)todo) - 1;
        const int32_t n0 = __builtin_amdgcn_readlane(node, first);
        const bool mine = active && node == n0;
        const unsigned long long grp = __ballot(mine);
        if (mine)
            leader = lane == 63 - __clzll((long long)grp);
        todo &= ~grp;
    }
    return leader;
}

template <int SLOTS>
__device__ inline uint32_t hash_slot(int32_t node)
{
    return (uint32_t)(((uint32_t)node * 2654435761u) >> 8) % (uint32_t)SLOTS;
}

// insert (node, key) with max-merge into an open-addressing LDS table that is never full
template <int SLOTS>
__device__ inline void table_insert_max(int32_t *t_node, unsigned long long *t_key, int32_t node,
                                        unsigned long long key)
{
    uint32_t h = hash_slot<SLOTS>(node);
    while (true) {
        const int32_t prev = atomicCAS(&t_node[h], -1, node);
        if (prev == -1 || prev == node) {
            atomicMax(&t_key[h], key);
            return;
        }
        h = h + 1 == (uint32_t)SLOTS ? 0u : h + 1;
    }
}

// All 1024 threads of the workgroup call this; smem holds kOneLds bytes, 16-byte aligned.
// Besides the winner list and the per-entry flags, every winner leaves its key in key[node]: a
// later lookup of "was this node updated by batch (first_eid, count), and by which entry" reads
// key[node] and checks that the event id inside lies in the batch (keys of other batches do not).
__device__ inline void winners_block(const StepArgs &g, const SelectJob &a, char *smem)
{
    unsigned long long *t_key = (unsigned long long *)smem;   // [kOneSlots]
    int32_t *t_node = (int32_t *)(smem + kOneSlots * 8);      // [kOneSlots]
    int *s_cnt = (int *)(smem + kOneSlots * 12);              // [kOneIters * waves + 1]
    const int lane = lane_id();
    const int wave = wave_id();
    const int n_entries = 2 * a.count;

    for (int sidx = threadIdx.x; sidx < kOneSlots; sidx += kScatterThreads) {
        t_node[sidx] = -1;
        t_key[sidx] = 0ull;
    }
    // the thread owns entries it*1024 + tid; all of their loads are issued together
    Entry ent[kOneIters];
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        const int i = it * kScatterThreads + threadIdx.x;
        ent[it].node = -1;
        ent[it].other = 0;
        ent[it].t = 0.0;
        ent[it].key = 0ull;
        if (i < n_entries)
            ent[it] = load_entry(g.src, g.dst, g.ts, a.first_eid, i);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        if (it * kScatterThreads < n_entries) {  // uniform
            const bool active = it * kScatterThreads + threadIdx.x < n_entries;
            if (wave_leader_of_node(active, ent[it].node))
                table_insert_max<kOneSlots>(t_node, t_key, ent[it].node, ent[it].key);
        }
    }
    __syncthreads();
    // an entry supplies its node's message iff the node's key is the entry's own
    bool win[kOneIters];
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        win[it] = false;
        if (it * kScatterThreads + threadIdx.x < n_entries) {
            uint32_t h = hash_slot<kOneSlots>(ent[it].node);
            while (t_node[h] != ent[it].node)
                h = h + 1 == (uint32_t)kOneSlots ? 0u : h + 1;
            win[it] = t_key[h] == ent[it].key;
        }
    }
    // ordered compaction: counts per (iteration, wavefront), exclusive prefix, then the writes
    int rank[kOneIters];
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        const unsigned long long m = __ballot(win[it]);
        rank[it] = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0)
            s_cnt[it * kScatterWaves + wave] = __popcll(m);
    }
    __syncthreads();
    if (wave == 0) {
        constexpr int kPer = kOneIters * kScatterWaves / kWave;  // counts per lane
        int c[kPer], sum = 0;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            c[j] = s_cnt[lane * kPer + j];
            sum += c[j];
        }
        int incl = sum;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off, kWave);
            if (lane >= off)
                incl += up;
        }
        int run = incl - sum;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            s_cnt[lane * kPer + j] = run;
            run += c[j];
        }
        if (lane == kWave - 1)
            *a.n_win = incl;
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        const int i = it * kScatterThreads + threadIdx.x;
        if (i < n_entries && a.flags)
            a.flags[i] = win[it] ? 1 : 0;
        if (win[it]) {
            a.key[ent[it].node] = ent[it].key;
            WinDesc d;
            d.entry = i;
            d.node = ent[it].node;
            d.other = ent[it].other;
            d.b = i >> 1;
            d.t = ent[it].t;
            a.win[s_cnt[it * kScatterWaves + wave] + rank[it]] = d;
        }
    }
}

// Memory overwrite M <- s_i(t) for the winners of the applied batch, and their last_update.
// Wavefront `w` of `n_waves` takes winner after winner.  While a step runs, every reader of an
// updated node's state takes the staged row through its row reference, never the memory row, so
// this may run beside the embedding.
__device__ inline void overwrite_memory(const StepArgs &a, int M, int w, int n_waves)
{
    const int lane = lane_id();
    int n_win = *a.n_win;
    n_win = n_win < 2 * a.msg_count ? n_win : 2 * a.msg_count;
    for (int r = w; r < n_win; r += n_waves) {
        const WinDesc d = a.win[r];
        if (d.node < 0 || (int64_t)d.node >= a.num_nodes || d.entry < 0 || d.entry >= 2 * a.msg_count)
            continue;  // (not a descriptor of this batch)
        for (int j = lane; j < M; j += kWave)
            a.mem[(size_t)d.node * M + j] = a.staging[(size_t)d.entry * M + j];
        if (lane == 0)
            a.lu[d.node] = d.t;
    }
}

}  // namespace tig
