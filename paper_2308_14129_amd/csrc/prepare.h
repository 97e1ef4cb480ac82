// Query preparation of one batch (device side).  The embedding of a query depends on (node, t)
// only (embedding module f of the paper's Sec. II-C: the node's state and its history before t),
// and the sources and destinations of a batch repeat the same pairs many times over: hub nodes
// take part in a large share of the events, and events that share a timestamp put the same hub
// at the same time.  So every distinct (node, t) is embedded ONCE:
//   dedup_block   merges equal pairs among the 2B source / destination entries of a batch through
//                 a hash table of claims and looks up the K most recent neighbours of every
//                 distinct pair.  It reads the event stream and the adjacency only, never the
//                 model state, so it can run a step early, beside the previous embedding launch.
//   finish_*      the rest: slots pointed at rows, the row references (which rows the step's GRU
//                 replaces), and the negatives' lookups (their ids arrive with the call).
// gfx950 only.
#pragma once

#include "kernels_common.h"
#include "lookup.h"

namespace tig {

constexpr int kPrepThreads = 1024;
constexpr int kPrepWaves = kPrepThreads / kWave;
constexpr int kPrepLds = kPrepThreads * 4 + (kPrepWaves + 2) * 4;  // representative list + counters

__device__ inline uint32_t query_hash(int32_t u, double t)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(t);
    uint32_t h = (uint32_t)u * 0x9E3779B1u ^ (uint32_t)b * 0x85EBCA77u ^ (uint32_t)(b >> 32) * 0xC2B2AE3Du;
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    h ^= h >> 13;
    return h;
}

__device__ inline void entry_query(const StepArgs &a, int64_t first_eid, int i, int32_t &u, double &t)
{
    const int64_t eid = first_eid + (i >> 1);
    u = (i & 1) ? a.dst[eid] : a.src[eid];
    t = a.ts[eid];
}

// The entry that represents query (u, t) of entry i: the first entry to claim the pair's slot in
// the table (open addressing; a slot holds (epoch << 32 | entry), other epochs count as empty).
// A slot changes once per job, from empty to claimed, and the compare-and-swap decides who
// claimed it, so a stale read of "empty" only costs the failed swap.  The probe count is bounded
// by the table size; if that bound were ever hit the entry simply represents itself.
__device__ inline int claim_query(const StepArgs &a, const DedupJob &j, int i, int32_t u, double t)
{
    const int entries = 2 * j.count;
    const unsigned long long mine = ((unsigned long long)j.epoch << 32) | (uint32_t)i;
    uint32_t h = query_hash(u, t) & j.tab_mask;
    for (uint32_t probes = 0; probes <= j.tab_mask; ++probes) {
        unsigned long long cur = __hip_atomic_load(&j.tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(cur >> 32) != j.epoch) {
            const unsigned long long old = atomicCAS(&j.tab[h], cur, mine);
            if (old == cur)
                return i;
            cur = old;
            if ((uint32_t)(cur >> 32) != j.epoch)
                continue;  // (not reachable: only this job's claims replace an empty slot)
        }
        const uint32_t other = (uint32_t)cur;
        if ((int)other < entries) {
            int32_t uo;
            double to;
            entry_query(a, j.first_eid, (int)other, uo, to);
            if (uo == u && to == t)
                return (int)other;
        }
        h = (h + 1) & j.tab_mask;
    }
    return i;
}

// Workgroup `wg` of j.n_wgs: its share of the entries is claimed one entry per thread; the
// representatives among them are compacted, take consecutive rows of the query set (one atomic
// per workgroup), and the wavefronts look up their neighbours.  smem: kPrepLds bytes.
// ceil(2 * count / n_wgs) must not exceed kPrepThreads.
__device__ inline void dedup_block(const StepArgs &a, const DedupJob &j, int K, int wg, char *smem)
{
    int *list = (int *)smem;            // [kPrepThreads] thread index of the n-th representative
    int *s_cnt = list + kPrepThreads;   // [waves] representatives per wavefront, then their prefix
    int *s_base = s_cnt + kPrepWaves;   // [1] first row of this workgroup, [1] its representatives
    const int lane = lane_id();
    const int wave = wave_id();
    const int entries = 2 * j.count;
    const int chunk = (entries + j.n_wgs - 1) / j.n_wgs;
    const int i0 = wg * chunk;
    const int i = i0 + (int)threadIdx.x;
    const bool active = (int)threadIdx.x < chunk && i < entries;
    bool is_rep = false;
    if (active) {
        int32_t u;
        double t;
        entry_query(a, j.first_eid, i, u, t);
        const int rep = claim_query(a, j, i, u, t);
        is_rep = rep == i;
        if (!is_rep)
            j.qs.slot[i] = -rep - 1;
    }
    const unsigned long long m = __ballot(is_rep);
    const int rank = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0)
        s_cnt[wave] = __popcll(m);
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int w = 0; w < kPrepWaves; ++w) {
            const int c = s_cnt[w];
            s_cnt[w] = run;
            run += c;
        }
        s_base[0] = run > 0 ? atomicAdd(j.qs.n_u, run) : 0;
        s_base[1] = run;
    }
    __syncthreads();
    if (is_rep)
        list[s_cnt[wave] + rank] = (int)threadIdx.x;
    __syncthreads();
    const int base = s_base[0], n_rep = s_base[1];
    for (int l = wave; l < n_rep; l += kPrepWaves) {
        if (base + l >= entries)
            break;  // (a set holds a row per entry at most: only a counter that did not start at 0 gets here)
        const int e = i0 + list[l];
        int32_t u;
        double t;
        entry_query(a, j.first_eid, e, u, t);
        const int64_t eid = j.first_eid + (e >> 1);
        int32_t my_nbr, my_eid;
        double my_ts;
        nbr_lookup_wave(a, K, u, t, (int64_t)a.pos[2 * eid + (e & 1)], j.qs, base + l, my_nbr, my_eid, my_ts);
        if (lane == 0)
            j.qs.slot[e] = base + l;
    }
}

// Where the current state row of node v lives during a step: the staged GRU output of the entry
// that won v's message in the batch the step applies, or v's memory row.  key[v] holds the key of
// v's latest winning entry in the selections that used this key array; it belongs to the applied
// batch iff its event id lies in that batch.
struct RefCtx {
    int64_t num_nodes;
    const unsigned long long *key;  // key array of the applied batch's selection
    int64_t first_eid;              // the applied batch
    int32_t count;                  // 0: the step applies nothing
};

__device__ inline RefCtx ref_ctx(const StepArgs &a)
{
    return RefCtx{a.num_nodes, a.msg_key, a.msg_first_eid, a.msg_count};
}

// ... given key k = c.key[v] of a valid node v (any value if the step applies nothing)
__device__ inline int32_t ref_of_key(const RefCtx &c, int32_t v, unsigned long long k)
{
    if (c.count > 0) {
        const uint32_t low = (uint32_t)k;
        const int64_t e = (int64_t)(low >> 1);
        if (k != 0ull && e >= c.first_eid && e < c.first_eid + c.count)
            return ~(int32_t)(2 * (e - c.first_eid) + (low & 1u));
    }
    return v;
}

__device__ inline int32_t resolve_ref(const RefCtx &c, int32_t v)
{
    if (v < 0 || (int64_t)v >= c.num_nodes)
        return kRefNone;
    return ref_of_key(c, v, c.count > 0 ? c.key[v] : 0ull);
}

// The finishing pass of a batch's preparation, in three parts that share nothing:
//   finish_slots      entry i of the batch: its slot is pointed straight at its row (one thread
//                     per entry; representatives' slots never change)
//   finish_row        row `row` of the source / destination queries: row references
//   finish_negative   the negative of event b: lookup into row 2 * count + b, then its row references
// The first two need the batch's queries and the applied batch's keys only, so for a batch that
// was prepared ahead they run a step early as well (in the previous step's closing launch); the
// negatives arrive with the call and are looked up by the embedding kernel itself.
__device__ inline void finish_slots(const QuerySet &qs, int i, int entries)
{
    const int sl = qs.slot[i];
    if (sl < 0 && -sl - 1 < entries)
        qs.slot[i] = qs.slot[-sl - 1];
}

__device__ inline void finish_refs(const RefCtx &c, const QuerySet &qs, int K, int row, int32_t my_nbr, int32_t u)
{
    const int lane = lane_id();
    if (lane < K)
        qs.ref[(size_t)row * K + lane] = resolve_ref(c, my_nbr);
    if (lane == kWave - 1)
        qs.self_ref[row] = resolve_ref(c, u);
}

__device__ inline void finish_row(const RefCtx &c, const QuerySet &qs, int K, int row)
{
    const int lane = lane_id();
    int32_t my_nbr = -1;
    if (lane < K)
        my_nbr = qs.nbr[(size_t)row * K + lane];
    finish_refs(c, qs, K, row, my_nbr, qs.node[row]);
}

// Returns the number of filled slots; my_ref / my_eid / my_ts: slot `lane` of the row (lanes
// below K), as written to the query set.
__device__ inline int finish_negative(const StepArgs &a, int K, int b, int32_t &my_ref, int32_t &my_eid,
                                      double &my_ts)
{
    int32_t my_nbr;
    const int32_t u = a.neg[b];
    const int row = 2 * a.count + b;
    const int cnt = nbr_lookup_wave(a, K, u, a.ts[a.first_eid + b], -1, a.qs, row, my_nbr, my_eid, my_ts);
    // (the node id is validated by resolve_ref as the lookup did; it is not read back from the row,
    // which another lane of this wavefront has just written)
    const RefCtx c = ref_ctx(a);
    my_ref = resolve_ref(c, my_nbr);
    if (lane_id() < K)
        a.qs.ref[(size_t)row * K + lane_id()] = my_ref;
    return cnt;
}

}  // namespace tig
