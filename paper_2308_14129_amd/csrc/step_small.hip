// The small kernels of one batch step (paper Sec. II-C), gfx950 only.
//
// Last-message aggregation (all messages of a node within a batch are aggregated; this build
// keeps the last one): per node, the (event, role) entry with the greatest 64-bit
// (time, event id) key wins, found with atomicMax.
//   k_winners  batches of up to 4096 events: ONE workgroup holds the keys of the whole batch in
//              an LDS hash table (atomicMax in LDS), selects the winners and writes their
//              descriptors in entry order.  No global atomics, two memory round trips in all.
//   k_scatter + k_select  larger batches: keys go to a per-node array in memory, pre-reduced per
//              wavefront and per workgroup; a second launch selects and compacts the winners.
//   k_commit   memory overwrite M <- s_i(t), last_update (and key clear on the second path)
#include <hip/hip_runtime.h>

#include "kernels_common.h"

namespace tig {

#ifdef TIG_PHASE_CLOCKS
static __device__ unsigned long long g_phase_clocks[8192 * 8];
extern "C" __attribute__((visibility("default"))) int tig_debug_phase_clocks_small(unsigned long long *out, int n)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_clocks), sizeof(unsigned long long) * (size_t)n);
}
#endif

namespace {

constexpr int kScatterThreads = 1024;  // one (event, role) entry per thread and iteration
constexpr int kScatterWaves = kScatterThreads / kWave;
constexpr int kHashSlots = 2048;       // k_scatter: power of two, 2 x entries per workgroup
constexpr int kOneIters = 8;           // k_winners: up to 8 entries per thread
constexpr int kOneMaxEntries = kOneIters * kScatterThreads;
constexpr int kOneSlots = 12288;       // k_winners: 1.5 x the most distinct nodes, never fills up
constexpr int kOneLds = kOneSlots * 12 + (kOneIters * kScatterWaves + 1) * 4;

struct Entry {
    int32_t node, other;
    double t;
    unsigned long long key;
};

__device__ inline Entry load_entry(const StepArgs &a, int i)
{
    Entry e;
    const int64_t eid = a.first_eid + (i >> 1);
    const int role = i & 1;
    const int32_t s = a.src[eid], d = a.dst[eid];
    e.node = role ? d : s;
    e.other = role ? s : d;
    e.t = a.ts[eid];
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

__global__ void __launch_bounds__(kScatterThreads) k_winners(StepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    unsigned long long *t_key = (unsigned long long *)smem;   // [kOneSlots]
    int32_t *t_node = (int32_t *)(smem + kOneSlots * 8);      // [kOneSlots]
    int *s_cnt = (int *)(smem + kOneSlots * 12);              // [kOneIters * waves + 1]
    const int lane = lane_id();
    const int wave = wave_id();
    const int n_entries = 2 * a.count;

    TIG_MARK(0);
    for (int sidx = threadIdx.x; sidx < kOneSlots; sidx += kScatterThreads) {
        t_node[sidx] = -1;
        t_key[sidx] = 0ull;
    }
    TIG_MARK(1);
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
            ent[it] = load_entry(a, i);
    }
    __syncthreads();
    TIG_MARK(2);
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        if (it * kScatterThreads < n_entries) {  // uniform
            const bool active = it * kScatterThreads + threadIdx.x < n_entries;
            if (wave_leader_of_node(active, ent[it].node))
                table_insert_max<kOneSlots>(t_node, t_key, ent[it].node, ent[it].key);
        }
    }
    __syncthreads();
    TIG_MARK(3);
    // an entry supplies its node's message iff the node's key is the entry's own
    bool win[kOneIters];
    double lu[kOneIters];
#pragma unroll
    for (int it = 0; it < kOneIters; ++it) {
        win[it] = false;
        lu[it] = 0.0;
        if (it * kScatterThreads + threadIdx.x < n_entries) {
            uint32_t h = hash_slot<kOneSlots>(ent[it].node);
            while (t_node[h] != ent[it].node)
                h = h + 1 == (uint32_t)kOneSlots ? 0u : h + 1;
            win[it] = t_key[h] == ent[it].key;
            if (win[it])
                lu[it] = a.lu[ent[it].node];
        }
    }
    TIG_MARK(4);
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
        if (i < n_entries && a.is_winner)
            a.is_winner[i] = win[it] ? 1 : 0;
        if (win[it]) {
            WinDesc d;
            d.entry = i;
            d.node = ent[it].node;
            d.other = ent[it].other;
            d.b = i >> 1;
            d.dt = ent[it].t - lu[it];
            d.t = ent[it].t;
            a.win[s_cnt[it * kScatterWaves + wave] + rank[it]] = d;
        }
    }
    TIG_MARK(5);
}

// Larger batches, part 1: keys to the per-node array in memory.  Lanes of a wavefront that hit
// the same node are merged first, then the workgroup merges across wavefronts in an LDS hash
// table (hub nodes take thousands of entries per batch, and same-address device atomics
// serialise), and finally one atomicMax per distinct node of the workgroup goes to memory.
__global__ void __launch_bounds__(kScatterThreads) k_scatter(StepArgs a)
{
    __shared__ int32_t t_node[kHashSlots];
    __shared__ unsigned long long t_key[kHashSlots];
    for (int sidx = threadIdx.x; sidx < kHashSlots; sidx += kScatterThreads) {
        t_node[sidx] = -1;
        t_key[sidx] = 0ull;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        *a.n_win = 0;  // counter of k_select, which follows
    __syncthreads();
    const int i = blockIdx.x * kScatterThreads + threadIdx.x;
    const bool active = i < 2 * a.count;
    Entry e;
    e.node = -1;
    e.key = 0ull;
    if (active)
        e = load_entry(a, i);
    if (wave_leader_of_node(active, e.node))
        table_insert_max<kHashSlots>(t_node, t_key, e.node, e.key);
    __syncthreads();
    for (int sidx = threadIdx.x; sidx < kHashSlots; sidx += kScatterThreads)
        if (t_node[sidx] >= 0)
            atomicMax(a.key + t_node[sidx], t_key[sidx]);
}

// Larger batches, part 2: an entry supplies its node's message iff the node's key is the entry's
// own.  Winners are compacted
// through an atomic counter; their order is irrelevant (rows are independent).
__global__ void __launch_bounds__(256) k_select(StepArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    bool win = false;
    Entry e;
    e.node = 0;
    e.other = 0;
    e.t = 0.0;
    e.key = 0ull;
    if (i < 2 * a.count) {
        e = load_entry(a, i);
        win = a.key[e.node] == e.key;
        if (a.is_winner)
            a.is_winner[i] = win ? 1 : 0;
    }
    const unsigned long long mask = __ballot(win);
    if (mask == 0ull)
        return;
    const int lane = lane_id();
    int base = 0;
    if (lane == 0)
        base = atomicAdd(a.n_win, __popcll(mask));
    base = __shfl(base, 0, kWave);
    if (win) {
        WinDesc d;
        d.entry = i;
        d.node = e.node;
        d.other = e.other;
        d.b = i >> 1;
        d.dt = e.t - a.lu[e.node];
        d.t = e.t;
        a.win[base + __popcll(mask & ((1ull << lane) - 1ull))] = d;
    }
}

// Memory overwrite M <- s_i(t) for the winners (after every message has read the batch-start
// memory), last_update, and key clear.  One wavefront per winner.
__global__ void __launch_bounds__(256) k_commit(StepArgs a, int M, int clear_keys)
{
    const int r = blockIdx.x * (blockDim.x / kWave) + wave_id();
    const WinDesc d = a.win[r];  // r < 2*count: in range; read together with the count
    if (r >= *a.n_win)
        return;
    const int lane = lane_id();
    for (int j = lane; j < M; j += kWave)
        a.mem[(size_t)d.node * M + j] = a.staging[(size_t)d.entry * M + j];
    if (lane == 0) {
        a.lu[d.node] = d.t;
        if (clear_keys)
            a.key[d.node] = 0ull;
    }
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
    return hipFuncSetAttribute((const void *)k_winners, hipFuncAttributeMaxDynamicSharedMemorySize, kOneLds);
}

bool winners_in_one_launch(int count) { return 2 * count <= kOneMaxEntries; }

hipError_t launch_scatter(const StepArgs &a, hipStream_t s, bool *needs_select)
{
    const int entries = 2 * a.count;
    *needs_select = !winners_in_one_launch(a.count);
    if (!*needs_select)
        hipLaunchKernelGGL(k_winners, dim3(1), dim3(kScatterThreads), kOneLds, s, a);
    else
        hipLaunchKernelGGL(k_scatter, dim3((entries + kScatterThreads - 1) / kScatterThreads),
                           dim3(kScatterThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_select(const StepArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(k_select, dim3((2 * a.count + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_commit(const StepArgs &a, int M, hipStream_t s)
{
    const int clear_keys = winners_in_one_launch(a.count) ? 0 : 1;
    hipLaunchKernelGGL(k_commit, dim3((2 * a.count + 3) / 4), dim3(256), 0, s, a, M, clear_keys);
    return hipGetLastError();
}

}  // namespace tig
