// The small kernels of one batch step (paper Sec. II-C), gfx950 only:
//   k_pre     two jobs in one launch: last-message aggregation (64-bit (time, event id) atomicMax
//             per node) and most-recent-K temporal neighbours (one wavefront per query)
//   k_select  winners = entries whose key survived; compacted list
//   k_commit  memory overwrite M <- s_i(t), last_update, key clear
#include <hip/hip_runtime.h>

#include "kernels_common.h"

namespace tig {

namespace {

// ------------------------------------------------------------------------------------------
// First launch of a step, two independent jobs side by side (block-uniform choice):
//
//  * blocks [0, n_scatter): last-message aggregation, part 1.  Each block takes 1024 (event,
//    role) entries.  Lanes of a wavefront that hit the same node are merged first, then the
//    block merges across wavefronts in an LDS hash table (hub nodes take thousands of entries
//    per batch, and same-address device atomics serialise), and finally issues one 64-bit
//    atomicMax of the (time, event id) key per distinct node of the block.
//  * remaining blocks: most-recent-K neighbours before the query time.  One wavefront per query:
//    64-way search for the first adjacency entry with time >= t, then lanes 0..K-1 read the K
//    entries below it.
constexpr int kScatterEntries = 1024;
constexpr int kHashSlots = 2048;  // power of two, >= 2 * kScatterEntries: never fills up

__device__ inline void scatter_keys_block(const StepArgs &a, int block)
{
    __shared__ int32_t t_node[kHashSlots];
    __shared__ unsigned long long t_key[kHashSlots];
    for (int sidx = threadIdx.x; sidx < kHashSlots; sidx += blockDim.x) {
        t_node[sidx] = -1;
        t_key[sidx] = 0ull;
    }
    if (block == 0 && threadIdx.x == 0)
        *a.n_win = 0;  // counter of the compaction that follows in the next launch
    __syncthreads();
    const int lane = lane_id();
    for (int it = 0; it < kScatterEntries / 256; ++it) {
        const int i = block * kScatterEntries + it * 256 + threadIdx.x;
        const bool active = i < 2 * a.count;
        int32_t node = -1;
        unsigned long long key = 0;
        if (active) {
            const int64_t eid = a.first_eid + (i >> 1);
            const int role = i & 1;
            node = role ? a.dst[eid] : a.src[eid];
            key = winner_key(a.ts[eid], (int32_t)eid, role);
        }
        unsigned long long todo = __ballot(active);
        bool insert = false;
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int32_t n0 = __shfl(node, leader, kWave);
            const unsigned long long grp = __ballot(active && node == n0);
            // keys grow with the entry index (time-sorted events): the highest lane holds the max
            if (lane == 63 - __clzll((long long)grp))
                insert = true;
            todo &= ~grp;
        }
        if (insert) {
            uint32_t h = ((uint32_t)node * 2654435761u) >> 21;  // 11 bits
            while (true) {
                const int32_t prev = atomicCAS(&t_node[h], -1, node);
                if (prev == -1 || prev == node) {
                    atomicMax(&t_key[h], key);
                    break;
                }
                h = (h + 1) & (kHashSlots - 1);
            }
        }
    }
    __syncthreads();
    for (int sidx = threadIdx.x; sidx < kHashSlots; sidx += blockDim.x)
        if (t_node[sidx] >= 0)
            atomicMax(a.key + t_node[sidx], t_key[sidx]);
}

__device__ inline void nbr_lookup_wave(const StepArgs &a, int K, int q)
{
    const int lane = lane_id();
    const int role = q / a.count;
    const int b = q - role * a.count;
    const int64_t eid = a.first_eid + b;
    const int32_t u = role == 0 ? a.src[eid] : (role == 1 ? a.dst[eid] : a.neg[b]);
    const double t = a.ts[eid];
    int64_t lo = 0, hi = 0;
    if (u >= 0 && (int64_t)u < a.num_nodes) {
        lo = a.indptr[u];
        hi = a.indptr[u + 1];
    }
    const int64_t base = lo;
    // invariant: entries below lo have time < t; entries at or above hi have time >= t
    while (hi - lo > kWave) {
        const int64_t step = (hi - lo + kWave - 1) / kWave;
        int64_t idx = lo + (int64_t)(lane + 1) * step - 1;
        if (idx > hi - 1)
            idx = hi - 1;
        const bool less = a.csr[idx].ts < t;
        const int c = __popcll(__ballot(less));  // lists are time-ordered: lanes 0..c-1 are true
        int64_t nlo = lo + (int64_t)c * step;
        if (nlo > hi)
            nlo = hi;
        if (c < kWave) {
            int64_t nhi = lo + (int64_t)(c + 1) * step - 1;
            if (nhi > hi - 1)
                nhi = hi - 1;
            hi = nhi;
        }
        lo = nlo;
    }
    {
        const int64_t idx = lo + lane;
        const bool less = idx < hi && a.csr[idx].ts < t;
        lo += __popcll(__ballot(less));
    }
    const int64_t avail = lo - base;
    if (lane < K) {
        const int64_t p = lo - 1 - lane;
        const size_t o = (size_t)q * K + lane;
        if (p >= base) {
            const CsrEntry e = a.csr[p];
            a.nbr_node[o] = e.nbr;
            a.nbr_eid[o] = e.eid;
            a.nbr_ts[o] = e.ts;
        } else {
            a.nbr_node[o] = -1;
            a.nbr_eid[o] = -1;
            a.nbr_ts[o] = 0.0;
        }
    }
    if (lane == 0)
        a.nbr_cnt[q] = (int32_t)(avail < K ? avail : K);
}

__global__ void __launch_bounds__(256) k_pre(StepArgs a, int K, int n_scatter)
{
    if ((int)blockIdx.x < n_scatter) {
        scatter_keys_block(a, blockIdx.x);
    } else {
        const int q = ((int)blockIdx.x - n_scatter) * (256 / kWave) + wave_id();
        if (q < a.roles * a.count)
            nbr_lookup_wave(a, K, q);
    }
}

// ------------------------------------------------------------------------------------------
// Last-message aggregation, part 2: an entry supplies its node's message iff the node's key is
// the entry's own.  Winners are compacted into win_list (order irrelevant: rows are independent).
__global__ void __launch_bounds__(256) k_select(StepArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    bool win = false;
    if (i < 2 * a.count) {
        const int64_t eid = a.first_eid + (i >> 1);
        const int role = i & 1;
        const int32_t node = role ? a.dst[eid] : a.src[eid];
        win = a.key[node] == winner_key(a.ts[eid], (int32_t)eid, role);
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
    if (win)
        a.win_list[base + __popcll(mask & ((1ull << lane) - 1ull))] = i;
}

// ------------------------------------------------------------------------------------------
// Memory overwrite M <- s_i(t) for the winners (after every message has read the batch-start
// memory), last_update, and key clear.  One wavefront per winner.
__global__ void __launch_bounds__(256) k_commit(StepArgs a, int M)
{
    const int r = blockIdx.x * (blockDim.x / kWave) + wave_id();
    if (r >= *a.n_win)
        return;
    const int lane = lane_id();
    const int i = a.win_list[r];
    const int64_t eid = a.first_eid + (i >> 1);
    const int32_t node = (i & 1) ? a.dst[eid] : a.src[eid];
    for (int j = lane; j < M; j += kWave)
        a.mem[(size_t)node * M + j] = a.staging[(size_t)i * M + j];
    if (lane == 0) {
        a.lu[node] = a.ts[eid];
        a.key[node] = 0ull;
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

hipError_t launch_pre(const StepArgs &a, int K, hipStream_t s)
{
    const int entries = 2 * a.count;
    const int Q = a.roles * a.count;
    const int n_scatter = (entries + kScatterEntries - 1) / kScatterEntries;
    hipLaunchKernelGGL(k_pre, dim3(n_scatter + (Q + 3) / 4), dim3(256), 0, s, a, K, n_scatter);
    return hipGetLastError();
}

hipError_t launch_select(const StepArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(k_select, dim3((2 * a.count + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_commit(const StepArgs &a, int M, hipStream_t s)
{
    hipLaunchKernelGGL(k_commit, dim3((2 * a.count + 3) / 4), dim3(256), 0, s, a, M);
    return hipGetLastError();
}

}  // namespace tig
