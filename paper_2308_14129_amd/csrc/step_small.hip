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
#include "winners.h"

namespace tig {

namespace {

constexpr int kHashSlots = 2048;       // k_scatter: power of two, 2 x entries per workgroup

__global__ void __launch_bounds__(kScatterThreads) k_winners(WinnersJob j)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    winners_block(j, smem);
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
        e = load_entry(a.src, a.dst, a.ts, a.first_eid, i);
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
        e = load_entry(a.src, a.dst, a.ts, a.first_eid, i);
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
        hipLaunchKernelGGL(k_winners, dim3(1), dim3(kScatterThreads), kOneLds, s, winners_job(a, false));
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
    if (a.msg_count <= 0)
        return hipSuccess;
    const int clear_keys = winners_in_one_launch(a.msg_count) ? 0 : 1;
    hipLaunchKernelGGL(k_commit, dim3((2 * a.msg_count + 3) / 4), dim3(256), 0, s, a, M, clear_keys);
    return hipGetLastError();
}

}  // namespace tig
