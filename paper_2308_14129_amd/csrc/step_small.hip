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

}  // namespace tig
