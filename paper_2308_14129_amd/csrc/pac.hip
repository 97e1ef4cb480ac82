// Epoch machinery of parallel training on partitions (paper Sec. II-C "Distributed Parallel
// Training", Alg. 2), device side.  gfx950 only.
//   sub-graph of a (combined) partition   E_k = {(i, j, t) in E | i, j in V_k}: an order-preserving
//       compaction of the event stream by a per-node membership test (count per workgroup, scan of
//       the counts, write), and the same compaction over the nodes for the local ids;
//   gather of the sub-graph's event arrays with endpoints relabelled to local ids;
//   memory synchronisation of the shared nodes across the partitions resident on this GPU.
#include <hip/hip_runtime.h>

#include "kernels_common.h"
#include "tig_internal.h"

namespace tig {

namespace {

constexpr int kCompThreads = 256;
constexpr int kCompPer = 8;                           // consecutive items per thread
constexpr int kCompBlock = kCompThreads * kCompPer;   // items per workgroup
constexpr int kScanThreads = 1024;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// A node with replicas in more than one part resides in every part (node loop of Alg. 1).
__device__ inline bool is_member(const uint64_t *node_parts, int64_t num_nodes, int64_t v, uint64_t group)
{
    if (v < 0 || v >= num_nodes)
        return false;
    const uint64_t m = node_parts[v];
    return __popcll(m) > 1 ? group != 0ull : (m & group) != 0ull;
}

struct EventPred {
    const int32_t *src, *dst;
    const uint64_t *node_parts;
    int64_t num_nodes;
    uint64_t group;
    __device__ bool operator()(int64_t e) const
    {
        return is_member(node_parts, num_nodes, src[e], group) && is_member(node_parts, num_nodes, dst[e], group);
    }
};

struct NodePred {
    const uint64_t *node_parts;
    int64_t num_nodes;
    uint64_t group;
    __device__ bool operator()(int64_t v) const { return is_member(node_parts, num_nodes, v, group); }
};

// The count pass also leaves the verdicts of a thread's 8 consecutive items as one byte, so the
// write pass neither re-reads the items nor repeats the test.
template <class Pred>
__global__ void __launch_bounds__(kCompThreads) k_comp_count(Pred pred, int64_t n, int32_t *block_counts,
                                                             uint8_t *keep_bits)
{
    __shared__ int total;
    if (threadIdx.x == 0)
        total = 0;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * kCompBlock + (int64_t)threadIdx.x * kCompPer;
    int c = 0;
    unsigned bits = 0;
#pragma unroll
    for (int u = 0; u < kCompPer; ++u)
        if (i0 + u < n && pred(i0 + u)) {
            ++c;
            bits |= 1u << u;
        }
    if (i0 < n)
        keep_bits[i0 / kCompPer] = (uint8_t)bits;
    if (c)
        atomicAdd(&total, c);
    __syncthreads();
    if (threadIdx.x == 0)
        block_counts[blockIdx.x] = total;
}

// exclusive scan of the workgroup counts (one workgroup; the counts of ~1e5 workgroups at most)
__global__ void __launch_bounds__(kScanThreads) k_comp_scan(const int32_t *block_counts, int64_t n_blocks,
                                                            int64_t *block_offsets, int64_t *total)
{
    __shared__ int64_t part[kScanThreads];
    const int64_t per = (n_blocks + kScanThreads - 1) / kScanThreads;
    const int64_t lo = (int64_t)threadIdx.x * per;
    const int64_t hi = lo + per < n_blocks ? lo + per : n_blocks;
    int64_t s = 0;
    for (int64_t b = lo; b < hi; ++b)
        s += block_counts[b];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t run = 0;
        for (int t = 0; t < kScanThreads; ++t) {
            const int64_t c = part[t];
            part[t] = run;
            run += c;
        }
        *total = run;
    }
    __syncthreads();
    int64_t run = part[threadIdx.x];
    for (int64_t b = lo; b < hi; ++b) {
        block_offsets[b] = run;
        run += block_counts[b];
    }
}

// kept items, in index order, to out[offset ..]; `rank_of` (may be NULL) gets every item's position or -1
__global__ void __launch_bounds__(kCompThreads) k_comp_write(const uint8_t *keep_bits, int64_t n,
                                                             const int64_t *block_offsets, int64_t capacity,
                                                             int32_t *out, int32_t *rank_of)
{
    __shared__ int wave_tot[kCompThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t i0 = (int64_t)blockIdx.x * kCompBlock + (int64_t)threadIdx.x * kCompPer;
    static_assert(kCompPer == 8, "one byte of verdicts per thread");
    const unsigned bits = i0 < n ? keep_bits[i0 / kCompPer] : 0u;
    bool keep[kCompPer];
#pragma unroll
    for (int u = 0; u < kCompPer; ++u)
        keep[u] = (bits >> u) & 1u;
    const int c = __popc(bits);
    int incl = c;  // inclusive scan over the wavefront
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off)
            incl += up;
    }
    if (lane == kWave - 1)
        wave_tot[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int w2 = 0; w2 < wave; ++w2)
        base += wave_tot[w2];
    int64_t pos = block_offsets[blockIdx.x] + base + incl - c;
#pragma unroll
    for (int u = 0; u < kCompPer; ++u) {
        if (i0 + u < n) {
            if (keep[u]) {
                if (out && pos < capacity)
                    out[pos] = (int32_t)(i0 + u);
                if (rank_of)
                    rank_of[i0 + u] = (int32_t)pos;
                ++pos;
            } else if (rank_of) {
                rank_of[i0 + u] = -1;
            }
        }
    }
}

__global__ void k_pac_gather(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                             const double *__restrict__ ts, const float *__restrict__ feat, int F,
                             const int32_t *__restrict__ eid, int64_t n, const int32_t *__restrict__ local,
                             int32_t *src_out, int32_t *dst_out, double *ts_out, float *feat_out)
{
    // one wavefront per event and turn: the feature row is copied by its lanes (a grid of one wavefront
    // per event would pass 2^32 threads beyond 67 M events, which a dispatch cannot express)
    const int64_t n_waves = (int64_t)gridDim.x * (blockDim.x / kWave);
    const int lane = threadIdx.x & (kWave - 1);
    for (int64_t w = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave; w < n; w += n_waves) {
        const int64_t e = eid[w];
        if (lane == 0) {
            src_out[w] = local[src[e]];
            dst_out[w] = local[dst[e]];
            ts_out[w] = ts[e];
        }
        for (int j = lane; j < F; j += kWave)
            feat_out[w * F + j] = feat[e * F + j];
    }
}

__global__ void __launch_bounds__(256) k_sync_shared(SyncArgs a)
{
    const int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    if (s >= a.n_shared)
        return;
    int32_t row[kMaxSyncParts];
    double t_star = 0.0;
    int win = -1;
    for (int k = 0; k < a.n_parts; ++k) {
        row[k] = a.ids[k][s];
        if (row[k] < 0 || (int64_t)row[k] >= a.num_nodes[k])
            return;  // not a row of that partition: the node is left alone everywhere
    }
    for (int k = 0; k < a.n_parts; ++k) {
        const double t = a.lu[k][row[k]];
        if (win < 0 || t > t_star) {  // the lowest partition among equal times
            t_star = t;
            win = k;
        }
    }
    for (int j = lane; j < a.M; j += kWave) {
        float v;
        if (a.mode == 0) {
            v = a.mem[win][(size_t)row[win] * a.M + j];
        } else {
            v = a.mem[0][(size_t)row[0] * a.M + j];
            for (int k = 1; k < a.n_parts; ++k)
                v += a.mem[k][(size_t)row[k] * a.M + j];
            v /= (float)a.n_parts;
        }
        for (int k = 0; k < a.n_parts; ++k)
            a.mem[k][(size_t)row[k] * a.M + j] = v;
    }
    if (lane == 0)
        for (int k = 0; k < a.n_parts; ++k)
            a.lu[k][row[k]] = t_star;
}

struct CompScratch {
    int32_t *block_counts;
    int64_t *block_offsets;
    int64_t *total;
    uint8_t *keep_bits;
    size_t bytes;
};

CompScratch comp_scratch(int64_t n_max, void *base)
{
    const int64_t nb = (n_max + kCompBlock - 1) / kCompBlock + 1;
    CompScratch c;
    char *p = (char *)base;
    size_t off = 0;
    c.block_counts = base ? (int32_t *)(p + off) : nullptr;
    off += align_up(4 * (size_t)nb);
    c.block_offsets = base ? (int64_t *)(p + off) : nullptr;
    off += align_up(8 * (size_t)nb);
    c.total = base ? (int64_t *)(p + off) : nullptr;
    off += 256;
    c.keep_bits = base ? (uint8_t *)(p + off) : nullptr;
    off += align_up((size_t)nb * kCompThreads);  // one byte per thread of every workgroup
    c.bytes = off;
    return c;
}

template <class Pred>
hipError_t compact(Pred pred, int64_t n, const CompScratch &c, int64_t capacity, int32_t *out, int32_t *rank_of,
                   int64_t *total_host, hipStream_t s)
{
    const int64_t nb = (n + kCompBlock - 1) / kCompBlock;
    if (nb == 0) {
        *total_host = 0;
        return hipSuccess;
    }
    hipLaunchKernelGGL(k_comp_count<Pred>, dim3((unsigned)nb), dim3(kCompThreads), 0, s, pred, n, c.block_counts,
                       c.keep_bits);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(k_comp_scan, dim3(1), dim3(kScanThreads), 0, s, c.block_counts, nb, c.block_offsets, c.total);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    hipLaunchKernelGGL(k_comp_write, dim3((unsigned)nb), dim3(kCompThreads), 0, s, c.keep_bits, n, c.block_offsets,
                       capacity, out, rank_of);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    e = hipMemcpyAsync(total_host, c.total, sizeof(int64_t), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess)
        e = hipStreamSynchronize(s);
    return e;
}

}  // namespace

hipError_t launch_sync_shared(const SyncArgs &a, hipStream_t s)
{
    if (a.n_shared == 0)
        return hipSuccess;
    const int64_t blocks = (a.n_shared * kWave + 255) / 256;
    hipLaunchKernelGGL(k_sync_shared, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace tig

using namespace tig;

extern "C" {

size_t tig_pac_scratch_bytes(int64_t num_events, int64_t num_nodes)
{
    if (num_events < 0 || num_nodes < 1)
        return 0;
    return comp_scratch(num_events > num_nodes ? num_events : num_nodes, nullptr).bytes;
}

int tig_pac_subgraph(const int32_t *src, const int32_t *dst, int64_t num_events, const uint64_t *node_parts,
                     int64_t num_nodes, uint64_t group, int32_t *eid_out, int32_t *local_out, int64_t *counts_out,
                     void *scratch, size_t scratch_bytes, void *hip_stream)
{
    if (num_events < 0 || num_events > 0x7FFFFFFF || num_nodes < 1 || num_nodes > 0x7FFFFFFF || !node_parts ||
        !local_out || !counts_out || !scratch || ((uintptr_t)scratch & 255) ||
        (num_events > 0 && (!src || !dst || !eid_out)))
        return TIG_EINVAL;
    if (scratch_bytes < tig_pac_scratch_bytes(num_events, num_nodes))
        return TIG_ENOSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    const CompScratch c = comp_scratch(num_events > num_nodes ? num_events : num_nodes, scratch);
    hipError_t e = compact(EventPred{src, dst, node_parts, num_nodes, group}, num_events, c, num_events, eid_out,
                           nullptr, &counts_out[0], s);
    if (e != hipSuccess)
        return fail_global("tig_pac_subgraph: event compaction", e);
    e = compact(NodePred{node_parts, num_nodes, group}, num_nodes, c, 0, nullptr, local_out, &counts_out[1], s);
    return e == hipSuccess ? TIG_OK : fail_global("tig_pac_subgraph: node compaction", e);
}

int tig_pac_gather(const int32_t *src, const int32_t *dst, const double *ts, const float *edge_feat, int32_t feat_dim,
                   const int32_t *eid, int64_t n, const int32_t *local, int32_t *src_out, int32_t *dst_out,
                   double *ts_out, float *feat_out, void *hip_stream)
{
    if (n < 0 || feat_dim < 1 || (n > 0 && (!src || !dst || !ts || !edge_feat || !eid || !local || !src_out ||
                                             !dst_out || !ts_out || !feat_out)))
        return TIG_EINVAL;
    if (n == 0)
        return TIG_OK;
    int64_t blocks = (n * kWave + 255) / 256;
    blocks = blocks > (1 << 20) ? (1 << 20) : blocks;  // (the kernel strides over the events)
    hipLaunchKernelGGL(k_pac_gather, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream, src, dst, ts,
                       edge_feat, (int)feat_dim, eid, n, local, src_out, dst_out, ts_out, feat_out);
    return hipGetLastError() == hipSuccess ? TIG_OK : TIG_EHIP;
}

int tig_pac_combine(const int32_t *order, int32_t num_parts, int32_t num_groups, uint64_t *group_masks_out)
{
    if (!order || !group_masks_out || num_parts < 1 || num_parts > 64 || num_groups < 1 || num_parts % num_groups)
        return TIG_EINVAL;
    uint64_t seen = 0;
    for (int i = 0; i < num_parts; ++i) {
        if (order[i] < 0 || order[i] >= num_parts || ((seen >> order[i]) & 1u))
            return TIG_EINVAL;  // not a permutation of the parts
        seen |= 1ull << order[i];
    }
    const int w = num_parts / num_groups;
    for (int g = 0; g < num_groups; ++g) {
        uint64_t m = 0;
        for (int i = g * w; i < (g + 1) * w; ++i)
            m |= 1ull << order[i];
        group_masks_out[g] = m;
    }
    return TIG_OK;
}

}  // extern "C"
