// Streaming edge partitioner (paper Sec. II-B, Alg. 1): the preprocessing step that cuts a
// temporal interaction graph into the per-GPU sub-graphs the batch step runs on.  gfx950 only.
//   k_centrality   Eq. 1 on the device: Cent(i) = sum over i's events of exp(beta (t - t_max)).
//                  One pass over the event stream (16 bytes per event); every workgroup merges
//                  its chunk's contributions per node in LDS first (a hub node takes part in a
//                  large share of all events, and same-address device atomics serialise), then
//                  adds one fp64 value per distinct node and workgroup to the node array.
//   top-k hubs     the floor(k |V|) nodes of greatest centrality, ties towards the smaller id:
//                  a stable descending radix sort of (centrality bits, node id) pairs.
//   assign         the edge loop of Alg. 1 (cases 1-5, score C = C_REP + C_BAL, Eq. 2-6).  Every
//                  decision depends on all earlier ones, so this part is sequential by
//                  definition and runs on the host.
#include <hip/hip_runtime.h>
#include <rocprim/device/device_radix_sort.hpp>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "tig_internal.h"

namespace tig {

namespace {

constexpr int kCentThreads = 512;
constexpr int kCentPerThread = 128;                        // events per thread
constexpr int kCentChunk = kCentThreads * kCentPerThread;  // events per workgroup
constexpr int kCentSlots = 4096;                           // LDS table: node id + fp64 sum per slot
constexpr int kCentProbes = 8;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

__device__ inline double wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}

// Adds w to node's sum in the workgroup's LDS table; a node that finds no slot within a few
// probes goes straight to the node array.
__device__ inline void table_add(int32_t *t_node, double *t_sum, double *cent, int32_t node, double w)
{
    uint32_t h = ((uint32_t)node * 2654435761u) >> 20;  // 12 bits
    for (int probe = 0; probe < kCentProbes; ++probe) {
        const int32_t prev = atomicCAS(&t_node[h], -1, node);
        if (prev == -1 || prev == node) {
            atomicAdd(&t_sum[h], w);
            return;
        }
        h = (h + 1) & (kCentSlots - 1);
    }
    unsafeAtomicAdd(&cent[node], w);
}

// The lanes of a wavefront that hold the node of the first active lane hand their sum to that
// lane and drop out (two rounds: the heaviest nodes of a power-law stream fill most lanes).
__device__ inline void merge_heavy(bool &active, int32_t node, double &w)
{
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        const unsigned long long todo = __ballot(active);
        if (todo == 0ull)
            break;
        const int first = __ffsll((long long)todo) - 1;
        const int32_t n0 = __builtin_amdgcn_readlane(node, first);
        const bool mine = active && node == n0;
        const unsigned long long grp = __ballot(mine);
        if (__popcll(grp) > 1) {  // uniform
            const double s = wave_sum_f64(mine ? w : 0.0);
            if (mine) {
                if ((int)(threadIdx.x & 63) == first)
                    w = s;
                else
                    active = false;
            }
        }
    }
}

__global__ void __launch_bounds__(kCentThreads)
k_centrality(const int32_t *__restrict__ src, const int32_t *__restrict__ dst, const double *__restrict__ ts,
             int64_t num_events, int64_t num_nodes, double beta, double t_max, double *__restrict__ cent)
{
    __shared__ int32_t t_node[kCentSlots];
    __shared__ double t_sum[kCentSlots];
    for (int i = threadIdx.x; i < kCentSlots; i += kCentThreads) {
        t_node[i] = -1;
        t_sum[i] = 0.0;
    }
    __syncthreads();
    const int64_t e0 = (int64_t)blockIdx.x * kCentChunk;
    for (int it = 0; it < kCentPerThread; ++it) {
        const int64_t e = e0 + (int64_t)it * kCentThreads + threadIdx.x;  // coalesced
        const bool in = e < num_events;
        int32_t s = 0, d = 0;
        double w = 0.0;
        if (in) {
            s = src[e];
            d = dst[e];
            w = exp(beta * (ts[e] - t_max));
        }
        // ids were validated by the caller's graph checks or are checked here: out-of-range ids are skipped
        bool as = in && s >= 0 && (int64_t)s < num_nodes, ad = in && d >= 0 && (int64_t)d < num_nodes;
        double ws = w, wd = w;
        merge_heavy(as, s, ws);
        merge_heavy(ad, d, wd);
        if (as)
            table_add(t_node, t_sum, cent, s, ws);
        if (ad)
            table_add(t_node, t_sum, cent, d, wd);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kCentSlots; i += kCentThreads)
        if (t_node[i] >= 0)
            unsafeAtomicAdd(&cent[t_node[i]], t_sum[i]);
}

__global__ void k_topk_keys(const double *__restrict__ cent, int64_t n, unsigned long long *keys, uint32_t *vals)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        // centralities are sums of positive terms: for non-negative doubles the bit pattern orders like the value
        const double c = cent[i];
        keys[i] = c > 0.0 ? (unsigned long long)__double_as_longlong(c) : 0ull;
        vals[i] = (uint32_t)i;
    }
}

__global__ void k_topk_flags(const uint32_t *__restrict__ vals_sorted, int64_t n_hubs, int32_t *hubs, uint8_t *is_hub)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_hubs; i += stride) {
        hubs[i] = (int32_t)vals_sorted[i];
        is_hub[vals_sorted[i]] = 1;
    }
}

struct TopkLayout {
    unsigned long long *keys_in, *keys_out;
    uint32_t *vals_in, *vals_out;
    void *temp;
    size_t temp_bytes, bytes;
};

TopkLayout topk_layout(int64_t n, void *base)
{
    TopkLayout L;
    char *p = (char *)base;
    size_t off = 0;
    auto take = [&](size_t b) {
        char *q = base ? p + off : nullptr;
        off += align_up(b);
        return q;
    };
    L.keys_in = (unsigned long long *)take(8 * (size_t)n);
    L.keys_out = (unsigned long long *)take(8 * (size_t)n);
    L.vals_in = (uint32_t *)take(4 * (size_t)n);
    L.vals_out = (uint32_t *)take(4 * (size_t)n);
    L.temp_bytes = 0;
    (void)rocprim::radix_sort_pairs_desc(nullptr, L.temp_bytes, (unsigned long long *)nullptr,
                                         (unsigned long long *)nullptr, (uint32_t *)nullptr, (uint32_t *)nullptr,
                                         (size_t)n, 0, 64, (hipStream_t)0);
    L.temp = take(L.temp_bytes);
    L.bytes = off;
    return L;
}

int grid_for(int64_t n, int threads)
{
    int64_t b = (n + threads - 1) / threads;
    return (int)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

}  // namespace

}  // namespace tig

using namespace tig;

extern "C" {

int tig_sep_centrality(const int32_t *src, const int32_t *dst, const double *ts, int64_t num_events,
                       int64_t num_nodes, double beta, double *cent_out, void *hip_stream)
{
    if (num_nodes < 1 || num_nodes > 0x7FFFFFFF || num_events < 0 || !cent_out || !(beta >= 0.0))
        return TIG_EINVAL;
    if (num_events > 0 && (!src || !dst || !ts))
        return TIG_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = launch_fill_zero(cent_out, sizeof(double) * (size_t)num_nodes, s);
    if (e != hipSuccess)
        return TIG_EHIP;
    if (num_events == 0)
        return TIG_OK;
    // the stream is chronological: the last event carries t_max
    double t_max = 0.0;
    if (hipMemcpyAsync(&t_max, ts + (num_events - 1), sizeof(double), hipMemcpyDefault, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return TIG_EHIP;
    const int64_t blocks = (num_events + kCentChunk - 1) / kCentChunk;
    hipLaunchKernelGGL(k_centrality, dim3((unsigned)blocks), dim3(kCentThreads), 0, s, src, dst, ts, num_events,
                       num_nodes, beta, t_max, cent_out);
    return hipGetLastError() == hipSuccess ? TIG_OK : TIG_EHIP;
}

size_t tig_sep_topk_scratch_bytes(int64_t num_nodes)
{
    if (num_nodes < 1 || num_nodes > 0x7FFFFFFF)
        return 0;
    return topk_layout(num_nodes, nullptr).bytes;
}

int tig_sep_top_k(const double *cent, int64_t num_nodes, int64_t n_hubs, int32_t *hubs_out, uint8_t *is_hub_out,
                  void *scratch, size_t scratch_bytes, void *hip_stream)
{
    if (!cent || !is_hub_out || num_nodes < 1 || num_nodes > 0x7FFFFFFF || n_hubs < 0 || n_hubs > num_nodes ||
        (n_hubs > 0 && !hubs_out) || !scratch || ((uintptr_t)scratch & 255))
        return TIG_EINVAL;
    const TopkLayout L = topk_layout(num_nodes, scratch);
    if (scratch_bytes < L.bytes)
        return TIG_ENOSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    if (hipMemsetAsync(is_hub_out, 0, (size_t)num_nodes, s) != hipSuccess)
        return TIG_EHIP;
    if (n_hubs == 0)
        return TIG_OK;
    hipLaunchKernelGGL(k_topk_keys, dim3(grid_for(num_nodes, 256)), dim3(256), 0, s, cent, num_nodes, L.keys_in,
                       L.vals_in);
    size_t temp_bytes = L.temp_bytes;
    if (rocprim::radix_sort_pairs_desc(L.temp, temp_bytes, L.keys_in, L.keys_out, L.vals_in, L.vals_out,
                                       (size_t)num_nodes, 0, 64, s) != hipSuccess)
        return TIG_EHIP;
    hipLaunchKernelGGL(k_topk_flags, dim3(grid_for(n_hubs, 256)), dim3(256), 0, s, L.vals_out, n_hubs, hubs_out,
                       is_hub_out);
    return hipGetLastError() == hipSuccess ? TIG_OK : TIG_EHIP;
}

#pragma clang fp contract(off)
int tig_sep_assign(const tig_sep_config *cfg, const int32_t *src, const int32_t *dst, int64_t num_events,
                   int64_t num_nodes, const double *cent, const uint8_t *is_hub, int32_t *edge_part_out,
                   uint64_t *node_parts_out, int64_t *part_edges_out)
{
    if (!cfg || cfg->struct_size != sizeof(tig_sep_config) || cfg->num_parts < 1 || cfg->num_parts > 64 ||
        !(cfg->lambda > 0.0) || !(cfg->epsilon > 0.0))
        return TIG_EINVAL;
    if (num_nodes < 1 || num_events < 0 || !cent || !is_hub || !node_parts_out || !part_edges_out ||
        (num_events > 0 && (!src || !dst || !edge_part_out)))
        return TIG_EINVAL;
    const int P = cfg->num_parts;
    const double lam = cfg->lambda, eps = cfg->epsilon;
    for (int64_t i = 0; i < num_nodes; ++i)
        node_parts_out[i] = 0;
    int64_t sizes[64];
    for (int p = 0; p < P; ++p)
        sizes[p] = 0;
    int64_t mx = 0, mn = 0;
    uint64_t *A = node_parts_out;

    // arg max over all partitions of C(i, j, p) = C_REP + C_BAL (Eq. 3), lowest index among equals
    auto best = [&](int64_t i, int64_t j) -> int {
        const double tot = cent[i] + cent[j];
        const double th_i = tot == 0.0 ? 0.5 : cent[i] / tot;
        const double th_j = tot == 0.0 ? 0.5 : cent[j] / tot;
        const double h_i = 1.0 + (1.0 - th_i), h_j = 1.0 + (1.0 - th_j);  // Eq. 5
        const double den = (eps + (double)mx) - (double)mn;
        int arg = 0;
        double top = 0.0;
        for (int p = 0; p < P; ++p) {
            const double c_rep = (((A[i] >> p) & 1u) ? h_i : 0.0) + (((A[j] >> p) & 1u) ? h_j : 0.0);  // Eq. 4
            const double c_bal = lam * (double)(mx - sizes[p]) / den;                                  // Eq. 6
            const double c = c_rep + c_bal;
            if (p == 0 || c > top) {
                top = c;
                arg = p;
            }
        }
        return arg;
    };
    auto only = [](uint64_t mask) -> int { return __builtin_ctzll(mask); };

    for (int64_t e = 0; e < num_events; ++e) {
        const int64_t i = src[e], j = dst[e];
        if (i < 0 || i >= num_nodes || j < 0 || j >= num_nodes)
            return TIG_ERANGE;
        const bool hi = is_hub[i] != 0, hj = is_hub[j] != 0;
        int p;
        if (A[i] && A[j]) {
            if (hi != hj)                                 // Case 1: where the non-hub resides
                p = only(hi ? A[j] : A[i]);
            else if (hi)                                  // Case 2
                p = best(i, j);
            else                                          // Case 3
                p = A[i] == A[j] ? only(A[i]) : -1;
        } else {                                          // Case 4 & 5
            if (A[i] && !hi)
                p = only(A[i]);                           // a resident non-hub is not replicated
            else if (A[j] && !hj)
                p = only(A[j]);
            else
                p = best(i, j);
        }
        edge_part_out[e] = p;
        if (p >= 0) {
            A[i] |= 1ull << p;
            A[j] |= 1ull << p;
            const bool was_min = sizes[p] == mn;
            ++sizes[p];
            if (sizes[p] > mx)
                mx = sizes[p];
            if (was_min) {
                mn = sizes[0];
                for (int q = 1; q < P; ++q)
                    mn = sizes[q] < mn ? sizes[q] : mn;
            }
        }
    }
    for (int p = 0; p < P; ++p)
        part_edges_out[p] = sizes[p];
    return TIG_OK;
}

size_t tig_sep_scratch_bytes(int64_t num_nodes)
{
    const size_t t = tig_sep_topk_scratch_bytes(num_nodes);
    if (t == 0)
        return 0;
    // [centrality | hub flags | hub list | top-k scratch]
    return align_up(8 * (size_t)num_nodes) + align_up((size_t)num_nodes) + align_up(4 * (size_t)num_nodes) + t;
}

int tig_sep_partition(const tig_sep_config *cfg, const int32_t *src, const int32_t *dst, const double *ts,
                      int64_t num_events, int64_t num_nodes, void *scratch, size_t scratch_bytes, void *hip_stream,
                      double *cent_out, uint8_t *is_hub_out, int32_t *edge_part_out, uint64_t *node_parts_out,
                      int64_t *part_edges_out)
{
    if (!cfg || cfg->struct_size != sizeof(tig_sep_config) || !(cfg->top_k >= 0.0) || !(cfg->top_k <= 1.0) ||
        !cent_out || !is_hub_out || !scratch || ((uintptr_t)scratch & 255))
        return TIG_EINVAL;
    const size_t need = tig_sep_scratch_bytes(num_nodes);
    if (need == 0)
        return TIG_EINVAL;
    if (scratch_bytes < need)
        return TIG_ENOSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *base = (char *)scratch;
    double *cent_d = (double *)base;
    uint8_t *hub_d = (uint8_t *)(base + align_up(8 * (size_t)num_nodes));
    int32_t *list_d = (int32_t *)((char *)hub_d + align_up((size_t)num_nodes));
    void *topk = (char *)list_d + align_up(4 * (size_t)num_nodes);
    int rc = tig_sep_centrality(src, dst, ts, num_events, num_nodes, cfg->beta, cent_d, hip_stream);
    if (rc != TIG_OK)
        return rc;
    const int64_t n_hubs = (int64_t)std::floor(cfg->top_k * (double)num_nodes);
    rc = tig_sep_top_k(cent_d, num_nodes, n_hubs, list_d, hub_d, topk, tig_sep_topk_scratch_bytes(num_nodes),
                       hip_stream);
    if (rc != TIG_OK)
        return rc;
    std::vector<int32_t> hs, hd;
    try {
        hs.resize((size_t)num_events);
        hd.resize((size_t)num_events);
    } catch (const std::bad_alloc &) {
        return TIG_ENOMEM;
    }
    if (hipMemcpyAsync(cent_out, cent_d, 8 * (size_t)num_nodes, hipMemcpyDefault, s) != hipSuccess ||
        hipMemcpyAsync(is_hub_out, hub_d, (size_t)num_nodes, hipMemcpyDefault, s) != hipSuccess ||
        (num_events > 0 &&
         (hipMemcpyAsync(hs.data(), src, 4 * (size_t)num_events, hipMemcpyDefault, s) != hipSuccess ||
          hipMemcpyAsync(hd.data(), dst, 4 * (size_t)num_events, hipMemcpyDefault, s) != hipSuccess)) ||
        hipStreamSynchronize(s) != hipSuccess)
        return TIG_EHIP;
    return tig_sep_assign(cfg, hs.data(), hd.data(), num_events, num_nodes, cent_out, is_hub_out, edge_part_out,
                          node_parts_out, part_edges_out);
}

}  // extern "C"
