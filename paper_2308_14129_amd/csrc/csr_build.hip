// Graph validation and construction of the temporal adjacency (once, in tig_init).
//
// The history of a node before time t (the set E_t of the paper's Notations section restricted
// to the node) must be searchable by time.  Events arrive in chronological order, so listing
// every event under both of its endpoints in event-id order yields per-node lists that are
// already ordered by (time, event id).  A stable radix sort of the 2E (endpoint, entry) pairs
// by endpoint id produces exactly that grouping.
#include <cstring>

#include <hip/hip_runtime.h>
#include <rocprim/device/device_radix_sort.hpp>

#include "tig_internal.h"

namespace tig {

namespace {

constexpr int kThreads = 256;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

__global__ void k_validate(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                           const double *__restrict__ ts, int64_t num_events, int64_t num_nodes,
                           int32_t *flags)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < num_events; e += stride) {
        const int32_t s = src[e], d = dst[e];
        if (s < 0 || s >= num_nodes || d < 0 || d >= num_nodes)
            flags[0] = 1;
        if (e > 0 && !(ts[e - 1] <= ts[e]))
            flags[1] = 1;
        if (s == d)
            flags[2] = 1;
    }
}

__global__ void k_fill_pairs(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                             int64_t num_entries, uint32_t *__restrict__ keys,
                             uint32_t *__restrict__ vals)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < num_entries; i += stride) {
        const int64_t e = i >> 1;
        keys[i] = (uint32_t)((i & 1) ? dst[e] : src[e]);
        vals[i] = (uint32_t)i;
    }
}

__global__ void k_fill_csr(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                           const double *__restrict__ ts, int64_t num_entries,
                           const uint32_t *__restrict__ vals_sorted, CsrEntry *__restrict__ csr,
                           int32_t *__restrict__ pos)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < num_entries; p += stride) {
        const uint32_t i = vals_sorted[p];
        const int32_t e = (int32_t)(i >> 1);
        CsrEntry ent;
        ent.nbr = (i & 1) ? src[e] : dst[e];
        ent.eid = e;
        ent.ts = ts[e];
        csr[p] = ent;
        pos[i] = (int32_t)p;  // where entry 2*eid + role sits in the adjacency array
    }
}

// indptr[n] = number of sorted keys smaller than n, n = 0..N
__global__ void k_indptr(const uint32_t *__restrict__ keys_sorted, int64_t num_entries,
                         int64_t num_nodes, int64_t *__restrict__ indptr)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; n <= num_nodes; n += stride) {
        int64_t lo = 0, hi = num_entries;
        while (lo < hi) {
            const int64_t mid = lo + ((hi - lo) >> 1);
            if ((int64_t)keys_sorted[mid] < n)
                lo = mid + 1;
            else
                hi = mid;
        }
        indptr[n] = lo;
    }
}

int grid_for(int64_t n)
{
    int64_t g = (n + kThreads - 1) / kThreads;
    if (g < 1)
        g = 1;
    if (g > 65536)
        g = 65536;
    return (int)g;
}

int key_bits(int64_t num_nodes)
{
    int bits = 1;
    while (bits < 32 && ((int64_t)1 << bits) < num_nodes)
        ++bits;
    return bits;
}

// Upper bound on rocPRIM's temporary storage for the in-place (double-buffer) pair sort: its
// per-block digit counters.  Checked against the real requirement in csr_build.
size_t sort_temp_bound(int64_t num_entries) { return (size_t)num_entries * 4 + ((size_t)64 << 20); }

}  // namespace

hipError_t launch_validate_graph(const int32_t *src, const int32_t *dst, const double *ts,
                                 int64_t num_events, int64_t num_nodes, int32_t *flags,
                                 hipStream_t s)
{
    hipLaunchKernelGGL(k_validate, dim3(grid_for(num_events)), dim3(kThreads), 0, s, src, dst, ts,
                       num_events, num_nodes, flags);
    return hipGetLastError();
}

size_t csr_build_scratch_bytes(int64_t num_events, int64_t num_nodes)
{
    (void)num_nodes;
    const int64_t n2 = 2 * num_events;
    if (n2 == 0)
        return 256;
    return 4 * align_up(sizeof(uint32_t) * (size_t)n2) + align_up(sort_temp_bound(n2));
}

hipError_t csr_build(const int32_t *src, const int32_t *dst, const double *ts, int64_t num_events,
                     int64_t num_nodes, int64_t *indptr, CsrEntry *csr, int32_t *pos, void *scratch,
                     size_t scratch_bytes, hipStream_t s)
{
    const int64_t n2 = 2 * num_events;
    if (n2 == 0)
        return launch_fill_zero(indptr, sizeof(int64_t) * (size_t)(num_nodes + 1), s);
    if (scratch_bytes < csr_build_scratch_bytes(num_events, num_nodes))
        return hipErrorInvalidValue;
    const int bits = key_bits(num_nodes);
    const size_t seg = align_up(sizeof(uint32_t) * (size_t)n2);
    char *base = (char *)scratch;
    rocprim::double_buffer<uint32_t> keys((uint32_t *)(base), (uint32_t *)(base + seg));
    rocprim::double_buffer<uint32_t> vals((uint32_t *)(base + 2 * seg), (uint32_t *)(base + 3 * seg));
    void *temp = base + 4 * seg;
    size_t temp_bytes = 0;
    hipError_t err = rocprim::radix_sort_pairs(nullptr, temp_bytes, keys, vals, (size_t)n2, 0u,
                                               (unsigned)bits, s);
    if (err != hipSuccess)
        return err;
    if (temp_bytes > sort_temp_bound(n2))
        return hipErrorOutOfMemory;

    hipLaunchKernelGGL(k_fill_pairs, dim3(grid_for(n2)), dim3(kThreads), 0, s, src, dst, n2,
                       keys.current(), vals.current());
    err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    // stable: entries of one node keep their input order, i.e. ascending event id
    err = rocprim::radix_sort_pairs(temp, temp_bytes, keys, vals, (size_t)n2, 0u, (unsigned)bits, s);
    if (err != hipSuccess)
        return err;
    hipLaunchKernelGGL(k_fill_csr, dim3(grid_for(n2)), dim3(kThreads), 0, s, src, dst, ts, n2,
                       (const uint32_t *)vals.current(), csr, pos);
    err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    hipLaunchKernelGGL(k_indptr, dim3(grid_for(num_nodes + 1)), dim3(kThreads), 0, s,
                       (const uint32_t *)keys.current(), n2, num_nodes, indptr);
    return hipGetLastError();
}

}  // namespace tig
