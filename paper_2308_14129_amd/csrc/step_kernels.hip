// The kernels of one batch step (paper Sec. II-C, "Training approach for TIGs"), gfx950 only.
//
//   k_pre           two jobs in one launch: last-message aggregation (64-bit (time, event id)
//                   atomicMax per node) and most-recent-K temporal neighbours (one wavefront
//                   per query, 64-way search)
//   k_select        winners = entries whose key survived; compacted list
//   k_gru           message gather + time encoding -> LDS tile -> MFMA gate GEMMs -> new rows
//   k_commit        memory overwrite M <- s_i(t), last_update, key clear
//   k_embed         attention over neighbours (folded projections), merge MLP, link decoder
//
// Tile GEMM convention (16x16 output tiles on the matrix cores, wave64):
//   operand A: activations in LDS, row-major; lane l supplies row l%16 and KB/4 consecutive k's
//              starting at k0 + (KB/4)*(l/16);
//   operand B: prepared weights, already lane-ordered in global memory (pack.hip);
//   result   : lane l holds rows 4*(l/16)+v (v = 0..3) of column l%16.
#include <hip/hip_runtime.h>

#include "tig_internal.h"

namespace tig {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr int kTileThreads = 512;  // 8 wavefronts per tile workgroup
constexpr int kTileWaves = kTileThreads / kWave;
constexpr int kMaxHeads = 4;

template <int PREC>
struct Prec;

// fp32 operands: one k-block = 16 k's = four 16x16x4 MFMAs fed by one 16-byte load per lane.
template <>
struct Prec<TIG_FP32> {
    struct frag {
        floatx4 v;
    };
    static constexpr int KB = 16;
    // activation element k of an LDS row
    static __device__ inline void store_a(char *row, int k, float v) { ((float *)row)[k] = v; }
    // lane's operand of k-block kb: 4 consecutive k's starting at kb*16 + 4*g, g = lane/16
    static __device__ inline frag load_a(const char *row, int kb, int g)
    {
        return frag{*(const floatx4 *)(row + (size_t)(kb * 16 + 4 * g) * 4)};
    }
    static __device__ inline frag load_w(const void *W, size_t idx) { return frag{((const floatx4 *)W)[idx]}; }
    static __device__ inline void mma(floatx4 &acc, const frag &a, const frag &b)
    {
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[0], b.v[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[1], b.v[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[2], b.v[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[3], b.v[3], acc, 0, 0, 0);
    }
};

// bf16 matrix cores with split operands: x = hi + lo, hi = bf16(x), lo = bf16(x - hi), for
// activations and weights alike; a*w ~ a_hi*w_hi + a_lo*w_hi + a_hi*w_lo (the dropped lo*lo term
// is ~2^-18 relative), accumulated in fp32.  One k-block = 32 k's = three 16x16x32 MFMAs.
// Storage: groups of 8 k's, 8 hi values (16 bytes) followed by their 8 lo values (16 bytes), so
// an element still takes 4 bytes and a lane's operand is one contiguous 32-byte read.
template <>
struct Prec<TIG_BF16_MFMA> {
    struct frag {
        bf16x8 hi, lo;
    };
    static constexpr int KB = 32;
    static __device__ inline uint16_t bf16_rne(float v)
    {
        uint32_t u = __float_as_uint(v);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    static __device__ inline void store_a(char *row, int k, float v)
    {
        uint16_t *p = (uint16_t *)row + ((k >> 3) << 4) + (k & 7);
        const uint16_t hi = bf16_rne(v);
        p[0] = hi;
        p[8] = bf16_rne(v - __uint_as_float((uint32_t)hi << 16));
    }
    static __device__ inline frag load_a(const char *row, int kb, int g)
    {
        const char *p = row + (size_t)(kb * 4 + g) * 32;
        return frag{*(const bf16x8 *)p, *(const bf16x8 *)(p + 16)};
    }
    static __device__ inline frag load_w(const void *W, size_t idx)
    {
        const char *p = (const char *)W + idx * 32;
        return frag{*(const bf16x8 *)p, *(const bf16x8 *)(p + 16)};
    }
    static __device__ inline void mma(floatx4 &acc, const frag &a, const frag &b)
    {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.lo, b.hi, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.hi, b.lo, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.hi, b.hi, acc, 0, 0, 0);
    }
};

__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ inline int wave_id() { return threadIdx.x / kWave; }

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, kWave);
    return v;
}

template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ inline float dpp_or_zero(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, BANK_MASK, true));
}

// Sum over the 64 lanes, returned as a wave-uniform value: a prefix sum inside each row of 16
// lanes (row_shr 1, 2, 4, 8; lanes shifted in from outside the row read as 0), then the row
// totals are carried forward (row_bcast 15, row_bcast 31) so that lane 63 holds the total.
// All 64 lanes must be active.
__device__ inline float wave_sum_uniform(float v)
{
    v += dpp_or_zero<0x111, 0xf, 0xf>(v);
    v += dpp_or_zero<0x112, 0xf, 0xf>(v);
    v += dpp_or_zero<0x114, 0xf, 0xf>(v);
    v += dpp_or_zero<0x118, 0xf, 0xf>(v);
    v += dpp_or_zero<0x142, 0xa, 0xf>(v);
    v += dpp_or_zero<0x143, 0xc, 0xf>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Phi(x)_k = cos(w*x + b): argument and reduction to [-pi/4, pi/4] + quadrant in fp64 (the
// argument reaches ~1e6 rad, beyond fp32), polynomial in fp32 (truncation < 3e-8).
__device__ inline float time_enc(float w, float b, double x)
{
    const double arg = fma((double)w, x, (double)b);
    const double kd = rint(arg * 0.63661977236758134308);
    double r = fma(-kd, 1.57079632679489655800e+00, arg);
    r = fma(-kd, 6.12323399573676603587e-17, r);
    const int q = (int)((long long)kd) & 3;
    const float rf = (float)r;
    const float r2 = rf * rf;
    const float c = 1.0f + r2 * (-0.5f + r2 * (4.16666667e-2f + r2 * (-1.38888889e-3f + r2 * 2.48015873e-5f)));
    const float s = rf * (1.0f + r2 * (-1.66666667e-1f + r2 * (8.33333333e-3f + r2 * (-1.98412698e-4f + r2 * 2.75573192e-6f))));
    const float v = (q & 1) ? s : c;
    return (q == 1 || q == 2) ? -v : v;
}

// (time, event id, role) -> 64-bit key whose unsigned order is the lexicographic order of
// (float(time), event id).  Events are time-sorted, so this equals the (time, event id) order.
// Always non-zero for finite times; 0 means "no message for this node".
__device__ inline unsigned long long winner_key(double t, int32_t eid, int role)
{
    const uint32_t bits = __float_as_uint((float)t);
    const uint32_t mono = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return ((unsigned long long)mono << 32) | (unsigned long long)(((uint32_t)eid << 1) | (uint32_t)role);
}

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
// acc[mt] += A[16*mt .. 16*mt+15][0 .. kblocks*KB) x W[nt]^T.
// A: LDS rows of `lda` BYTES (4 bytes per element in either precision).  W: lane-ordered blocks,
// `w_kblocks` per output tile, starting at k-block `w_kb0`.
template <int PREC, int MT>
__device__ inline void tile_gemm(floatx4 (&acc)[MT], const char *A, int lda, const void *W,
                                 int w_kblocks, int w_kb0, int kblocks, int nt, int m_tiles)
{
    using P = Prec<PREC>;
    using frag = typename P::frag;
    const int lane = lane_id();
    const size_t w0 = ((size_t)nt * w_kblocks + w_kb0) * kWave + lane;
    const char *ap = A + (size_t)(lane & 15) * lda;
    const int g = lane >> 4;
    // weight operands come from L2: keep kPrefetch loads in flight ahead of the MFMAs
    constexpr int kPrefetch = 4;
    int kb = 0;
    for (; kb + kPrefetch <= kblocks; kb += kPrefetch) {
        frag bfrag[kPrefetch];
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u)
            bfrag[u] = P::load_w(W, w0 + (size_t)(kb + u) * kWave);
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (mt < m_tiles) {
                    const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, kb + u, g);
                    P::mma(acc[mt], afrag, bfrag[u]);
                }
            }
        }
    }
    for (; kb < kblocks; ++kb) {
        const frag bfrag = P::load_w(W, w0 + (size_t)kb * kWave);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt < m_tiles) {
                const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, kb, g);
                P::mma(acc[mt], afrag, bfrag);
            }
        }
    }
}

// Row stride in bytes >= 4*width whose 16-byte chunk count is odd: the 16 rows read by one
// operand load then fall into distinct LDS bank groups.
__host__ __device__ inline int lds_row_bytes(int width_elems)
{
    int chunks = (width_elems * 4 + 15) / 16;
    if ((chunks & 1) == 0)
        ++chunks;
    return chunks * 16;
}

// ------------------------------------------------------------------------------------------
// GRU memory update for the winners among 16*MT consecutive (event, role) entries.
struct GruParams {
    int M, T, F, Dmsg;
    int Kg, Khn, Ng;
    int ldx;  // LDS row stride of the message tile, bytes
};

template <int PREC, int MT>
__global__ void __launch_bounds__(kTileThreads)
k_gru(StepArgs a, PackedWeights w, GruParams g)
{
    using P = Prec<PREC>;
    constexpr int EC = 16 * MT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *row_entry = (int *)smem;            // [EC]
    char *X = smem + 512;                    // [EC rows x ldx bytes]

    const int lane = lane_id();
    const int wave = wave_id();

    // 1. this block's slice of the compacted winner list
    const int n_win = *a.n_win;
    const int r0 = blockIdx.x * EC;
    if (r0 >= n_win)
        return;
    const int n_rows = n_win - r0 < EC ? n_win - r0 : EC;
    if (threadIdx.x < n_rows)
        row_entry[threadIdx.x] = a.win_list[r0 + threadIdx.x];
    __syncthreads();
    const int m_tiles = (n_rows + 15) / 16;

    // 2. message rows [s_self | s_other | Phi(t - last_update[self]) | e] from batch-start memory
    for (int r = wave; r < m_tiles * 16; r += kTileWaves) {
        char *xr = X + (size_t)r * g.ldx;
        if (r < n_rows) {
            const int i = row_entry[r];
            const int64_t eid = a.first_eid + (i >> 1);
            const int role = i & 1;
            const int32_t s = a.src[eid], d = a.dst[eid];
            const int32_t u = role ? d : s, o = role ? s : d;
            const double dt = a.ts[eid] - a.lu[u];
            const float *mu = a.mem + (size_t)u * g.M;
            const float *mo = a.mem + (size_t)o * g.M;
            const float *ef = a.edge_feat + (size_t)eid * g.F;
            for (int j = lane; j < g.Kg; j += kWave) {
                float v = 0.0f;
                if (j < g.M)
                    v = mu[j];
                else if (j < 2 * g.M)
                    v = mo[j - g.M];
                else if (j < 2 * g.M + g.T)
                    v = time_enc(w.time_w[j - 2 * g.M], w.time_b[j - 2 * g.M], dt);
                else if (j < g.Dmsg)
                    v = ef[j - 2 * g.M - g.T];
                P::store_a(xr, j, v);
            }
        } else {
            for (int j = lane; j < g.Kg; j += kWave)
                P::store_a(xr, j, 0.0f);
        }
    }
    __syncthreads();

    // 3. gate pre-activations on the matrix cores; 4. gates and the new state
    const int kblocks = g.Kg / P::KB;
    const int kblocks_hn = g.Khn / P::KB;
    for (int ct = wave; ct < g.Ng / 16; ct += kTileWaves) {
        floatx4 acc_r[MT], acc_z[MT], acc_in[MT], acc_hn[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc_r[mt] = floatx4{0, 0, 0, 0};
            acc_z[mt] = floatx4{0, 0, 0, 0};
            acc_in[mt] = floatx4{0, 0, 0, 0};
            acc_hn[mt] = floatx4{0, 0, 0, 0};
        }
        tile_gemm<PREC, MT>(acc_r, X, g.ldx, w.gru_Wr, kblocks, 0, kblocks, ct, m_tiles);
        tile_gemm<PREC, MT>(acc_z, X, g.ldx, w.gru_Wz, kblocks, 0, kblocks, ct, m_tiles);
        tile_gemm<PREC, MT>(acc_in, X, g.ldx, w.gru_Win, kblocks, 0, kblocks, ct, m_tiles);
        tile_gemm<PREC, MT>(acc_hn, X, g.ldx, w.gru_Whn, kblocks_hn, 0, kblocks_hn, ct, m_tiles);
        const int col = ct * 16 + (lane & 15);
        if (col < g.M) {
            const float br = w.gru_br[col], bz = w.gru_bz[col], bin = w.gru_bin[col], bhn = w.gru_bhn[col];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = mt * 16 + 4 * (lane >> 4) + v;
                    if (row < n_rows) {
                        const int i = row_entry[row];
                        const int64_t eid = a.first_eid + (i >> 1);
                        const int32_t u = (i & 1) ? a.dst[eid] : a.src[eid];
                        const float h = a.mem[(size_t)u * g.M + col];
                        const float r = 1.0f / (1.0f + expf(-(acc_r[mt][v] + br)));
                        const float z = 1.0f / (1.0f + expf(-(acc_z[mt][v] + bz)));
                        const float n = tanhf(acc_in[mt][v] + bin + r * (acc_hn[mt][v] + bhn));
                        a.staging[(size_t)i * g.M + col] = (1.0f - z) * n + z * h;
                    }
                }
            }
        }
    }
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

// ------------------------------------------------------------------------------------------
// Embedding + decoder for TE consecutive events x {source, destination, negative} query rows.
struct EmbedParams {
    int M, T, F, E, K, H;
    int dkv, dkvp, Mq, N1, K2, Ep, Ek;
    int TE;         // events per workgroup; rows = roles * TE <= 16 * MT
    int row_bytes;  // LDS bytes per query row of the main buffer
    int mem_off;    // byte offset of the s_u operand inside a row
    int ld1;        // row stride of the E-wide buffers, bytes
    int off_h1, off_meta;  // byte offsets in LDS
    int dec_off;    // byte offset of the decoder pre-activations (inside the main buffer)
};

template <int PREC, int MT, int NPL>
__global__ void __launch_bounds__(kTileThreads)
k_embed(StepArgs a, PackedWeights w, EmbedParams p)
{
    using P = Prec<PREC>;
    constexpr int ROWS = 16 * MT;
    constexpr int KC = (64 / NPL) < 16 ? (64 / NPL) : 16;  // neighbour rows in flight per chunk
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *rowbuf = smem;
    char *h1buf = smem + p.off_h1;
    int *row_q = (int *)(smem + p.off_meta);  // [ROWS] query index or -1
    int *row_cnt = row_q + ROWS;              // [ROWS]
    int *row_node = row_cnt + ROWS;           // [ROWS]

    const int lane = lane_id();
    const int wave = wave_id();
    const int ev0 = blockIdx.x * p.TE;

    // ---- A. query rows: node, query index, s_u (post-update memory) -------------------------
    for (int r = wave; r < ROWS; r += kTileWaves) {
        const int role = r / p.TE;
        const int b = ev0 + (r - role * p.TE);
        const bool act = role < a.roles && b < a.count;
        int32_t u = -1;
        int q = -1;
        if (act) {
            const int64_t eid = a.first_eid + b;
            u = role == 0 ? a.src[eid] : (role == 1 ? a.dst[eid] : a.neg[b]);
            q = role * a.count + b;
        }
        const bool has_row = u >= 0 && (int64_t)u < a.num_nodes;
        char *mrow = rowbuf + (size_t)r * p.row_bytes + p.mem_off;
        for (int j = lane; j < p.Mq; j += kWave) {
            float v = 0.0f;
            if (has_row && j < p.M)
                v = a.mem[(size_t)u * p.M + j];
            P::store_a(mrow, j, v);
        }
        if (lane == 0) {
            row_q[r] = q;
            row_node[r] = has_row ? u : -1;
            row_cnt[r] = act ? a.nbr_cnt[q] : 0;
        }
    }
    __syncthreads();

    // ---- B. folded query: q~ = A1 s_u + a1  (fp32, [H x dkvp] per row) -----------------------
    for (int nt = wave; nt < p.N1 / 16; nt += kTileWaves) {
        floatx4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[mt] = floatx4{0, 0, 0, 0};
        tile_gemm<PREC, MT>(acc, rowbuf + p.mem_off, p.row_bytes, w.emb_A1, p.Mq / P::KB, 0,
                            p.Mq / P::KB, nt, MT);
        const int col = nt * 16 + (lane & 15);
        const float bias = w.emb_a1[col];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = mt * 16 + 4 * (lane >> 4) + v;
                ((float *)(rowbuf + (size_t)row * p.row_bytes))[col] = acc[mt][v] + bias;
            }
    }
    __syncthreads();

    // ---- C. attention over the neighbours: scores <q~_h, kv_k>, softmax, kvbar_h = sum a_k kv_k
    {
        // per-lane view of the key/value row, kernel order [Phi (T) | s_v (M) | e (F) | 0]:
        // lane owns dims j = lane + 64 n.  (Time encoding first: its lanes are densely packed.)
        float tw[NPL], tb[NPL];
#pragma unroll
        for (int n = 0; n < NPL; ++n) {
            const int j = lane + kWave * n;
            tw[n] = j < p.T ? w.time_w[j] : 0.0f;
            tb[n] = j < p.T ? w.time_b[j] : 0.0f;
        }
        for (int r = wave; r < ROWS; r += kTileWaves) {
            const int q = row_q[r];
            if (q < 0)
                continue;
            const int cnt = row_cnt[r];
            float *qrow = (float *)(rowbuf + (size_t)r * p.row_bytes);
            char *arow = rowbuf + (size_t)r * p.row_bytes;
            float qv[kMaxHeads][NPL], accv[kMaxHeads][NPL];
            float mx[kMaxHeads], den[kMaxHeads];
#pragma unroll
            for (int h = 0; h < kMaxHeads; ++h) {
                mx[h] = -INFINITY;
                den[h] = 0.0f;
#pragma unroll
                for (int n = 0; n < NPL; ++n) {
                    const int j = lane + kWave * n;
                    qv[h][n] = (h < p.H && j < p.dkvp) ? qrow[h * p.dkvp + j] : 0.0f;
                    accv[h][n] = 0.0f;
                }
            }
            // neighbour slot k lives in lane k
            int32_t nb_v = -1, nb_e = -1;
            double nb_t = 0.0;
            if (lane < cnt) {
                nb_v = a.nbr_node[(size_t)q * p.K + lane];
                nb_e = a.nbr_eid[(size_t)q * p.K + lane];
                nb_t = a.nbr_ts[(size_t)q * p.K + lane];
            }
            const int64_t eid_q = a.first_eid + (q % a.count);
            const double tq = a.ts[eid_q];
            const double dt_lane = tq - nb_t;
            for (int c0 = 0; c0 < cnt; c0 += KC) {
                float raw[KC][NPL];
                // issue every gather of the chunk before using any of them
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
                    const int k = c0 + kk;
                    const int32_t v = __shfl(nb_v, k & 63, kWave);
                    const int32_t e = __shfl(nb_e, k & 63, kWave);
#pragma unroll
                    for (int n = 0; n < NPL; ++n) {
                        const int j = lane + kWave * n - p.T;
                        float x = 0.0f;
                        if (k < cnt && j >= 0) {
                            if (j < p.M)
                                x = a.mem[(size_t)v * p.M + j];
                            else if (j < p.M + p.F)
                                x = a.edge_feat[(size_t)e * p.F + (j - p.M)];
                        }
                        raw[kk][n] = x;
                    }
                }
                // time encoding of t - t_k, then every score of the chunk (independent reductions)
                float sc[KC][kMaxHeads];
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
                    const int k = c0 + kk;
#pragma unroll
                    for (int h = 0; h < kMaxHeads; ++h)
                        sc[kk][h] = -INFINITY;
                    if (k < cnt) {  // wave-uniform
                        const double dt = __shfl(dt_lane, k & 63, kWave);
#pragma unroll
                        for (int n = 0; n < NPL; ++n) {
                            if (kWave * n < p.T) {  // uniform: this register holds Phi dims
                                if (lane + kWave * n < p.T)
                                    raw[kk][n] = time_enc(tw[n], tb[n], dt);
                            }
                        }
#pragma unroll
                        for (int h = 0; h < kMaxHeads; ++h) {
                            if (h < p.H) {  // uniform
                                float part = 0.0f;
#pragma unroll
                                for (int n = 0; n < NPL; ++n)
                                    part += qv[h][n] * raw[kk][n];
                                sc[kk][h] = wave_sum_uniform(part);
                            }
                        }
                    }
                }
                // softmax across the chunk, merged with earlier chunks by rescaling
#pragma unroll
                for (int h = 0; h < kMaxHeads; ++h) {
                    if (h < p.H) {
                        float mnew = mx[h];
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk)
                            mnew = fmaxf(mnew, sc[kk][h]);
                        const float corr = expf(mx[h] - mnew);  // first chunk: exp(-inf) = 0
                        float dsum = den[h] * corr;
#pragma unroll
                        for (int n = 0; n < NPL; ++n)
                            accv[h][n] *= corr;
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk) {
                            if (c0 + kk < cnt) {
                                const float pk = expf(sc[kk][h] - mnew);
                                dsum += pk;
#pragma unroll
                                for (int n = 0; n < NPL; ++n)
                                    accv[h][n] += pk * raw[kk][n];
                            }
                        }
                        den[h] = dsum;
                        mx[h] = mnew;
                    }
                }
            }
            // kvbar overwrites q~ in place (as matrix-core operand elements)
#pragma unroll
            for (int h = 0; h < kMaxHeads; ++h) {
                if (h < p.H) {
                    const float inv = cnt > 0 ? 1.0f / den[h] : 0.0f;
#pragma unroll
                    for (int n = 0; n < NPL; ++n) {
                        const int j = lane + kWave * n;
                        if (j < p.dkvp)
                            P::store_a(arow, h * p.dkvp + j, accv[h][n] * inv);
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- D. merge layer 1: h1 = relu(P kvbar + R s_u + c)   (c0 when there is no neighbour) ---
    for (int nt = wave; nt < p.Ep / 16; nt += kTileWaves) {
        floatx4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[mt] = floatx4{0, 0, 0, 0};
        const int kb1 = p.N1 / P::KB, kb2 = p.Mq / P::KB;
        tile_gemm<PREC, MT>(acc, rowbuf, p.row_bytes, w.emb_PR, kb1 + kb2, 0, kb1, nt, MT);
        tile_gemm<PREC, MT>(acc, rowbuf + p.mem_off, p.row_bytes, w.emb_PR, kb1 + kb2, kb1, kb2,
                            nt, MT);
        const int col = nt * 16 + (lane & 15);
        const float c = w.emb_c[col], c0 = w.emb_c0[col];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = mt * 16 + 4 * (lane >> 4) + v;
                const float x = acc[mt][v] + (row_cnt[row] > 0 ? c : c0);
                P::store_a(h1buf + (size_t)row * p.ld1, col, fmaxf(x, 0.0f));
            }
    }
    // k-depth padding of the E-wide buffers (columns Ep..Ek-1)
    for (int idx = threadIdx.x; idx < ROWS * (p.Ek - p.Ep); idx += kTileThreads) {
        const int row = idx / (p.Ek - p.Ep), col = p.Ep + idx % (p.Ek - p.Ep);
        P::store_a(h1buf + (size_t)row * p.ld1, col, 0.0f);
    }
    __syncthreads();

    // ---- E. merge layer 2: emb = W_m2 h1 + b_m2 -> global, and kept as the decoder operand ---
    char *embbuf = rowbuf;  // [ROWS rows x ld1 bytes], the main buffer is free again
    for (int nt = wave; nt < p.Ep / 16; nt += kTileWaves) {
        floatx4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[mt] = floatx4{0, 0, 0, 0};
        tile_gemm<PREC, MT>(acc, h1buf, p.ld1, w.emb_Wm2, p.Ek / P::KB, 0, p.Ek / P::KB, nt, MT);
        const int col = nt * 16 + (lane & 15);
        const float bias = w.emb_bm2[col];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = mt * 16 + 4 * (lane >> 4) + v;
                const float x = acc[mt][v] + bias;
                const int q = row_q[row];
                if (q >= 0 && col < p.E)
                    a.emb[(size_t)q * p.E + col] = x;
                P::store_a(embbuf + (size_t)row * p.ld1, col, x);
            }
    }
    for (int idx = threadIdx.x; idx < ROWS * (p.Ek - p.Ep); idx += kTileThreads) {
        const int row = idx / (p.Ek - p.Ep), col = p.Ep + idx % (p.Ek - p.Ep);
        P::store_a(embbuf + (size_t)row * p.ld1, col, 0.0f);
    }
    __syncthreads();

    // ---- F. decoder layer 1, split by operand: [W_a emb | W_b emb] for every row -------------
    float *decbuf = (float *)(rowbuf + p.dec_off);  // [ROWS x 2Ep]
    for (int nt = wave; nt < 2 * p.Ep / 16; nt += kTileWaves) {
        floatx4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[mt] = floatx4{0, 0, 0, 0};
        tile_gemm<PREC, MT>(acc, embbuf, p.ld1, w.dec_W, p.Ek / P::KB, 0, p.Ek / P::KB, nt, MT);
        const int col = nt * 16 + (lane & 15);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = mt * 16 + 4 * (lane >> 4) + v;
                decbuf[(size_t)row * 2 * p.Ep + col] = acc[mt][v];
            }
    }
    __syncthreads();

    // ---- G. logits: w_d2 . relu(W_a emb_src + W_b emb_other + b_d1) + b_d2 --------------------
    const int pairs = p.TE * (a.roles - 1);
    for (int pr = wave; pr < pairs; pr += kTileWaves) {
        const int which = pr / p.TE;  // 0: destination, 1: negative
        const int ev = pr - which * p.TE;
        const int b = ev0 + ev;
        if (b >= a.count)
            continue;
        const float *da = decbuf + (size_t)ev * 2 * p.Ep;
        const float *db = decbuf + (size_t)((which + 1) * p.TE + ev) * 2 * p.Ep + p.Ep;
        float part = 0.0f;
        for (int j = lane; j < p.E; j += kWave)
            part += w.dec_w2[j] * fmaxf(da[j] + db[j] + w.dec_b1[j], 0.0f);
        const float s = wave_sum(part) + w.dec_b2[0];
        if (lane == 0)
            (which == 0 ? a.score_pos : a.score_neg)[b] = s;
    }
}

__global__ void k_fill_zero(uint32_t *p, size_t words)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride)
        p[i] = 0u;
}

// ------------------------------------------------------------------------------------------
// host side: launch shapes

GruParams gru_params(const Dims &d)
{
    GruParams g;
    g.M = d.M;
    g.T = d.T;
    g.F = d.F;
    g.Dmsg = d.Dmsg;
    g.Kg = d.Kg;
    g.Khn = d.Khn;
    g.Ng = d.Ng;
    g.ldx = lds_row_bytes(d.Kg);
    return g;
}

int gru_lds_bytes(const Dims &d, int mt) { return 512 + 16 * mt * lds_row_bytes(d.Kg); }

EmbedParams embed_params(const Dims &d, int mt, int roles)
{
    EmbedParams p;
    p.M = d.M;
    p.T = d.T;
    p.F = d.F;
    p.E = d.E;
    p.K = d.K;
    p.H = d.H;
    p.dkv = d.dkv;
    p.dkvp = d.dkvp;
    p.Mq = d.Mq;
    p.N1 = d.N1;
    p.K2 = d.K2;
    p.Ep = d.Ep;
    p.Ek = d.Ek;
    const int rows = 16 * mt;
    p.TE = rows / roles;
    // main buffer row: q~ (fp32, N1) / kvbar (operand elements, N1) first, then s_u (Mq elements)
    p.mem_off = 4 * d.N1;
    p.row_bytes = lds_row_bytes(d.N1 + d.Mq);
    p.ld1 = lds_row_bytes(d.Ek);
    const int emb_bytes = rows * p.ld1;
    p.dec_off = (emb_bytes + 15) / 16 * 16;
    int main_bytes = rows * p.row_bytes;
    const int tail_bytes = p.dec_off + rows * 2 * d.Ep * 4;
    if (tail_bytes > main_bytes)
        main_bytes = tail_bytes;
    main_bytes = (main_bytes + 15) / 16 * 16;
    p.off_h1 = main_bytes;
    p.off_meta = p.off_h1 + rows * p.ld1;
    return p;
}

int embed_lds_bytes(const Dims &d, int mt)
{
    const EmbedParams p = embed_params(d, mt, 3);
    return p.off_meta + 3 * 16 * mt * 4;
}

int npl_for(const Dims &d)
{
    const int need = (d.dkvp + 63) / 64;
    int npl = 1;
    while (npl < need)
        npl *= 2;
    return npl;
}

template <int PREC, int MT>
const void *gru_fn() { return (const void *)k_gru<PREC, MT>; }

template <int PREC, int MT, int NPL>
const void *embed_fn() { return (const void *)k_embed<PREC, MT, NPL>; }

template <int PREC>
const void *gru_fn_mt(int mt)
{
    switch (mt) {
    case 1: return gru_fn<PREC, 1>();
    case 2: return gru_fn<PREC, 2>();
    case 3: return gru_fn<PREC, 3>();
    default: return gru_fn<PREC, 4>();
    }
}

template <int PREC, int MT>
const void *embed_fn_npl(int npl)
{
    switch (npl) {
    case 1: return embed_fn<PREC, MT, 1>();
    case 2: return embed_fn<PREC, MT, 2>();
    case 4: return embed_fn<PREC, MT, 4>();
    default: return embed_fn<PREC, MT, 8>();
    }
}

template <int PREC>
const void *embed_fn_mt(int mt, int npl)
{
    switch (mt) {
    case 1: return embed_fn_npl<PREC, 1>(npl);
    case 2: return embed_fn_npl<PREC, 2>(npl);
    default: return embed_fn_npl<PREC, 3>(npl);
    }
}

const void *gru_kernel(const Dims &d, int mt)
{
    return d.prec == TIG_BF16_MFMA ? gru_fn_mt<TIG_BF16_MFMA>(mt) : gru_fn_mt<TIG_FP32>(mt);
}

const void *embed_kernel(const Dims &d, int mt)
{
    const int npl = npl_for(d);
    return d.prec == TIG_BF16_MFMA ? embed_fn_mt<TIG_BF16_MFMA>(mt, npl) : embed_fn_mt<TIG_FP32>(mt, npl);
}

}  // namespace

bool plan_launch(const Dims &d, int lds_limit, LaunchPlan *plan)
{
    if (d.dkvp > 512)
        return false;
    // GRU rows are the compacted winners (often a small fraction of the 2B entries): small
    // tiles spread them over many compute units; very large batches use tall tiles so that the
    // gate weights are streamed from L2 fewer times.
    plan->gru_mt = 0;
    for (int mt = (2 * d.max_batch <= 16384 ? 1 : 4); mt >= 1; --mt)
        if (gru_lds_bytes(d, mt) <= lds_limit) {
            plan->gru_mt = mt;
            break;
        }
    plan->emb_mt = 0;
    for (int mt = 3; mt >= 1; --mt)
        if (embed_lds_bytes(d, mt) <= lds_limit) {
            plan->emb_mt = mt;
            break;
        }
    if (!plan->gru_mt || !plan->emb_mt)
        return false;
    plan->gru_entries = 16 * plan->gru_mt;
    plan->gru_lds = gru_lds_bytes(d, plan->gru_mt);
    plan->emb_lds = embed_lds_bytes(d, plan->emb_mt);
    return true;
}

hipError_t prepare_kernels(const Dims &d, const LaunchPlan &plan)
{
    hipError_t e = hipFuncSetAttribute(gru_kernel(d, plan.gru_mt),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, plan.gru_lds);
    if (e != hipSuccess)
        return e;
    return hipFuncSetAttribute(embed_kernel(d, plan.emb_mt), hipFuncAttributeMaxDynamicSharedMemorySize,
                               plan.emb_lds);
}

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

hipError_t launch_step(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw,
                       const StepArgs &a, hipStream_t s, hipEvent_t *marks)
{
    const int entries = 2 * a.count;
    const int Q = a.roles * a.count;
    hipError_t e;
    int mark = 0;
    auto stamp = [&]() -> hipError_t { return marks ? hipEventRecord(marks[mark++], s) : hipSuccess; };

    if ((e = stamp()) != hipSuccess)
        return e;
    const int n_scatter = (entries + kScatterEntries - 1) / kScatterEntries;
    hipLaunchKernelGGL(k_pre, dim3(n_scatter + (Q + 3) / 4), dim3(256), 0, s, a, d.K, n_scatter);
    if ((e = hipGetLastError()) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    hipLaunchKernelGGL(k_select, dim3((entries + 255) / 256), dim3(256), 0, s, a);
    if ((e = hipGetLastError()) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    {
        StepArgs aa = a;
        PackedWeights ww = pw;
        GruParams g = gru_params(d);
        void *args[] = {&aa, &ww, &g};
        const int grid = (entries + plan.gru_entries - 1) / plan.gru_entries;
        e = hipLaunchKernel(gru_kernel(d, plan.gru_mt), dim3(grid), dim3(kTileThreads), args,
                            (size_t)plan.gru_lds, s);
        if (e != hipSuccess || (e = stamp()) != hipSuccess)
            return e;
    }
    hipLaunchKernelGGL(k_commit, dim3((entries + 3) / 4), dim3(256), 0, s, a, d.M);
    if ((e = hipGetLastError()) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    {
        StepArgs aa = a;
        PackedWeights ww = pw;
        EmbedParams p = embed_params(d, plan.emb_mt, a.roles);
        void *args[] = {&aa, &ww, &p};
        const int grid = (a.count + p.TE - 1) / p.TE;
        e = hipLaunchKernel(embed_kernel(d, plan.emb_mt), dim3(grid), dim3(kTileThreads), args,
                            (size_t)plan.emb_lds, s);
        if (e != hipSuccess || (e = stamp()) != hipSuccess)
            return e;
    }
    return hipSuccess;
}

}  // namespace tig
