// A layer product over all rows of a step at once on the matrix cores (fp32 16x16x4), shared by the
// training step and the attention embedding of the module instances.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels_common.h"

namespace tig {

namespace {

struct RowCount {  // rows = min(rows_max, (*dev + add) * mul), or rows_max if dev is NULL
    const int32_t *dev;
    int add, mul, rows_max;
};
__device__ inline int row_count(const RowCount &rc)
{
    if (!rc.dev)
        return rc.rows_max;
    const long long r = ((long long)*rc.dev + rc.add) * rc.mul;
    return r < 0 ? 0 : (r < rc.rows_max ? (int)r : rc.rows_max);
}

// A layer product over all rows at once: C[r][n] = f(sum_k A[r][k] W[n][k] (+ sum_k A2[r][k] W2[n][k]) + bias[n])
// on the matrix cores (fp32 16x16x4).  A and W are both k-contiguous: a forward product takes the
// weight matrix as stored ([out x in]), a backward product dX = dY W its transposed copy
// ([in x out]).  A workgroup takes 32 rows; each of its four wavefronts one block of 32 columns
// (blockIdx.y counts groups of four column blocks; the workgroups stride over the row blocks).  A lane
// loads four consecutive k of its row per step (k = k0 + 4 g + v for lane group g: the four groups
// cover 16 k, and the v-th products of a step pair the same k in both operands).
struct RowGemm {
    const float *A, *W, *A2, *W2, *bias;
    float *C;
    int lda, ldw, lda2, ldw2, ldc;
    int N, Kd, Kd2;
    RowCount rc;
    int relu;                // f = max(., 0)
    const float *gate;       // NULL, or: the result is kept where gate[row][n] > 0, else 0
    int ldg;
    const int32_t *rowmask;  // NULL, or: rows with rowmask[row] == 0 give 0 (no bias)
    const int32_t *remap_nu; // NULL, or: output row of r is r below min(*remap_nu, remap_2b), else remap_2b + (r - that)
    int remap_2b;
    int vecA, vecW, vecA2, vecW2;  // operand rows are 16-byte aligned: four k in one load
    // two products that share A in one launch: columns n >= n_split (n_split > 0) take the weight rows
    // W_hi[n - n_split] and bias_hi[n - n_split] and go to C_hi[row][n - n_split]; rowmask then covers
    // the columns below n_split only
    int n_split;
    const float *W_hi, *bias_hi;
    float *C_hi;
    int ldc_hi;
    int ldw_hi, Kd_hi;  // 0: as W; else the rows of W_hi are Kd_hi <= Kd long (A's columns beyond count as 0 for them)
    // a batch of products in one launch (one per attention head): product z = blockIdx.z reads A + z * zA,
    // W + z * zW, bias + z * zBias and writes C + z * zC (element offsets)
    int zA, zW, zC, zBias;
};

// Four consecutive k of one operand row.  VEC (rows 16-byte aligned, Kd a multiple of 4): one load,
// no branch -- a k outside the operand reads a valid address and is zeroed afterwards (finite values
// are assumed there: the row's first elements).
template <bool VEC>
__device__ inline floatx4 load_k4(const float *row, int k, int Kd, bool ok, int vec)
{
    floatx4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (VEC) {
        // (a load behind a condition is waited for at the end of its branch, and the compiler makes a
        // branch of a choice between a loaded value and zero: the load is unconditional from a valid
        // address and a k beyond the row is multiplied away; rows and columns outside the product
        // read row 0 and are never stored)
        const floatx4 r = *(const floatx4 *)(row + (k < Kd ? k : 0));
        const float m = k < Kd ? 1.0f : 0.0f;
        return floatx4{r[0] * m, r[1] * m, r[2] * m, r[3] * m};
    }
    if (!ok)
        return v;
    if (vec && k + 3 < Kd)
        return *(const floatx4 *)(row + k);
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (k + u < Kd)
            v[u] = row[k + u];
    return v;
}

// acc += the part over k in [k_lo, k_hi) (k_lo a multiple of 16) of one block of 32 rows x 32 columns
// of product z of p, by one wavefront: rows r0 .., columns 32 tn ..
template <bool VEC>
__device__ inline void rowgemm_accumulate(const RowGemm &p, int rows, int r0, int tn, int z, int pass, int k_lo, int k_hi,
                                          floatx4 (&acc)[2][2])
{
    const int lane = threadIdx.x & (kWave - 1);
    const int c = lane & 15, g = lane >> 4;
    const int n0 = tn * 32;
    const int split = p.n_split > 0 ? p.n_split : p.N;
    // the two rows whose operand this lane loads (rows r0 + c and r0 + 16 + c)
    size_t arow[2];
    bool aok[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = r0 + 16 * i + c;
        const bool ok = r < rows;
        arow[i] = (size_t)(ok ? r : 0);
        aok[i] = ok;
    }
    const float *A = pass ? p.A2 : p.A + (size_t)z * p.zA, *W = pass ? p.W2 : p.W + (size_t)z * p.zW;
    const int lda = pass ? p.lda2 : p.lda, ldw = pass ? p.ldw2 : p.ldw, Kd = pass ? p.Kd2 : p.Kd;
    const int vA = pass ? p.vecA2 : p.vecA, vW = pass ? p.vecW2 : p.vecW;
    const float *ar[2] = {A + arow[0] * lda, A + arow[1] * lda};
    const int nn0 = n0 + c, nn1 = n0 + 16 + c;
    const bool wok[2] = {nn0 < p.N, nn1 < p.N};
    const float *wr[2];
    int wkd[2];  // length of the lane's weight rows
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int nn = wok[i] ? (i ? nn1 : nn0) : 0;
        const bool hi = nn >= split;  // (no second pass with a split)
        wr[i] = hi ? p.W_hi + (size_t)(nn - split) * (p.ldw_hi ? p.ldw_hi : ldw) : W + (size_t)nn * ldw;
        wkd[i] = hi && p.Kd_hi ? p.Kd_hi : Kd;
    }
    const int k_end = k_hi < Kd ? k_hi : Kd;
    constexpr int kU = 4;  // steps of 16 k whose loads are issued together
    for (int k0 = k_lo; k0 < k_end; k0 += 16 * kU) {
        floatx4 av[kU][2], wv[kU][2];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kk = k0 + 16 * u + 4 * g;
            const bool on = k0 + 16 * u < k_end;  // (uniform)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                av[u][i] = load_k4<VEC>(ar[i], kk, Kd, aok[i] && on, vA);
                wv[u][i] = load_k4<VEC>(wr[i], kk, wkd[i], wok[i] && on, vW);
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (k0 + 16 * u >= k_end)
                break;  // (uniform: nothing but zeros was loaded for this step)
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][i][v], wv[u][j][v], acc[i][j], 0, 0, 0);
        }
    }
}

// Epilogue of one 16 x 16 sub-block (i, j) of a block: the lane holds rows 16 i + 4 g + v (v = 0..3) of
// column 16 j + c.  What the epilogue reads (bias, gate, row mask) is loaded unconditionally -- from a
// valid address where the product has no such input, the value then plays no part -- and ahead of
// the first store, so that a sub-block costs one round trip (a load inside a branch is waited for at
// the end of the branch: one round trip per load).
struct RowGemmEpi {
    float bias, gate[4];
    int32_t mask[4];
};

// the output-row remapping's row count (0 without one), requested early
__device__ inline int rowgemm_remap_count(const RowGemm &p)
{
    const int32_t *src = p.remap_nu ? p.remap_nu : (const int32_t *)p.W;
    const int nu = *src;
    return p.remap_nu ? (nu < 0 ? 0 : (nu < p.remap_2b ? nu : p.remap_2b)) : 0;
}

__device__ inline int rowgemm_out_row(const RowGemm &p, int r, int nu)
{
    return p.remap_nu ? (r < nu ? r : p.remap_2b + (r - nu)) : r;
}

__device__ inline RowGemmEpi rowgemm_epi_load(const RowGemm &p, int rows, int r0, int tn, int z, int i, int j, int nu)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int c = lane & 15, g = lane >> 4;
    const int split = p.n_split > 0 ? p.n_split : p.N;
    const int n = tn * 32 + 16 * j + c;
    const int nc = n < p.N ? n : 0;
    const bool hi = nc >= split;
    const float *bptr = hi ? p.bias_hi : (p.bias ? p.bias + (size_t)z * p.zBias : nullptr);
    RowGemmEpi e;
    e.bias = (bptr ? bptr : p.W)[bptr ? (hi ? nc - split : nc) : 0] * (bptr ? 1.0f : 0.0f);
    const float *gp = p.gate ? p.gate : p.W;
    const int32_t *mp = p.rowmask ? p.rowmask : (const int32_t *)p.W;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int r = r0 + 16 * i + 4 * g + v;
        const int rc = r < rows ? r : 0;
        e.mask[v] = mp[p.rowmask ? rc : 0];
        e.gate[v] = gp[p.gate ? (size_t)rowgemm_out_row(p, rc, nu) * p.ldg + nc : 0];
    }
    return e;
}

__device__ inline void rowgemm_epi_store(const RowGemm &p, int rows, int r0, int tn, int z, const floatx4 &acc, int i, int j,
                                         int nu, const RowGemmEpi &e)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int c = lane & 15, g = lane >> 4;
    const int split = p.n_split > 0 ? p.n_split : p.N;
    const int n = tn * 32 + 16 * j + c;
    if (n >= p.N)
        return;
    const bool hi = n >= split;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int r = r0 + 16 * i + 4 * g + v;
        if (r >= rows)
            continue;
        const int orow = rowgemm_out_row(p, r, nu);
        float val = acc[v] + e.bias;
        if (p.relu)
            val = fmaxf(val, 0.0f);
        const bool gated_off = (p.gate != nullptr) & !(e.gate[v] > 0.0f);
        const bool dead = (p.rowmask != nullptr) & (e.mask[v] == 0) & !hi;
        val = (gated_off | dead) ? 0.0f : val;
        if (hi)
            p.C_hi[(size_t)orow * p.ldc_hi + (n - split)] = val;
        else
            p.C[(size_t)z * p.zC + (size_t)orow * p.ldc + n] = val;
    }
}

template <bool VEC>
__device__ inline void rowgemm_tile(const RowGemm &p, int rows, int r0, int tn, int z)
{
    floatx4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[i][j] = floatx4{0, 0, 0, 0};
    const int nu = rowgemm_remap_count(p);
    for (int pass = 0; pass < (p.A2 ? 2 : 1); ++pass)
        rowgemm_accumulate<VEC>(p, rows, r0, tn, z, pass, 0, pass ? p.Kd2 : p.Kd, acc);
    RowGemmEpi e[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            e[i][j] = rowgemm_epi_load(p, rows, r0, tn, z, i, j, nu);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            rowgemm_epi_store(p, rows, r0, tn, z, acc[i][j], i, j, nu, e[i][j]);
}

// The same product with the k range of a block split over the four wavefronts of a workgroup
// (partial blocks added up in LDS; wavefront w then finishes sub-block (w / 2, w % 2)): for products
// over few rows, where one wavefront per block leaves one wavefront per SIMD walking its whole k
// range as a chain of load -> multiply rounds with nothing to overlap them.
template <bool VEC>
__global__ void __launch_bounds__(256) k_rowgemm_ks(RowGemm p)
{
    __shared__ float red[4][16][kWave];
    const int rows = row_count(p.rc);
    const int lane = threadIdx.x & (kWave - 1), w = (int)threadIdx.x / kWave;
    const int tn = (int)blockIdx.y, z = (int)blockIdx.z;
    const int kq = ((p.Kd + 3) / 4 + 15) / 16 * 16;  // k per wavefront, a multiple of 16
    const int nu = rowgemm_remap_count(p);
    for (int r0 = (int)blockIdx.x * 32; r0 < rows; r0 += (int)gridDim.x * 32) {
        floatx4 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = floatx4{0, 0, 0, 0};
        // (what this wavefront's sub-block (w / 2, w % 2) needs for its epilogue is requested ahead of the products)
        const RowGemmEpi e = rowgemm_epi_load(p, rows, r0, tn, z, w >> 1, w & 1, nu);
        rowgemm_accumulate<VEC>(p, rows, r0, tn, z, 0, w * kq, (w + 1) * kq, acc);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    red[w][(i * 2 + j) * 4 + v][lane] = acc[i][j][v];
        __syncthreads();
        const int si = w >> 1, sj = w & 1;
        floatx4 sum;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            sum[v] = (red[0][w * 4 + v][lane] + red[1][w * 4 + v][lane]) + (red[2][w * 4 + v][lane] + red[3][w * 4 + v][lane]);
        rowgemm_epi_store(p, rows, r0, tn, z, sum, si, sj, nu, e);
        __syncthreads();  // (the partial blocks are reused by the next row block)
    }
}

template <bool VEC>
__global__ void __launch_bounds__(256) k_rowgemm(RowGemm p)
{
    const int rows = row_count(p.rc);
    const int tiles_n = (p.N + 31) / 32;
    const int tn = (int)blockIdx.y * 4 + (int)threadIdx.x / kWave;  // this wavefront's block of 32 columns
    if (tn >= tiles_n)
        return;
    for (int r0 = (int)blockIdx.x * 32; r0 < rows; r0 += (int)gridDim.x * 32)
        rowgemm_tile<VEC>(p, rows, r0, tn, (int)blockIdx.z);
}

inline bool rowgemm_all_vec(const RowGemm &g)
{
    return g.vecA && g.vecW && g.Kd % 4 == 0 && g.Kd_hi % 4 == 0 && g.ldw_hi % 4 == 0 &&
           (!g.A2 || (g.vecA2 && g.vecW2 && g.Kd2 % 4 == 0));
}

// (the row count is known on the device only: at most 1024 row blocks are launched and stride)
inline void launch_rowgemm(const RowGemm &g, int nz, hipStream_t s)
{
    const int row_blocks = (g.rc.rows_max + 31) / 32, tiles_n = (g.N + 31) / 32;
    const int gx = row_blocks < 1024 ? (row_blocks > 0 ? row_blocks : 1) : 1024;
    if (!g.A2 && g.Kd >= 64 && row_blocks <= 512) {  // few rows: four wavefronts per block, each a quarter of k
        const dim3 grid(gx, tiles_n, nz);
        if (rowgemm_all_vec(g))
            hipLaunchKernelGGL(k_rowgemm_ks<true>, grid, dim3(256), 0, s, g);
        else
            hipLaunchKernelGGL(k_rowgemm_ks<false>, grid, dim3(256), 0, s, g);
        return;
    }
    const dim3 grid(gx, (tiles_n + 3) / 4, nz);
    if (rowgemm_all_vec(g))
        hipLaunchKernelGGL(k_rowgemm<true>, grid, dim3(256), 0, s, g);
    else
        hipLaunchKernelGGL(k_rowgemm<false>, grid, dim3(256), 0, s, g);
}

// operand rows start on 16-byte boundaries: four k in one load
inline int rowgemm_vec_ok(const float *p, int ld) { return (((uintptr_t)p & 15) == 0 && ld % 4 == 0) ? 1 : 0; }

}  // namespace

}  // namespace tig
