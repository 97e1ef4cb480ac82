// Device-side building blocks shared by the step kernels (gfx950, wave64).
//
// Tile GEMM convention (16x16 output tiles on the matrix cores):
//   operand A: activations in LDS, row-major; lane l supplies row l%16 and KB/4 consecutive k's
//              starting at k0 + (KB/4)*(l/16);
//   operand B: prepared weights, already lane-ordered in global memory (pack.hip);
//   result   : lane l holds rows 4*(l/16)+v (v = 0..3) of column l%16.
#pragma once

#include <hip/hip_runtime.h>

#include "tig_internal.h"

namespace tig {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

#ifdef TIG_PHASE_CLOCKS
// Debug build only: per-block timestamps (100 MHz real-time counter) at phase boundaries.  The
// translation unit that uses TIG_MARK defines g_phase_clocks.
#define TIG_MARK(slot)                                                    \
    do {                                                                  \
        if (threadIdx.x == 0 && blockIdx.x < 8192)                        \
            g_phase_clocks[blockIdx.x * 8 + (slot)] = wall_clock64();     \
    } while (0)
#else
#define TIG_MARK(slot) \
    do {               \
    } while (0)
#endif

constexpr int kWave = 64;

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
    static __device__ inline float load_elem(const char *row, int k) { return ((const float *)row)[k]; }
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
    static __device__ inline void store_a(char *row, int k, float v)
    {
        __bf16 *p = (__bf16 *)row + ((k >> 3) << 4) + (k & 7);
        const __bf16 hi = (__bf16)v;  // round to nearest even
        p[0] = hi;
        p[8] = (__bf16)(v - (float)hi);
    }
    static __device__ inline float load_elem(const char *row, int k)  // hi + lo: v to ~2^-17 relative
    {
        const __bf16 *p = (const __bf16 *)row + ((k >> 3) << 4) + (k & 7);
        return (float)p[0] + (float)p[8];
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

template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ inline float dpp_or_zero(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, BANK_MASK, true));
}

// The two cross-row steps of wave_sum_uniform for several values at once, as fused DPP adds: rows
// outside the row mask keep their value, which the compiler does not express in one instruction.
// The leading s_nop covers the two wait states a DPP read needs after a vector-ALU write of the
// same register, and the trailing one keeps whatever the compiler places next (it does not see
// inside the block) clear of the last results; inside the block two instructions on one register
// are far enough apart.
__device__ inline void add_row_bcasts(float &a, float &b)
{
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "v_add_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "s_nop 0\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "v_add_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "s_nop 1"
                 : "+v"(a), "+v"(b));
}

__device__ inline void add_row_bcasts(float &a, float &b, float &c, float &d)
{
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "v_add_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "v_add_f32_dpp %2, %2, %2 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "v_add_f32_dpp %3, %3, %3 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "v_add_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "v_add_f32_dpp %2, %2, %2 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "v_add_f32_dpp %3, %3, %3 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "s_nop 1"
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// One cross-row step on a single register: rows 1 and 3 combine with lane 15 of rows 0 and 2,
// rows 0 and 2 keep their value.  (s_nop: see add_row_bcasts.)
__device__ inline void add_row_bcast15(float &a)
{
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "s_nop 1"
                 : "+v"(a));
}
__device__ inline void max_row_bcast15(float &a)
{
    asm volatile("s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "s_nop 1"
                 : "+v"(a));
}

// lane i of each 16-lane row takes lane i + n of v's row; the last n lanes of the row keep `old`
template <int N>
__device__ inline float row_shl_keep_n(float old, float v)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), 0x100 + N, 0xf, 0xf, false));
}
__device__ inline float row_shl_keep(float old, float v, int n)
{
    switch (n) {
    case 0: return v;
    case 1: return row_shl_keep_n<1>(old, v);
    case 2: return row_shl_keep_n<2>(old, v);
    case 3: return row_shl_keep_n<3>(old, v);
    case 4: return row_shl_keep_n<4>(old, v);
    case 5: return row_shl_keep_n<5>(old, v);
    case 6: return row_shl_keep_n<6>(old, v);
    case 7: return row_shl_keep_n<7>(old, v);
    case 8: return row_shl_keep_n<8>(old, v);
    case 9: return row_shl_keep_n<9>(old, v);
    case 10: return row_shl_keep_n<10>(old, v);
    case 11: return row_shl_keep_n<11>(old, v);
    case 12: return row_shl_keep_n<12>(old, v);
    case 13: return row_shl_keep_n<13>(old, v);
    case 14: return row_shl_keep_n<14>(old, v);
    default: return row_shl_keep_n<15>(old, v);
    }
}

// every lane of a 16-lane row takes the maximum / the sum over the row (rotations: no lane is empty)
__device__ inline float row_max_all(float v)
{
    // written out: the compiler would canonicalise both operands of every maximum
    asm volatile("s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_ror:1 row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_ror:2 row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1"
                 : "+v"(v));
    return v;
}
__device__ inline float row_sum_all(float v)
{
    v += dpp_or_zero<0x121, 0xf, 0xf>(v);
    v += dpp_or_zero<0x122, 0xf, 0xf>(v);
    v += dpp_or_zero<0x124, 0xf, 0xf>(v);
    return v + dpp_or_zero<0x128, 0xf, 0xf>(v);
}

// Wavefront sums of four values at once: returns a register whose lanes 15, 31, 47 and 63 hold
// the sums over all 64 lanes of a, b, c and d.  v_permlane32_swap exchanges the upper half of its
// first operand with the lower half of its second, v_permlane16_swap the odd 16-lane rows of the
// first with the even rows of the second; an add after each folds two registers into one.
__device__ inline float wave_sum_four(float a, float b, float c, float d)
{
    const auto ac = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(c), false, false);
    const auto bd = __builtin_amdgcn_permlane32_swap(__float_as_uint(b), __float_as_uint(d), false, false);
    const float x = __uint_as_float(ac[0]) + __uint_as_float(ac[1]);  // [a | c], 32 partial sums each
    const float y = __uint_as_float(bd[0]) + __uint_as_float(bd[1]);  // [b | d]
    const auto xy = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    float z = __uint_as_float(xy[0]) + __uint_as_float(xy[1]);        // rows [a, b, c, d], 16 partial sums each
    z += dpp_or_zero<0x111, 0xf, 0xf>(z);
    z += dpp_or_zero<0x112, 0xf, 0xf>(z);
    z += dpp_or_zero<0x114, 0xf, 0xf>(z);
    z += dpp_or_zero<0x118, 0xf, 0xf>(z);
    return z;
}

// Raw buffer descriptor word 3 for gfx950: 32-bit data format, no swizzle.  With stride 0 a lane
// whose byte offset is not inside [0, extent - 4] reads 0.
constexpr int kBufferFlags = 0x00020000;

__device__ inline float buffer_load_f32(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_offset)
{
    return __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)byte_offset, 0, 0));
}

// value of lane `src` (wave-uniform) as a scalar
__device__ inline double readlane_f64(double v, int src)
{
    const long long b = __double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(b & 0xffffffffll), src);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(b >> 32), src);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
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

// Phi(x)_k = cos(w_k x + b_k) (the time encoding of Sec. II-C).  The phase is formed in
// revolutions in fp64 -- w_rev = w / 2pi, b_rev = b / 2pi prepared at init; the argument reaches
// ~1e6 rad, far beyond fp32 -- reduced to [0, 1) in fp64, and the hardware cosine (input in
// revolutions, measured max abs error 1.3e-7 on [0, 1)) is applied to the fp32 fraction.
// Total abs error < 6e-7.
__device__ inline float time_enc(double w_rev, double b_rev, double x)
{
    const double phase = fma(w_rev, x, b_rev);
    return __builtin_amdgcn_cosf((float)__builtin_amdgcn_fract(phase));
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

// acc[mt] += A[16*mt .. 16*mt+15][k-blocks kb0 .. kb0+kblocks) x W[nt]^T.
// A: LDS rows of `lda` BYTES (4 bytes per element in either precision); A's k-block kb0+i pairs
// with W's k-block w_kb0+i.  W: lane-ordered blocks, `w_kblocks` per output tile.
// Weight operands come from L2 and the loop is latency-bound, so up to DEPTH operand loads are
// issued before the first MFMA of a group.
template <int PREC, int MT, int DEPTH>
__device__ inline void tile_gemm(floatx4 (&acc)[MT], const char *A, int lda, int a_kb0, const void *W,
                                 int w_kblocks, int w_kb0, int kblocks, int nt)
{
    using P = Prec<PREC>;
    using frag = typename P::frag;
    const int lane = lane_id();
    const size_t w0 = ((size_t)nt * w_kblocks + w_kb0) * kWave + lane;
    const char *ap = A + (size_t)(lane & 15) * lda;
    const int g = lane >> 4;
    int kb = 0;
    for (; kb + DEPTH <= kblocks; kb += DEPTH) {
        frag bfrag[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            bfrag[u] = P::load_w(W, w0 + (size_t)(kb + u) * kWave);
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, a_kb0 + kb + u, g);
                P::mma(acc[mt], afrag, bfrag[u]);
            }
        }
    }
    if (kb < kblocks) {  // remainder: same depth, predicated
        frag bfrag[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks)
                bfrag[u] = P::load_w(W, w0 + (size_t)(kb + u) * kWave);
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            if (kb + u < kblocks) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, a_kb0 + kb + u, g);
                    P::mma(acc[mt], afrag, bfrag[u]);
                }
            }
        }
    }
}

// The same for two output tiles nt1, nt2 of one weight matrix: every operand of A is read from
// LDS once and meets the weights of both tiles (the A reads, not the matrix cores, bound these
// small products).
template <int PREC, int MT, int DEPTH>
__device__ inline void tile_gemm_two(floatx4 (&acc1)[MT], floatx4 (&acc2)[MT], const char *A, int lda, int a_kb0,
                                     const void *W, int w_kblocks, int kblocks, int nt1, int nt2)
{
    using P = Prec<PREC>;
    using frag = typename P::frag;
    const int lane = lane_id();
    const size_t w1 = (size_t)nt1 * w_kblocks * kWave + lane;
    const size_t w2 = (size_t)nt2 * w_kblocks * kWave + lane;
    const char *ap = A + (size_t)(lane & 15) * lda;
    const int g = lane >> 4;
    for (int kb = 0; kb < kblocks; kb += DEPTH) {
        frag b1[DEPTH], b2[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks) {
                b1[u] = P::load_w(W, w1 + (size_t)(kb + u) * kWave);
                b2[u] = P::load_w(W, w2 + (size_t)(kb + u) * kWave);
            }
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, a_kb0 + kb + u, g);
                    P::mma(acc1[mt], afrag, b1[u]);
                    P::mma(acc2[mt], afrag, b2[u]);
                }
            }
    }
}

// The same for one output tile of each of two weight matrices with equal k depth (both over all
// k-blocks of A from 0).
template <int PREC, int MT, int DEPTH>
__device__ inline void tile_gemm_pair(floatx4 (&acc1)[MT], floatx4 (&acc2)[MT], const char *A, int lda,
                                      const void *W1, const void *W2, int kblocks, int nt1, int nt2)
{
    using P = Prec<PREC>;
    using frag = typename P::frag;
    const int lane = lane_id();
    const size_t w1 = (size_t)nt1 * kblocks * kWave + lane;
    const size_t w2 = (size_t)nt2 * kblocks * kWave + lane;
    const char *ap = A + (size_t)(lane & 15) * lda;
    const int g = lane >> 4;
    for (int kb = 0; kb < kblocks; kb += DEPTH) {
        frag b1[DEPTH], b2[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks) {
                b1[u] = P::load_w(W1, w1 + (size_t)(kb + u) * kWave);
                b2[u] = P::load_w(W2, w2 + (size_t)(kb + u) * kWave);
            }
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (kb + u < kblocks) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const frag afrag = P::load_a(ap + (size_t)mt * 16 * lda, kb + u, g);
                    P::mma(acc1[mt], afrag, b1[u]);
                    P::mma(acc2[mt], afrag, b2[u]);
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

}  // namespace tig
