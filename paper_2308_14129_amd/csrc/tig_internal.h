// Internal declarations shared by the translation units of libtig (host side + kernel launchers).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/tig.h"

namespace tig {

// One adjacency entry of the per-node, time-ordered event lists: 16 bytes, so the K most
// recent entries of a node are one contiguous 16*K-byte read.
struct __attribute__((aligned(16))) CsrEntry {
    int32_t nbr;  // the other endpoint
    int32_t eid;  // event id
    double ts;    // event time
};

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Derived dimensions.  KB = depth of one matrix-core k-block (16 for fp32: four 16x16x4 MFMAs
// fed by one 16-byte operand load per lane; 32 for bf16: 16x16x32 MFMAs on hi/lo split operands).
struct Dims {
    int M, T, F, E, K, H;
    int Dmsg, da, dh, dkv;
    int prec;     // tig_precision
    int KB;       // 16 | 32
    int esz;      // bytes per stored matrix-core operand element: 4 (fp32, or a bf16 hi/lo pair)
    // GRU tile GEMM: A row = [s_self | s_other | Phi | e] padded to Kg; per gate Ng output cols
    int Kg, Khn, Ng;
    // embedding tile GEMMs
    int dkvp;     // d_kv padded to KB
    int Mq;       // M padded to KB
    int N1;       // H * dkvp      (folded query rows)
    int K2;       // H * dkvp + Mq (merge layer-1 input)
    int Ep;       // E padded to 16 (output cols)
    int Ek;       // E padded to KB (k depth of the E-wide layers)
    int max_batch;
    int deferred;  // message order: 0 update first, 1 deferred
};

// Prepared (folded, padded, lane-ordered) weights in `persistent`.
struct PackedWeights {
    const double *time_w_rev, *time_b_rev;     // [T] time-encoding frequency / phase in revolutions (w/2pi, b/2pi)
    const void *gru_Wr, *gru_Wz, *gru_Win;     // [Ng x Kg] packed
    const void *gru_Whn;                       // [Ng x Khn] packed
    const float *gru_br, *gru_bz, *gru_bin, *gru_bhn;  // [Ng]
    const void *emb_A1;                        // [N1 x Mq] packed: folded W_K^T W_Q / sqrt(d_h)
    const float *emb_a1;                       // [N1]
    const void *emb_PR;                        // [Ep x K2] packed: folded W_m1 W_O W_V | W_m1 (memory part)
    const float *emb_c, *emb_c0;               // [Ep] layer-1 bias with / without neighbours
    const void *emb_Wm2;                       // [Ep x Ek] packed
    const float *emb_bm2;                      // [Ep]
    const void *dec_W;                         // [2Ep x Ek] packed: W_d1[:, :E] ; W_d1[:, E:]
    const float *dec_b1, *dec_w2;              // [Ep]
    const void *dec_WF;                        // [2Ep x Ek] packed: the same times W_m2 (acts on h1)
    const float *dec_b1f;                      // [Ep] b_d1 + (W_d1[:, :E] + W_d1[:, E:]) b_m2
    const float *dec_b2;                       // [1]
};

// One winner of the last-message aggregation: everything the GRU and the memory overwrite need.
struct __attribute__((aligned(8))) WinDesc {
    int32_t entry;  // 2*b + role within the batch
    int32_t node;   // the node whose memory is updated
    int32_t other;  // the partner of the event
    int32_t b;      // event position in the batch
    double t;       // event time
};

struct StepArgs {
    // graph (device)
    const int32_t *src, *dst;
    const double *ts;
    const float *edge_feat;
    const int64_t *indptr;
    const CsrEntry *csr;
    const int32_t *pos;  // [2E] adjacency position of entry 2*eid + role (in its node's list)
    int64_t num_nodes;
    // state (device)
    float *mem;
    double *lu;
    unsigned long long *key;
    // batch
    int64_t first_eid;
    int32_t count;
    int32_t roles;  // 2 | 3
    const int32_t *neg;
    // the batch whose winners (`win`) feed the GRU and the memory overwrite: this batch, or the
    // previous step's in the deferred order (msg_count 0: nothing to apply)
    int64_t msg_first_eid;
    int32_t msg_count;
    // intermediates (device)
    int32_t *nbr_node, *nbr_eid, *nbr_cnt;
    double *nbr_ts;
    float *staging;  // [2*count x M] new memory rows of the winners, by entry 2b+role
    WinDesc *win;       // [2*count] entries that supply their node's message (compacted)
    int32_t *n_win;     // [1] their number
    uint8_t *is_winner;  // may be NULL
    // the batch expected to follow (next_count 0: none): its winners are selected by one extra
    // workgroup of this step's embedding launch
    int64_t next_first_eid;
    int32_t next_count;
    WinDesc *next_win;
    int32_t *next_n_win;
    uint8_t *next_is_winner;  // may be NULL
    // outputs
    float *emb, *score_pos, *score_neg;
};

struct LaunchPlan {
    int gru_entries;     // entries (event, role) per GRU workgroup: 16*gru_mt
    int gru_mt;          // 16-row tiles per GRU workgroup
    int gru_lds;         // bytes
    int emb_mt;          // most 16-row tiles per embedding workgroup (what LDS holds)
    int num_cus;         // compute units of the device (0 until known)
    int emb_lds;         // bytes
};

// ---- launchers (each returns the hipError_t of the launch) -------------------------------
hipError_t launch_validate_graph(const int32_t *src, const int32_t *dst, const double *ts,
                                 int64_t num_events, int64_t num_nodes, int32_t *flags,
                                 hipStream_t s);
size_t csr_build_scratch_bytes(int64_t num_events, int64_t num_nodes);
hipError_t csr_build(const int32_t *src, const int32_t *dst, const double *ts, int64_t num_events,
                     int64_t num_nodes, int64_t *indptr, CsrEntry *csr, int32_t *pos, void *scratch,
                     size_t scratch_bytes, hipStream_t s);

size_t pack_scratch_bytes(const Dims &d);
size_t packed_weights_bytes(const Dims &d);
// Folds / pads / reorders the weights into `dst` (device, packed_weights_bytes) and fills `pw`.
hipError_t pack_weights(const Dims &d, const tig_weights &w_dev_f32, void *dst, void *scratch,
                        PackedWeights *pw, hipStream_t s);

bool plan_launch(const Dims &d, int lds_limit, LaunchPlan *plan);
int gru_lds_bytes(const Dims &d, int mt);
int embed_lds_bytes(const Dims &d, int mt);
hipError_t prepare_gru(const Dims &d, const LaunchPlan &plan);
hipError_t prepare_embed(const Dims &d, const LaunchPlan &plan);
hipError_t prepare_small();
// winners of the batch in one launch when it is small enough; otherwise scatter + *needs_select
hipError_t launch_scatter(const StepArgs &a, hipStream_t s, bool *needs_select);
hipError_t launch_select(const StepArgs &a, hipStream_t s);
// GRU tiles and, in the same launch, the neighbour lookup of every query
hipError_t launch_gru(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                      hipStream_t s);
hipError_t launch_commit(const StepArgs &a, int M, hipStream_t s);
hipError_t launch_embed(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                        hipStream_t s);
// whether the embedding launch of a batch of `count` events can carry one more workgroup that
// selects the winners of a following batch of `next_count` events without delaying anything
bool embed_can_select_ahead(const Dims &d, const LaunchPlan &plan, int roles, int count, int next_count);
hipError_t prepare_kernels(const Dims &d, const LaunchPlan &plan);
constexpr int kNumStepKernels = 5;
// `marks`: NULL, or kNumStepKernels + 1 events recorded before the first and after every kernel.
// `sel`: NULL, or the arguments of a last-message selection to run first (its first_eid / count /
// win / n_win / is_winner name the batch and where the winners go).
hipError_t launch_step(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw,
                       const StepArgs &a, const StepArgs *sel, hipStream_t s, hipEvent_t *marks);
hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t s);

}  // namespace tig
