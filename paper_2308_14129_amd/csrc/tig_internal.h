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

// A row reference names where the CURRENT state row of a node lives while a step runs: the
// memory table (the node was not updated by this step), or the staged GRU output of the entry
// that supplied the node's message (the memory overwrite happens after the embedding).
//   ref >= 0: memory row `ref`;  ref < 0 (not kRefNone): staging row ~ref;  kRefNone: a zero row.
constexpr int32_t kRefNone = INT32_MIN;

// The distinct embedding queries (node, t) of one batch.  Source and destination queries of a
// batch repeat heavily (hub nodes, events sharing a timestamp); each distinct pair gets ONE row
// here, `slot` maps every (event, role) entry to its row.  Rows [0, *n_u) belong to source /
// destination queries (*n_u <= 2 * count), row 2 * count + b to the negative of event b
// (negatives are not merged; their place does not depend on the device-side count).
struct QuerySet {
    int32_t *node;      // [R] node id, -1: none
    double *t;          // [R] query time
    int32_t *cnt;       // [R] filled neighbour slots
    int32_t *self_ref;  // [R] row reference of the node's own state
    int32_t *nbr;       // [R x K] neighbour node ids, -1 = unused slot
    int32_t *ref;       // [R x K] their row references
    int32_t *eid;       // [R x K] their event ids, -1 = unused
    double *ts;         // [R x K] their event times, 0.0 = unused
    int32_t *slot;      // [2B] entry 2b+role -> row (>= 0), or -(entry of its representative) - 1
    int32_t *n_u;       // [1]
};

// Last-message selection of one batch (count 0: nothing to do).  Besides the compacted winner
// list it leaves key[node] = the winning entry's 64-bit (time, event id, role) key.  There are two
// winner lists (the one a step applies and the one selected meanwhile), each with a key array of
// its own; a key array is only ever written by selections of chronologically later batches, or
// cleared (tig_reset / tig_state_import), so a stale key is never greater than a batch's own.
struct SelectJob {
    int64_t first_eid;
    int32_t count;
    WinDesc *win;       // out: winners
    int32_t *n_win;     // out: their number
    uint8_t *flags;     // out: [2 * count] 1 where the entry supplied its node's message
    unsigned long long *key;  // in/out: [N] the key array that goes with this winner list
};

// Merging of equal (node, t) queries of one batch's sources and destinations + the neighbour
// lookup of every distinct one (count 0: nothing to do).
struct DedupJob {
    int64_t first_eid;
    int32_t count;
    QuerySet qs;                // out (n_u must be 0 when the job starts)
    unsigned long long *tab;    // hash table of claims, (epoch << 32 | entry); other epochs = empty
    uint32_t tab_mask;          // slots - 1 (power of two, >= 4 * count)
    uint32_t epoch;             // != 0, different from every earlier job on this table
    int32_t n_wgs;              // workgroups that share the job
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
    // batch
    int64_t first_eid;
    int32_t count;
    int32_t roles;  // 2 | 3
    const int32_t *neg;
    // the batch whose winners (`win`) feed the GRU and the memory overwrite: this batch, or the
    // previous step's in the deferred order (msg_count 0: nothing to apply)
    int64_t msg_first_eid;
    int32_t msg_count;
    WinDesc *win;
    int32_t *n_win;
    const unsigned long long *msg_key;  // [N] key array of that selection (see SelectJob)
    const uint8_t *win_flags;  // flags of THIS batch's selection (copied out when asked for), may be NULL
    // intermediates (device)
    QuerySet qs;     // distinct queries of this batch
    float *staging;  // [2*msg_count x M] new memory rows of the winners, by entry 2b+role
    float *gru_gates;  // NULL, or [2*msg_count x 4 x M]: r, z, n and the hidden half of n's pre-activation of winner r of the list (a training step's backward pass reads them)
    float *emb_u;    // [R x E] embedding of every distinct query
    float *dec_a;    // [R x Ep] first decoder layer, source half, of every distinct query
    float *dec_b;    // [R x Ep] the same, second-operand half
    // finishing pass of the preparation (prepare.h): in the GRU launch for this batch if its slots /
    // row references are not final yet, and in the closing launch for the batch prepared ahead (whose
    // applied batch is (fin_first_eid, fin_count) with key array fin_key)
    int32_t finish_here;        // 1: the GRU launch also fixes this batch's slots and row references
    int32_t fin_count;          // 0: the decode launch finishes nothing
    int64_t fin_msg_first_eid;
    int32_t fin_msg_count;
    const unsigned long long *fin_msg_key;
    int32_t *n_u_clear; // counter of a query set that no kernel reads any more (cleared by the closing launch), may be NULL
    int32_t *rows_seen; // host memory mapped into the device: the step leaves its numbers of distinct rows [0] and of winners [1] here, may be NULL
    int32_t rows_est;   // host side only: expected number of distinct rows (sizes the embedding tiles)
    int32_t wins_est;   // host side only: expected number of winners (sizes the GRU column slices)
    // work done on compute units the embedding launch leaves idle: selection of a batch's winners
    // and preparation of a batch's queries
    SelectJob sel;
    DedupJob ded;
    // outputs
    float *emb, *score_pos, *score_neg;
    int32_t *out_nbr_node, *out_nbr_eid, *out_nbr_cnt;  // optional
    double *out_nbr_ts;                                 // optional
    uint8_t *out_is_winner;                             // optional
};

struct LaunchPlan {
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
// parts: kPackGru = the state update's matrices (W_i / W_h are read), kPackEmbed = attention, merge
// MLP and decoder; the time-encoding parameters go with either.  A part that is left out keeps what
// `dst` holds (zeros after tig_init's clear for a context whose state update runs elsewhere).
enum PackParts { kPackGru = 1, kPackEmbed = 2, kPackAll = 3 };
hipError_t pack_weights(const Dims &d, const tig_weights &w_dev_f32, void *dst, void *scratch,
                        PackedWeights *pw, hipStream_t s, int parts = kPackAll);

bool plan_launch(const Dims &d, int lds_limit, LaunchPlan *plan);
int gru_lds_bytes(const Dims &d);
int embed_lds_bytes(const Dims &d, int mt);
hipError_t prepare_gru(const Dims &d, const LaunchPlan &plan);
hipError_t prepare_embed(const Dims &d, const LaunchPlan &plan);
hipError_t prepare_small();
bool winners_in_one_launch(int count);
// batches above the one-workgroup limit: keys to the per-node array, then winners + flags
hipError_t launch_scatter(const StepArgs &a, const SelectJob &j, hipStream_t s);
hipError_t launch_select(const StepArgs &a, const SelectJob &j, hipStream_t s);
// selection (one workgroup, if sel.count > 0) and query preparation (if ded.count > 0) as a launch
hipError_t launch_prepare(const StepArgs &a, const SelectJob &sel, const DedupJob &ded, int K, hipStream_t s);
// The batch whose winners the NEXT step applies, for the GRU workgroups of a step's closing launch
// (count 0: none; that step runs the GRU itself).
struct GruAhead {
    int64_t first_eid;
    int32_t count;
    const WinDesc *win;
    const int32_t *n_win;
};
// GRU of the batch a step applies and, in the same launch, what is left of its query preparation
// (slots, row references), ahead of the embedding launch
// (gru_work = false: only the finishing pass -- the staged rows come from elsewhere)
hipError_t launch_gru(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                      hipStream_t s, bool gru_work = true);
// embedding of the distinct queries (the negatives' neighbours are looked up here); memory overwrite;
// selection and query preparation for the batch expected next
hipError_t launch_embed(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                        hipStream_t s);
// scores and per-query embeddings from the distinct rows, optional inspection outputs, finishing pass
// of the batch prepared ahead, GRU of the batch the next step applies
hipError_t launch_closing(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                          const GruAhead &ahead, hipStream_t s, bool events = true);
// workgroups the embedding launch can spare for a following batch's preparation (0: none)
int embed_spare_workgroups(const Dims &d, const LaunchPlan &plan, int roles, int count);
// workgroups of a batch's query preparation; `shared`: in a launch whose workgroups each occupy a
// compute unit (beside the embedding tiles or the one-workgroup selection)
int prepare_workgroups(int count, bool shared);
hipError_t prepare_kernels(const Dims &d, const LaunchPlan &plan);
constexpr int kNumStepKernels = TIG_NUM_STEP_KERNELS;
// What one step launches, in order: [scatter, select] (up-front selection of a batch above the
// one-workgroup limit), [prepare] (selection and / or query preparation not done ahead),
// [gru] (unless the previous step's closing launch ran it), embed, closing.
// `marks`: NULL, or kNumStepKernels + 1 events.
struct StepPlan {
    const SelectJob *big_sel;   // scatter + select launches, or NULL
    const SelectJob *prep_sel;  // selection inside the prepare launch, or NULL
    const DedupJob *prep_ded;   // query preparation inside the prepare launch, or NULL
    bool clear_tab;             // clear prep_ded's claim table first
    bool gru_now;               // the GRU launch ahead of the embedding
    // a training step: forward in direct form, loss, backward and SGD instead of the embedding launch
    bool train;
    void *train_ws;
    void *packed;
    PackedWeights *pw_out;
    float lr;
    float *loss_out;
    const struct TrainSide *train_side;  // NULL, or the side stream of the weight-gradient contractions
    // a training step with a side stream: preparation that nothing of this step reads (this batch's
    // selection in the deferred order, the next batch's queries), launched on that stream; or NULL
    const SelectJob *side_sel;
    const DedupJob *side_ded;
    int32_t *clear_first;       // a counter to clear ahead of everything, or NULL
    GruAhead ahead;             // GRU workgroups of the closing launch
    const struct ModParams *mods;  // a context with a module selection: its kernels instead of GRU, embedding and closing launches
};
// does the step copy neighbour lists or winner flags out
inline bool wants_inspection(const StepArgs &a)
{
    return a.out_nbr_node || a.out_nbr_eid || a.out_nbr_ts || a.out_nbr_cnt || a.out_is_winner;
}
hipError_t launch_step(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw,
                       const StepArgs &a, const StepPlan &sp, hipStream_t s, hipEvent_t *marks);
hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t s);

// Memory synchronisation of shared nodes across the partitions resident on one GPU.
constexpr int kMaxSyncParts = 32;
struct SyncArgs {
    float *mem[kMaxSyncParts];
    double *lu[kMaxSyncParts];
    const int32_t *ids[kMaxSyncParts];  // [n_shared] row of shared node s in partition k
    int64_t num_nodes[kMaxSyncParts];
    int32_t n_parts, M, mode;           // mode 0: the row with the largest last-update time, 1: the mean
    int64_t n_shared;
};
hipError_t launch_sync_shared(const SyncArgs &a, hipStream_t s);
// ---- training step (train.hip) ----
size_t train_workspace_bytes(const Dims &d);
bool train_supported(const Dims &d);
hipError_t prepare_train(const Dims &d);
hipError_t train_attach(const Dims &d, const tig_weights &w, void *workspace, void *packed, PackedWeights *pw,
                        hipStream_t s);
hipError_t train_copy_out(const Dims &d, void *workspace, bool grads, const tig_weights &out, hipStream_t s);
// A second stream for the weight-gradient contractions of a training step: they depend on nothing
// but their own (delta, input) rows, so they run beside the rest of the backward pass; `fork[i]` is
// recorded on the step's stream when the rows of group i are complete, `join` on the side stream
// after the last contraction (the step's stream waits for it ahead of the update).
constexpr int kTrainForks = 7;  // (the last one: the preparation launched beside the step)
struct TrainSide {
    hipStream_t stream;
    hipEvent_t fork[kTrainForks], join;
};
// side: NULL = everything on s
hipError_t launch_train(const Dims &d, const StepArgs &a, void *workspace, void *packed, PackedWeights *pw, float lr,
                        float *loss_out, hipStream_t s, const TrainSide *side);
// after training steps with lr != 0 only the state update's prepared weights follow the masters: this
// re-folds the rest (attention, merge MLP, decoder) for the fused inference kernels
hipError_t train_refold_embed(const Dims &d, void *workspace, void *packed, PackedWeights *pw, hipStream_t s);
// where the step's GRU launch leaves the gates of the applied winners for the backward pass
float *train_gates_buffer(const Dims &d, void *workspace);
// ---- other instances of the general architecture (modules.hip) ----
// Module selection of a context and its weights: transposed copies ([in x out]) in the attached workspace.
constexpr int kAccCopies = 8;  // accumulation rows per node of the mean aggregator (entries are dealt out to them: less same-address traffic)
struct AttnLayer {
    const float *T_Q, *T_K, *T_V, *T_O, *b_Q, *b_K, *b_V, *b_O;  // attention
    const float *T_m1, *T_m2, *b_m1, *b_m2;    // merge MLP
    const float *N_Q, *N_V, *N_O, *N_m1, *N_m2;  // the matrices as given ([out x in]) for the contractions over all rows
};
struct ModParams {
    int agg, upd, emb;                         // tig_aggregator, tig_updater, tig_embedding
    int layers;                                // attention embedding: 1 or 2 stacked layers
    const double *time_w_rev, *time_b_rev;     // [T] time-encoding frequency / phase in revolutions
    const float *T_i, *T_h, *b_i, *b_h;        // state update: [D_msg x GM], [M x GM], [GM], [GM] (G = 3 GRU, 1 RNN)
    AttnLayer L[2];                            // first layer (input width M) and second (input width E)
    QuerySet hop2;                             // two layers: neighbour tables of (neighbour k of query row q, t_q) at row q * K + k
    float *h1;                                 // two layers: first-layer rows [3 * max_batch x (K + 1) x E], one per item in the items' order
    // the attention embedding as contractions over all items of a layer (an item: a distinct query, or --
    // first of two layers -- neighbour j of a distinct query at the query's time); widths are the larger of
    // the two layers'
    float *mr_qin, *mr_qv, *mr_qt, *mr_kvb, *mr_o, *mr_x1, *mr_h1;
    int32_t *mr_has;                           // [items] 1 for an item with at least one filled neighbour slot
    int32_t *mr_itq, *mr_itj;                  // [items] the item's query row and slot (K: the query itself)
    int32_t *mr_ci;                            // [3 * max_batch x (K + 1)] first layer: item of (query row x, slot j), or -(1 + the (x, j) index that represents its (node, t) pair)
    int32_t *mr_n;                             // [1] items of the first layer (cleared every step)
    uint32_t *mr_tab;                          // first layer: claims of equal (node, t) pairs, 1 + the claimant's (x, j) index, 0 = empty (cleared every step)
    uint32_t mr_tab_mask;                      // its size - 1 (a power of two)
    const float *T_d1, *b_d1, *w_d2, *b_d2;    // decoder: [2E x E], [E], [E], [1]
    const float *node_feat;                    // [N x M] or NULL
    const float *time_proj_w;                  // [M] or NULL
    bool fused_embed;                          // attention without node features: the fused embedding / closing launches run it
    double *acc;                               // mean aggregator: [2 * max_batch x kAccCopies x (M + T + F)] message sums by winning entry, zero between steps
    int32_t *acc_cnt;                          // ... and the number of messages in each
};
size_t modules_workspace_bytes(const Dims &d, const tig_modules &m, int64_t num_nodes);
bool modules_supported(const Dims &d, const tig_modules &m);
hipError_t modules_attach(const Dims &d, const tig_modules &m, const tig_weights &w, int64_t num_nodes, void *workspace,
                          ModParams *out, hipStream_t s);
// state update, memory overwrite, embedding, decoder and inspection outputs of a step of a context
// with a module selection; marks: NULL, or two events (after the overwrite, after the rest)
hipError_t launch_modules(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw, const StepArgs &a,
                          const ModParams &p, hipStream_t s, hipEvent_t *marks);
// records a failed HIP call of a context-free entry point (read back with tig_last_error(NULL)); returns TIG_EHIP
int fail_global(const char *what, hipError_t e);

}  // namespace tig
