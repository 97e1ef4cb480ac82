/*
 * libtig -- the chronological mini-batch step of a memory-based temporal-interaction-graph
 * (TIG) model on one AMD MI355X (gfx950), as a C ABI.
 *
 * The step is the encoder/decoder data flow of the paper's Sec. II-C ("Training approach for
 * TIGs") on the shape one GPU's partition sees under the paper's partition-parallel training
 * (Sec. II-C "Distributed Parallel Training": one sub-graph, one N^(k) x d memory and one model
 * replica per GPU):
 *
 *   memory fetch -> message [s_self | s_other | Phi(dt) | e_ij] -> last message per node ->
 *   GRU state update -> memory overwrite -> attention embedding over the K most recent
 *   neighbours (history strictly before the event time, Sec. II-A) -> MLP link decoder.
 *
 * Conventions
 *   - every call returns TIG_OK (0) or a negative tig_status; nothing throws or aborts;
 *   - structs are plain data and start with `struct_size = sizeof(the struct)`;
 *   - the CALLER owns all device memory: the two workspaces handed to tig_init and every
 *     output buffer.  The library allocates no device memory;
 *   - pointers documented "host or device" are resolved through HIP's unified addressing;
 *     pointers documented "device" must be device memory readable by kernels;
 *   - a context is not thread-safe; distinct contexts are independent;
 *   - all validation that can be done on the host happens before anything is launched: a call
 *     that fails with an argument error (TIG_EINVAL, TIG_ERANGE, TIG_EORDER, TIG_ENOSPACE) leaves
 *     the model state (memory, last_update) unchanged.  TIG_EHIP from a step means a launch failed
 *     after earlier kernels of that step may have been enqueued: the state is then undefined until
 *     tig_reset or tig_state_import.
 */
#ifndef TIG_H
#define TIG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIG_API __attribute__((visibility("default")))

typedef enum tig_status {
    TIG_OK = 0,
    TIG_EINVAL = -1,    /* NULL pointer, bad struct_size, dimension out of the supported range */
    TIG_ERANGE = -2,    /* a node id or event id is out of range */
    TIG_EUNSORTED = -3, /* event times are not non-decreasing */
    TIG_ESELFLOOP = -4, /* an event has src == dst */
    TIG_ENOSPACE = -5,  /* a workspace is smaller than tig_workspace_bytes reports */
    TIG_EHIP = -6,      /* a HIP call failed; text via tig_last_error */
    TIG_ENOMEM = -7,    /* host allocation of the context failed */
    TIG_EORDER = -8     /* the batch starts before the end of the previous one (no reset / import between) */
} tig_status;

typedef enum tig_precision {
    TIG_FP32 = 0,      /* fp32 operands, fp32 accumulation on the matrix cores */
    TIG_BF16_MFMA = 1  /* bf16 matrix cores, fp32 accumulation.  Weights and matrix-core
                          activations are held as bf16 pairs x = hi + lo (hi = bf16(x) RNE,
                          lo = bf16(x - hi)) and a product is hi*hi + lo*hi + hi*lo: three bf16
                          MFMAs instead of eight fp32 ones per 32-deep block.  Biases, gates,
                          softmax, time encoding and the stored state stay fp32 */
} tig_precision;

/* Model / launch shape.  Notation: M memory width, T time-encoding width, F edge-feature
 * width, E embedding width, K neighbours, H heads, B events per batch.
 * D_msg = 2M+T+F, d_a = M+T (must be divisible by H), d_kv = M+F+T.
 * Limits: 1 <= M,T,F,E <= 512; 1 <= K <= 64; H in {1,2,4}; 1 <= max_batch <= 65536. */
/* Order of memory update and embedding inside a step (Sec. II-C describes the update-first data
 * flow; the deferred order is the one a training loop uses so that a prediction never sees its
 * own event through the memory). */
typedef enum tig_message_order {
    TIG_UPDATE_FIRST = 0, /* the step applies the messages of ITS batch, then embeds */
    TIG_DEFERRED = 1      /* the step applies the messages of the PREVIOUS step's batch (built from the
                             memory as it stands now), embeds, and keeps its own batch's last-message
                             winners for the next step; tig_reset / tig_state_import drop what is kept */
} tig_message_order;

typedef struct tig_config {
    uint32_t struct_size;
    int32_t mem_dim;       /* M */
    int32_t time_dim;      /* T */
    int32_t feat_dim;      /* F */
    int32_t emb_dim;       /* E */
    int32_t num_neighbors; /* K */
    int32_t num_heads;     /* H */
    int32_t max_batch;     /* largest `count` tig_step will be given */
    int32_t precision;     /* tig_precision, fixed for the life of the context */
    int32_t message_order; /* tig_message_order, fixed for the life of the context */
} tig_config;

/* The temporal interaction graph G = (V, E) of Sec. II-A: events (i, j, t) with a feature row
 * each, listed in chronological order; event id = position in the list.  All arrays: host or
 * device.  The library copies what it needs; the caller may free its copies after tig_init. */
typedef struct tig_graph {
    uint32_t struct_size;
    uint32_t reserved;
    int64_t num_nodes;      /* N: ids are 0..N-1 */
    int64_t num_events;     /* < 2^30 */
    const int32_t *src;     /* [num_events] */
    const int32_t *dst;     /* [num_events], dst != src */
    const double *ts;       /* [num_events], non-decreasing */
    const float *edge_feat; /* [num_events x F] row-major */
} tig_graph;

/* Model parameters, fp32, row-major [out x in]; host or device.
 *   time encoding      Phi(x)_k = cos(time_w[k] * x + time_b[k])              [T], [T]
 *   GRU (gates r,z,n)  W_i [3M x D_msg], b_i [3M], W_h [3M x M], b_h [3M]
 *   attention          W_Q [d_a x d_a], W_K, W_V [d_a x d_kv], W_O [d_a x d_a], biases [d_a]
 *   merge MLP          W_m1 [E x (d_a+M)], b_m1 [E], W_m2 [E x E], b_m2 [E]
 *   decoder MLP        W_d1 [E x 2E], b_d1 [E], w_d2 [E], b_d2 [1]
 * Message layout is [s_self (M) | s_other (M) | Phi (T) | e_ij (F)]; key/value rows are
 * [s_neighbour (M) | e (F) | Phi (T)]; the query row is [s_node (M) | Phi(0) (T)]. */
typedef struct tig_weights {
    uint32_t struct_size;
    uint32_t reserved;
    const float *time_w, *time_b;
    const float *W_i, *b_i, *W_h, *b_h;
    const float *W_Q, *b_Q, *W_K, *b_K, *W_V, *b_V, *W_O, *b_O;
    const float *W_m1, *b_m1, *W_m2, *b_m2;
    const float *W_d1, *b_d1, *w_d2, *b_d2;
} tig_weights;

/* One chronological mini-batch: the `count` events first_eid .. first_eid+count-1. */
typedef struct tig_batch {
    uint32_t struct_size;
    int32_t count;          /* 1 .. max_batch */
    int64_t first_eid;      /* first_eid + count <= num_events */
    const int32_t *neg_dst; /* device, [count]: one negative destination per event, or NULL
                               (then no negative rows and no score_neg are produced) */
} tig_batch;

/* Outputs, all device memory owned by the caller.  Q = 3*count with negatives, else 2*count;
 * query rows are ordered [sources | destinations | negatives].  NULL = not wanted. */
typedef struct tig_out {
    uint32_t struct_size;
    uint32_t reserved;
    float *emb;         /* [Q x E] embeddings emb_i(t)                      (required) */
    float *score_pos;   /* [count] logit g(emb_src, emb_dst)                (required) */
    float *score_neg;   /* [count] logit g(emb_src, emb_neg); required iff neg_dst != NULL */
    int32_t *nbr_node;  /* [Q x K] neighbour ids, slot 0 most recent, -1 = unused slot */
    int32_t *nbr_eid;   /* [Q x K] their event ids, -1 = unused */
    double *nbr_ts;     /* [Q x K] their event times, 0.0 = unused */
    int32_t *nbr_cnt;   /* [Q] number of used slots */
    uint8_t *is_winner; /* [2*count] entry 2*b+role (role 0 = source): 1 if that occurrence
                           supplied the node's (last) message of this batch */
} tig_out;

typedef struct tig_ctx tig_ctx;

/*
 * Sizes of the two device buffers the caller must allocate (256-byte aligned) for tig_init.
 * `persistent` holds the graph copy, the temporal adjacency, the model state and the prepared
 * weights for the life of the context; `scratch` holds per-step intermediates (and transient
 * data during tig_init).  Only num_nodes / num_events of `graph` are read (pointers may be NULL).
 */
TIG_API int tig_workspace_bytes(const tig_config *cfg, const tig_graph *graph,
                                size_t *persistent_bytes, size_t *scratch_bytes);

/*
 * Creates a context: copies graph and weights into `persistent`, validates the graph on the
 * device (ids in range -> TIG_ERANGE, times non-decreasing -> TIG_EUNSORTED, no self-loops ->
 * TIG_ESELFLOOP), builds the per-node time-ordered adjacency over ALL events (each event is
 * listed under both endpoints), prepares the weights for the matrix cores, and zeroes the
 * state (memory and last_update), which is the state after a reset (Alg. 2).
 * `hip_stream` is a hipStream_t (NULL = the default stream); every later call enqueues on it.
 * `weights` may be NULL: the context then has graph, adjacency and state but no model of its own,
 * and tig_step fails with TIG_EINVAL until tig_modules_attach has given it one.
 * Synchronous: returns after the device has finished.  On failure *out is NULL.
 */
TIG_API int tig_init(const tig_config *cfg, const tig_graph *graph, const tig_weights *weights,
                     void *persistent, size_t persistent_bytes, void *scratch, size_t scratch_bytes,
                     void *hip_stream, tig_ctx **out);

/*
 * One batch step (Sec. II-C), enqueued on the context's stream; does NOT synchronise.
 *   1. messages are built from the memory as it stands when the step starts;
 *   2. per node, the occurrence with the greatest (time, event id) supplies the message;
 *   3. GRU update; memory rows and last_update of exactly those nodes are overwritten;
 *   4. for every query (node, t_event): the K most recent incident events with time < t_event,
 *      taken from the whole graph given at tig_init, ordered by (time, event id) descending;
 *   5. attention over them with the UPDATED memory, merge MLP -> emb; decoder -> scores.
 * Steps run chronologically: a batch must not start before the end of the previous one unless
 * tig_reset or tig_state_import was called in between (they rewind the cursor to event 0).
 * Errors (nothing is launched, the state is unchanged): TIG_EINVAL for NULL required pointers or
 * count out of 1..max_batch, TIG_ERANGE if the event range leaves the graph, TIG_EORDER for a batch
 * that starts before the cursor.  neg_dst values must be valid node ids (they
 * are not checked on the device; an id outside 0..N-1 is treated as a node without history and
 * with zero memory).
 * The embedding of a query depends on (node, t_event) only, and the sources and destinations of a
 * batch repeat the same pairs many times (hub nodes, events sharing a timestamp): every distinct
 * pair is embedded once and its row is handed to every query that asked for it, so equal queries
 * get bit-identical embeddings.  Negatives are not merged.
 * Chronological passes hand over consecutive batches of one size, so every step also prepares,
 * inside its embedding launch, the batch that would follow it (first_eid + count, same count,
 * clipped at the end of the stream): its step-2 winners and the neighbour lists of its distinct
 * source / destination queries.  That preparation reads the event stream and the adjacency only,
 * never the model state; the next call uses it if its batch is exactly that one, and otherwise
 * prepares its batch itself in one more launch.  The step's last launch (scores, embedding rows)
 * also computes, into staging rows, the GRU output of the batch the next call would apply, from
 * the memory as this step leaves it; the next call takes those rows if its batch is that one and
 * the state has not been replaced since, else it runs the GRU itself.  A step of a chronological
 * pass is therefore two launches.  Results do not depend on whether the guess was right, and
 * tig_reset / tig_state_import in between are fine.
 */
TIG_API int tig_step(tig_ctx *ctx, const tig_batch *batch, const tig_out *out);

/*
 * The same step, same launches, with a HIP event recorded on the context's stream before the first
 * and after every kernel; waits for the step to finish and writes the kernel durations in
 * milliseconds to kernel_ms[0..TIG_NUM_STEP_KERNELS-1] (host), in launch order:
 *   0, 1  key scatter and winner selection of a batch above 4096 events (else 0)
 *   2     preparation of a batch that the previous step did not prepare (else 0)
 *   3     message + GRU and what is left of the query preparation, for a step whose applied batch
 *         the previous step's last launch did not cover (else 0)
 *   4     attention embedding (with the negatives' neighbour lookups), merge MLP, first decoder
 *         layer, memory overwrite (and the next batch's preparation)
 *   5     scores, per-query embedding rows (and message + GRU of the batch the next step applies)
 * For measurement: the event records add gaps between kernels, so time throughput with tig_step.
 */
#define TIG_NUM_STEP_KERNELS 6
TIG_API int tig_step_profiled(tig_ctx *ctx, const tig_batch *batch, const tig_out *out,
                              float *kernel_ms);

/*
 * tig_step for callers that must not allocate device memory or touch an allocator while stepping
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) and want the
 * step's intermediates out of their own workspace: the same step, same kernels, but every per-step
 * intermediate (query rows, staged rows, winner lists, counters) lives in an array that the
 * library holds statically on each GPU (TIG_STATIC_SCRATCH_BYTES per GPU, from library load to
 * process end; its device address is resolved once per device in tig_init).  Inputs, outputs and
 * the model state stay where tig_init put them.  The call allocates nothing and calls no
 * allocating routine.
 *   - only contexts with message_order = TIG_UPDATE_FIRST (else TIG_EINVAL);
 *   - TIG_ENOSPACE if the intermediates of the context's configuration (about
 *     max_batch * (120 * num_neighbors + 8 * mem_dim + 36 * emb_dim + 250) bytes) exceed
 *     TIG_STATIC_SCRATCH_BYTES;
 *   - the call prepares its batch itself (winners, queries) and keeps nothing in the array for a
 *     later call, so calls may be mixed freely with tig_step on any context;
 *   - every call on one GPU uses the same array: calls whose kernels may overlap on one GPU (two
 *     contexts on different streams) race and must be serialised by the caller.
 * Otherwise as tig_step (arguments, outputs, errors, chronological order).
 */
#define TIG_STATIC_SCRATCH_BYTES (32u << 20)
TIG_API int tig_step_static(tig_ctx *ctx, const tig_batch *batch, const tig_out *out);

/* ------------------------------------------------------------------------------------------
 * Training step (Sec. II-C: the decoder's edge probabilities provide the self-supervised signal;
 * Alg. 2: "Training and compute loss", "Backward and Optimize").  fp32 contexts only.
 *   loss  = mean_b softplus(-score_pos[b]) + mean_b softplus(score_neg[b])   (binary cross-entropy
 *           on the logits; the paper names neither loss nor optimiser: this build's reading)
 *   the node memory is a constant of the step: gradients reach the GRU (and, through its message,
 *   the time encoding) only through the memory rows that the step itself overwrites and its
 *   embeddings then read; edge features take no gradient
 *   update: W <- W - lr * dL/dW on fp32 master copies of the weights (plain SGD); the prepared
 *   weights that tig_step reads are rebuilt from the masters afterwards
 * ------------------------------------------------------------------------------------------ */

/* Size of the training workspace of a configuration (device memory the caller allocates):
 * master weights, gradients and the buffers of the backward pass, about
 * 12 * max_batch * ((2 * num_neighbors + 4 * num_heads) * (mem + feat + time) + 14 * (mem + time)) bytes
 * (the raw key / value rows of the neighbour slots and their gradients, and per-query rows).
 * TIG_EINVAL for a precision other than TIG_FP32 or a row shape the backward kernels cannot hold
 * (more than 4 heads, heads * neighbours above 64, key / value rows above 512 columns). */
TIG_API int tig_train_workspace_bytes(const tig_config *cfg, size_t *bytes);

/* Makes a context trainable: `weights` (host or device, as in tig_init; normally the same values)
 * become the master weights in `workspace` (device, 256-byte aligned, owned by the caller until
 * tig_destroy), and the context's prepared weights are rebuilt from them.  Synchronous.
 * The first call on a context also creates one HIP stream (default priority, non-blocking) and a few
 * events, which tig_destroy releases: no device memory, but host-side runtime objects. */
TIG_API int tig_train_attach(tig_ctx *ctx, const tig_weights *weights, void *workspace, size_t workspace_bytes);

/* One training step on a batch: the step of tig_step (same outputs, same state update, in the
 * context's message order), the loss, the gradient of every weight, and the SGD update with
 * learning rate lr >= 0 (0: gradients only, weights untouched).  batch->neg_dst is required.
 * loss_out: device pointer to one float, or NULL.  Enqueued on the context's stream; the weight-gradient
 * contractions run on the stream that tig_train_attach created, ordered against the context's stream
 * by events on both ends (they start when their inputs are complete and the context's stream waits for
 * them ahead of the update), so whatever the caller orders against the context's stream -- later
 * calls, copies, events -- sees the finished step.  On that stream the call also prepares the queries
 * of the batch it expects next (the same number of events, continuing where this one ends), as tig_step
 * does; a following tig_step or tig_train_step on another batch prepares its own. */
TIG_API int tig_train_step(tig_ctx *ctx, const tig_batch *batch, const tig_out *out, float lr, float *loss_out);

/* Copies the master weights (what = 0) or the gradients of the last training step (what = 1) to
 * the non-NULL pointers of `dst` (host or device), laid out as in tig_weights.  Synchronous. */
TIG_API int tig_train_get(tig_ctx *ctx, int32_t what, const tig_weights *dst);

/* ------------------------------------------------------------------------------------------
 * Other instances of the general architecture (Sec. II-C "Training approach for TIGs": the messages
 * of a node within a batch may be aggregated by their mean, the state update may be a GRU or a plain
 * RNN, the embedding function f may be identity, time projection or attention; Sec. II-A: nodes may
 * carry static features).  A module selection is attached to a context; tig_step, tig_reset,
 * tig_state_export / _import and the epoch machinery then run that instance, in the context's
 * message order, with the same arguments, outputs and errors.  fp32 contexts only.
 *   aggregator  LAST: the node's message of greatest (time, event id).  MEAN: the element-wise mean of
 *               all the node's messages of the batch, either role, each built from the memory at the
 *               start of the step with its own event's time, partner and feature row; last_update
 *               becomes the time of the node's last event of the batch either way
 *   updater     GRU as in tig_step.  RNN: s = tanh(W_i m + b_i + W_h s' + b_h), with
 *               W_i [M x D_msg], b_i [M], W_h [M x M], b_h [M] in tig_weights
 *   embedding   ATTENTION as in tig_step.  IDENTITY: emb_i(t) = r_i(t).  TIME_PROJECTION:
 *               emb_i(t) = (1 + (t - last_update_i) * time_proj_w) * r_i(t), element-wise, with the
 *               last_update the step's memory overwrite left.  Both need emb_dim == mem_dim, read no
 *               neighbours (the nbr_* outputs are not written) and ignore the attention and merge
 *               weights (may be NULL); the decoder is W_d1 [M x 2M], b_d1 [M], w_d2 [M], b_d2 [1]
 *   node_feat   [N x M] static node features (host or device) or NULL: wherever the embedding
 *               reads a node's state, its own or a neighbour's, it reads r_i(t) = s_i(t) + v_i;
 *               messages carry the raw memory rows
 * (The paper names these options and gives no formulas: the formulas are this build's reading.)
 * ------------------------------------------------------------------------------------------ */
typedef enum tig_aggregator { TIG_AGG_LAST = 0, TIG_AGG_MEAN = 1 } tig_aggregator;
typedef enum tig_updater { TIG_UPD_GRU = 0, TIG_UPD_RNN = 1 } tig_updater;
typedef enum tig_embedding { TIG_EMB_ATTENTION = 0, TIG_EMB_IDENTITY = 1, TIG_EMB_TIME_PROJECTION = 2 } tig_embedding;

/* Weights of a second attention layer (fp32, row-major [out x in], host or device).  Its input rows
 * are first-layer embeddings, so it has the width E where the first layer has the state width M:
 * d_a2 = E + T, d_kv2 = E + F + T (d_a2 divisible by num_heads);
 *   W_Q, W_O [d_a2 x d_a2], W_K, W_V [d_a2 x d_kv2], biases [d_a2],
 *   W_m1 [E x (d_a2 + E)], b_m1 [E], W_m2 [E x E], b_m2 [E]. */
typedef struct tig_layer_weights {
    uint32_t struct_size;
    uint32_t reserved;
    const float *W_Q, *b_Q, *W_K, *b_K, *W_V, *b_V, *W_O, *b_O;
    const float *W_m1, *b_m1, *W_m2, *b_m2;
} tig_layer_weights;

typedef struct tig_modules {
    uint32_t struct_size;
    int32_t aggregator;       /* tig_aggregator */
    int32_t updater;          /* tig_updater */
    int32_t embedding;        /* tig_embedding */
    const float *node_feat;   /* [N x M], host or device, or NULL */
    const float *time_proj_w; /* [M], host or device; required for TIG_EMB_TIME_PROJECTION */
    /* Attention embedding over the 2-hop temporal neighbourhood (the embedding module of Sec. II-C
     * sums over neighbor_i^k([0, t])): num_layers = 2 stacks a second layer on the first,
     *   h1_i(t)  = merge_1(attention_1([r_i(t) | Phi(0)], {[r_j(t) | e_ij | Phi(t - t_ij)]}), r_i(t))
     *   emb_i(t) = merge_2(attention_2([h1_i(t) | Phi(0)], {[h1_j(t) | e_ij | Phi(t - t_ij)]}), h1_i(t))
     * over the K most recent neighbours j of i before t; a neighbour's first-layer row is taken at the
     * QUERY's time t, over that neighbour's own K most recent events before t.  The first layer uses
     * the attention / merge weights of tig_weights, the second `layer2`.  0 or 1: one layer. */
    int32_t num_layers;
    int32_t reserved;
    const tig_layer_weights *layer2; /* required iff num_layers == 2 (TIG_EMB_ATTENTION only) */
} tig_modules;

/* Size of the workspace of a module selection (device memory the caller allocates): transposed
 * copies of the weights and, if node features are given, a copy of them.  TIG_EINVAL for a
 * precision other than TIG_FP32, an unknown selector, emb_dim != mem_dim with an embedding that
 * needs it, two layers without the attention embedding or without `layer2`, or rows the kernels
 * cannot hold (attention: more than 4 heads, heads * K above 64, key / value rows above 512 columns;
 * two layers: K above 63).  The attention embedding with node features or two layers runs as
 * contractions over all items of a layer (distinct queries; first of two layers: also their used
 * neighbour slots) and keeps the items' matrices here: about items * 4 * (5 * (w + T) + 4 * H *
 * (w + F + T) + E) bytes with w = max(mem_dim, emb_dim) and items = 3 * max_batch * (K + 1) for two
 * layers (1 GB at 2.6 M nodes' shape with batch 4000, K = 10), 3 * max_batch for one.  Two layers also
 * add the second hop's neighbour tables and the first layer's rows:
 * 3 * max_batch * (K * K * 16 + (K + 1) * 4 * E) bytes. */
TIG_API int tig_modules_workspace_bytes(const tig_config *cfg, const tig_modules *modules, int64_t num_nodes,
                                        size_t *bytes);

/* Makes the context compute the selected instance with `weights` (host or device; shapes as above).
 * `workspace`: device, 256-byte aligned, owned by the caller until tig_destroy.  Anything prepared
 * ahead by earlier steps, and the winners a deferred step kept for the next one, are dropped; the
 * state (memory, last_update, cursor) is kept.  Afterwards
 * tig_step_static and the tig_train_* calls refuse the context (TIG_EINVAL), and a context with a
 * training workspace cannot take a module selection.  Synchronous. */
TIG_API int tig_modules_attach(tig_ctx *ctx, const tig_modules *modules, const tig_weights *weights,
                               void *workspace, size_t workspace_bytes);

/* Memory reset at the start of a data cycle (Alg. 2): memory <- 0, last_update <- 0. Async. */
TIG_API int tig_reset(tig_ctx *ctx);

/*
 * Backup / restore of the node memory (end-of-cycle backup and end-of-epoch restore, Sec. II-C
 * and Alg. 2).  mem: [N x M] fp32 row-major, last_update: [N] fp64; host or device.
 * Synchronous (they wait for the stream, copy, and return).
 */
TIG_API int tig_state_export(tig_ctx *ctx, float *mem_out, double *last_update_out);
TIG_API int tig_state_import(tig_ctx *ctx, const float *mem_in, const double *last_update_in);

/* Frees the host-side context.  Device buffers belong to the caller and are not touched. */
TIG_API void tig_destroy(tig_ctx *ctx);

/* Static text for a status code / detail of the last failure on this context ("" if none);
 * tig_last_error(NULL) gives the detail of the last failed tig_init on the calling thread. */
TIG_API const char *tig_strerror(int status);
TIG_API const char *tig_last_error(const tig_ctx *ctx);

/* For reports: the number of kernels the last step enqueued (2 when the previous step had
 * prepared this batch, 4 otherwise, 6 for batches above 4096 events; 0 before the first step) and
 * the dynamic LDS bytes of the two tile kernels at their largest tile count.
 * Any pointer may be NULL. */
TIG_API int tig_launch_info(const tig_ctx *ctx, int32_t *kernels_per_step, int32_t *gru_lds_bytes,
                            int32_t *embed_lds_bytes);

/* ------------------------------------------------------------------------------------------
 * Streaming edge partitioner (Sec. II-B "Streaming Edge Partitioning Component", Alg. 1): the
 * preprocessing step that cuts the event stream into the per-GPU sub-graphs.  Independent of any
 * tig_ctx.
 * ------------------------------------------------------------------------------------------ */
typedef struct tig_sep_config {
    uint32_t struct_size;
    int32_t num_parts;   /* |P|, 1..64 */
    double beta;         /* time-decay rate of Eq. 1, >= 0 */
    double top_k;        /* fraction k of the nodes that may be replicated (the hubs), 0..1 */
    double lambda;       /* weight of the balance term, Eq. 6, > 0 */
    double epsilon;      /* added to the denominator of Eq. 6, > 0 */
} tig_sep_config;

/*
 * Node centrality with exponential time decay (Eq. 1): cent_out[i] = sum over the events incident
 * to node i of exp(beta * (t - t_max)), t_max = ts[num_events - 1] (the stream is chronological).
 * src, dst [E] int32, ts [E] fp64, cent_out [N] fp64: device pointers.  Enqueued on hip_stream
 * (one small synchronous read of t_max aside).  The per-node sums are accumulated with fp64
 * atomics, so their last bits depend on the order the device happened to add in.
 * Events with an endpoint outside 0..N-1 are skipped.
 */
TIG_API int tig_sep_centrality(const int32_t *src, const int32_t *dst, const double *ts, int64_t num_events,
                               int64_t num_nodes, double beta, double *cent_out, void *hip_stream);

/*
 * The hubs of Alg. 1 (first step): the n_hubs nodes of greatest centrality, equal centralities in
 * order of node id.  cent [N] fp64, hubs_out [n_hubs] int32 (by rank), is_hub_out [N] bytes (1 for a
 * hub), scratch (256-byte aligned, tig_sep_topk_scratch_bytes(N) bytes): device pointers.
 * TIG_ENOSPACE if scratch is too small.  Enqueued on hip_stream.
 */
TIG_API size_t tig_sep_topk_scratch_bytes(int64_t num_nodes);
TIG_API int tig_sep_top_k(const double *cent, int64_t num_nodes, int64_t n_hubs, int32_t *hubs_out,
                          uint8_t *is_hub_out, void *scratch, size_t scratch_bytes, void *hip_stream);

/*
 * The edge loop of Alg. 1 (cases 1-5 with the score C = C_REP + C_BAL of Eq. 2-6).  Every
 * decision depends on all earlier ones: sequential, on the host; ALL pointers are host pointers.
 *   edge_part_out [E]   partition the edge went to, -1 for a discarded edge (Case 3)
 *   node_parts_out [N]  bit p set: the node has a replica in partition p (the set A(i) of Alg. 1).
 *                       A node with more than one bit is a shared node; the node loop of Alg. 1
 *                       then lists it in every partition (the caller's part, from this mask).
 *   part_edges_out [|P|] edges per partition (the |p| of Eq. 6)
 * Readings: |p| counts edges; a resident non-hub is never replicated, so its partition is the
 * only candidate whenever it is an endpoint; the arg max takes the lowest index among equal
 * scores.  TIG_ERANGE if an endpoint is outside 0..N-1 (outputs are then partial).
 */
TIG_API int tig_sep_assign(const tig_sep_config *cfg, const int32_t *src, const int32_t *dst, int64_t num_events,
                           int64_t num_nodes, const double *cent, const uint8_t *is_hub, int32_t *edge_part_out,
                           uint64_t *node_parts_out, int64_t *part_edges_out);

/*
 * All of Alg. 1 up to the node masks: centrality and hubs (floor(top_k * N) of them) on the
 * device, then the edge loop on the host.  src, dst, ts: device pointers; scratch: device,
 * 256-byte aligned, tig_sep_scratch_bytes(N) bytes; every output is a HOST pointer (cent_out [N],
 * is_hub_out [N], the rest as in tig_sep_assign).  Synchronous; allocates host staging for the
 * endpoint arrays (TIG_ENOMEM if that fails).
 */
TIG_API size_t tig_sep_scratch_bytes(int64_t num_nodes);
TIG_API int tig_sep_partition(const tig_sep_config *cfg, const int32_t *src, const int32_t *dst, const double *ts,
                              int64_t num_events, int64_t num_nodes, void *scratch, size_t scratch_bytes,
                              void *hip_stream, double *cent_out, uint8_t *is_hub_out, int32_t *edge_part_out,
                              uint64_t *node_parts_out, int64_t *part_edges_out);

/* ------------------------------------------------------------------------------------------
 * Epoch machinery of parallel training on partitions, as one GPU sees it when it holds several
 * partitions at once (Sec. II-C "Distributed Parallel Training", Alg. 2).
 * ------------------------------------------------------------------------------------------ */

/*
 * Shuffle-and-combine: the |P| small parts, in the caller's shuffled `order` (a permutation of
 * 0..num_parts-1), are joined num_parts / num_groups at a time into num_groups groups;
 * group_masks_out[g] has the bits of group g's parts.  Host pointers.  TIG_EINVAL if num_groups does
 * not divide num_parts or `order` is not a permutation.
 */
TIG_API int tig_pac_combine(const int32_t *order, int32_t num_parts, int32_t num_groups, uint64_t *group_masks_out);

/*
 * Sub-graph of the (combined) partition `group`: E_k = {(i, j, t) in E | i, j in V_k}, where V_k
 * holds the nodes with a replica in one of the group's parts and every shared node (a node with
 * more than one bit in node_parts, tig_sep_assign's output).
 *   src, dst [E], node_parts [N]: device;  eid_out [E] (capacity): the event ids of E_k in
 *   chronological order;  local_out [N]: rank of the node among the members of V_k in id order, -1
 *   for a non-member;  counts_out (HOST) [2]: |E_k|, |V_k|;  scratch: device, 256-byte aligned,
 *   tig_pac_scratch_bytes(E, N) bytes (TIG_ENOSPACE if smaller).  Synchronous.
 */
TIG_API size_t tig_pac_scratch_bytes(int64_t num_events, int64_t num_nodes);
TIG_API int tig_pac_subgraph(const int32_t *src, const int32_t *dst, int64_t num_events, const uint64_t *node_parts,
                             int64_t num_nodes, uint64_t group, int32_t *eid_out, int32_t *local_out,
                             int64_t *counts_out, void *scratch, size_t scratch_bytes, void *hip_stream);

/*
 * The sub-graph's event arrays from the whole graph's (all device pointers): for n event ids,
 * endpoints relabelled through `local`, times, and feature rows [n x feat_dim].  Enqueued.
 */
TIG_API int tig_pac_gather(const int32_t *src, const int32_t *dst, const double *ts, const float *edge_feat,
                           int32_t feat_dim, const int32_t *eid, int64_t n, const int32_t *local, int32_t *src_out,
                           int32_t *dst_out, double *ts_out, float *feat_out, void *hip_stream);

/* One resident partition of an epoch: a context over its sub-graph and what its steps need. */
typedef struct tig_pac_part {
    uint32_t struct_size;
    int32_t batch;              /* events per step, 1..max_batch of the context */
    tig_ctx *ctx;
    int64_t num_events;         /* events of the sub-graph that take part (a prefix of the context's) */
    const int32_t *neg_dst;     /* device [num_events]: one negative per event, or NULL */
    float *backup_mem;          /* device [N_k x M]: the partition's memory backup */
    double *backup_lu;          /* device [N_k] */
    const tig_out *out;         /* outputs of the partition's steps (overwritten by every step) */
} tig_pac_part;

/*
 * One epoch of Alg. 2 over the resident partitions, in lock step: every partition cycles over its
 * own batches (memory reset at the start of a data cycle, backup at the end of one) until the
 * partition with the most batches has finished a cycle (*steps_out, may be NULL, = that number of
 * steps); then every partition's memory is restored from its latest backup.  Uses tig_reset,
 * tig_step, tig_state_export and tig_state_import of the contexts; synchronous.
 */
TIG_API int tig_pac_epoch(tig_pac_part *parts, int32_t n_parts, int64_t *steps_out);

/*
 * Memory synchronisation of the shared nodes across resident partitions (end of Sec. II-C):
 * local_ids (HOST array of n_parts DEVICE pointers) gives, for shared node s, its row
 * local_ids[k][s] in partition k.  mode 0: every replica takes the row and the last-update time of
 * the partition with the largest last-update time (the lowest partition among equal times);
 * mode 1: the mean of the rows (summed in partition order, fp32) and the largest time.  The
 * contexts must share memory width and stream and be distinct; ids of one partition must be
 * distinct; at most 32 partitions.  A node with an id outside a partition is left alone.  Enqueued.
 */
TIG_API int tig_pac_sync_shared(tig_ctx *const *ctxs, int32_t n_parts, const int32_t *const *local_ids,
                                int64_t n_shared, int32_t mode);

#ifdef __cplusplus
}
#endif
#endif /* TIG_H */
