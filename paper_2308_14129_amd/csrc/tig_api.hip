// C ABI of libtig (see include/tig.h): argument validation, workspace layout, context.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>

#include "tig_internal.h"

using namespace tig;

// Per-step intermediates of tig_step_static: one array per GPU, held until the process ends.
// The name below is a host-side stand-in, not a device address: host code resolves the array's
// address on each device once (static_scratch_of) and only ever uses that pointer.
static __device__ __align__(256) unsigned char g_static_scratch[TIG_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void *g_static_ptr[kMaxDevices];  // device address of the array on each GPU, NULL until resolved

// Address of the static scratch array on the CURRENT device `dev` (resolved on first use).
static hipError_t static_scratch_of(int dev, void **out)
{
    if (dev < 0 || dev >= kMaxDevices)
        return hipErrorInvalidDevice;
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
        if (e != hipSuccess)
            return e;
        g_static_ptr[dev] = p;
    }
    *out = g_static_ptr[dev];
    return hipSuccess;
}

// Per-step intermediates, carved from the scratch workspace (or from the static array).
struct StepScratch {
    QuerySet qs[2];        // distinct queries: the set a step uses, and the one prepared meanwhile
    float *staging, *emb_u, *dec_a, *dec_b;
    WinDesc *win[2];       // winner lists: the one a step applies, and the one selected meanwhile
    int32_t *n_win[2];
    uint8_t *flags[2];     // per-entry winner flags of each list's batch
    unsigned long long *tab;  // claim table of the query preparation
    uint32_t tab_slots;       // power of two
    size_t bytes;
};

struct tig_ctx {
    Dims d;
    LaunchPlan plan;
    PackedWeights pw;
    hipStream_t stream;
    int64_t num_nodes, num_events;
    // persistent
    int32_t *src, *dst;
    double *ts;
    float *edge_feat;
    int64_t *indptr;
    CsrEntry *csr;
    int32_t *pos;
    float *mem;
    double *lu;
    unsigned long long *key[2];  // one key array per winner list
    void *packed;
    StepScratch S;     // in the scratch workspace
    void *scratch;     // the scratch workspace itself
    int wcur;          // update-first: winner list the last step applied; deferred: list with the pending winners
    int qcur;          // query set the last step used
    bool ahead_w_valid;  // update-first: list wcur ^ 1 holds the winners of batch (ahead_w_first, ahead_w_count)
    int64_t ahead_w_first;
    int32_t ahead_w_count;
    // the staging rows hold the GRU output for the winners of batch (ahead_g_first, ahead_g_count),
    // computed by the last step's closing launch from the memory as that step left it
    bool ahead_g_valid;
    int64_t ahead_g_first;
    int32_t ahead_g_count;
    bool ahead_q_valid;  // set qcur ^ 1 holds the queries of batch (ahead_q_first, ahead_q_count)
    bool ahead_q_finished;  // ... with final slots and row references (else the step finishes them)
    int64_t ahead_q_first;
    int32_t ahead_q_count;
    // deferred order: list wcur holds the winners of batch (pend_first, pend_count), not yet applied
    bool pend_valid;
    int64_t pend_first;
    int32_t pend_count;
    uint32_t epoch;    // of the last query preparation on S.tab
    int num_cus;
    int64_t cursor;    // end of the last batch stepped since the last reset / import
    int last_launches; // kernels enqueued by the last tig_step
    void *static_scratch;  // this device's copy of g_static_scratch
    bool embed_stale;      // training steps have moved the master weights since the attention / merge / decoder weights were last folded
    void *train_ws;        // training workspace (master weights, gradients, the backward pass's buffers), or NULL
    TrainSide train_side;  // side stream and events of the training step's weight-gradient contractions
    bool have_train_side;
    bool has_model;        // tig_init was given weights (the headline instance's prepared weights exist)
    void *mods_ws;         // workspace of an attached module selection, or NULL
    ModParams mods;        // ... and its parameters
    // Two pinned host words that the device can write: every step leaves its numbers of distinct
    // query rows and of winners there, and later calls shape their launches by them (hints that
    // may be a few steps old; results do not depend on them).  NULL if the allocation failed.
    int32_t *rows_seen_host;
    int32_t *rows_seen_dev;
    hipEvent_t marks[kNumStepKernels + 1];
    unsigned last_ran;  // which intervals between the marks held a kernel in the last step
    bool have_marks;
    char err[256];
};

namespace {

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base((char *)p) {}
    template <typename T>
    T *take(size_t count)
    {
        T *p = base ? (T *)(base + off) : nullptr;
        off += align_up(sizeof(T) * (count ? count : 1));
        return p;
    }
};

int check_config(const tig_config *c)
{
    if (!c || c->struct_size != sizeof(tig_config))
        return TIG_EINVAL;
    auto in = [](int v, int lo, int hi) { return v >= lo && v <= hi; };
    if (!in(c->mem_dim, 1, 512) || !in(c->time_dim, 1, 512) || !in(c->feat_dim, 1, 512) ||
        !in(c->emb_dim, 1, 512) || !in(c->num_neighbors, 1, 64) || !in(c->max_batch, 1, 65536))
        return TIG_EINVAL;
    if (c->num_heads != 1 && c->num_heads != 2 && c->num_heads != 4)
        return TIG_EINVAL;
    if ((c->mem_dim + c->time_dim) % c->num_heads != 0)
        return TIG_EINVAL;
    if (c->mem_dim + c->feat_dim + c->time_dim > 512)
        return TIG_EINVAL;
    if (c->precision != TIG_FP32 && c->precision != TIG_BF16_MFMA)
        return TIG_EINVAL;
    if (c->message_order != TIG_UPDATE_FIRST && c->message_order != TIG_DEFERRED)
        return TIG_EINVAL;
    return TIG_OK;
}

Dims make_dims(const tig_config &c)
{
    Dims d;
    d.M = c.mem_dim;
    d.T = c.time_dim;
    d.F = c.feat_dim;
    d.E = c.emb_dim;
    d.K = c.num_neighbors;
    d.H = c.num_heads;
    d.Dmsg = 2 * d.M + d.T + d.F;
    d.da = d.M + d.T;
    d.dh = d.da / d.H;
    d.dkv = d.M + d.F + d.T;
    d.prec = c.precision;
    d.KB = d.prec == TIG_BF16_MFMA ? 32 : 16;
    d.esz = 4;  // fp32, or a bf16 (hi, lo) pair
    d.Kg = round_up(d.Dmsg, d.KB);
    d.Khn = round_up(d.M, d.KB);
    d.Ng = round_up(d.M, 16);
    d.dkvp = round_up(d.dkv, d.KB);
    d.Mq = round_up(d.M, d.KB);
    d.N1 = d.H * d.dkvp;
    d.K2 = d.N1 + d.Mq;
    d.Ep = round_up(d.E, 16);
    d.Ek = round_up(d.E, d.KB);
    d.max_batch = c.max_batch;
    d.deferred = c.message_order == TIG_DEFERRED ? 1 : 0;
    return d;
}

constexpr int kLdsLimit = 160 * 1024;  // LDS per workgroup on gfx950

struct PersistentLayout {
    int32_t *src, *dst;
    double *ts;
    float *edge_feat;
    int64_t *indptr;
    CsrEntry *csr;
    int32_t *pos;
    float *mem;
    double *lu;
    unsigned long long *key[2];
    void *packed;
    size_t bytes;
};

PersistentLayout persistent_layout(const Dims &d, int64_t N, int64_t E, void *base)
{
    Carver c(base);
    PersistentLayout L;
    L.src = c.take<int32_t>((size_t)E);
    L.dst = c.take<int32_t>((size_t)E);
    L.ts = c.take<double>((size_t)E);
    L.edge_feat = c.take<float>((size_t)E * d.F);
    L.indptr = c.take<int64_t>((size_t)N + 1);
    L.csr = c.take<CsrEntry>((size_t)2 * E);
    L.pos = c.take<int32_t>((size_t)2 * E);
    L.mem = c.take<float>((size_t)N * d.M);
    L.lu = c.take<double>((size_t)N);
    L.key[0] = c.take<unsigned long long>((size_t)N);
    L.key[1] = c.take<unsigned long long>((size_t)N);
    L.packed = c.take<char>(packed_weights_bytes(d));
    L.bytes = c.off;
    return L;
}

StepScratch step_scratch(const Dims &d, void *base)
{
    Carver c(base);
    StepScratch S;
    const size_t B = (size_t)d.max_batch, R = 3 * B;
    for (int i = 0; i < 2; ++i) {
        QuerySet &q = S.qs[i];
        q.node = c.take<int32_t>(R);
        q.t = c.take<double>(R);
        q.cnt = c.take<int32_t>(R);
        q.self_ref = c.take<int32_t>(R);
        q.nbr = c.take<int32_t>(R * d.K);
        q.ref = c.take<int32_t>(R * d.K);
        q.eid = c.take<int32_t>(R * d.K);
        q.ts = c.take<double>(R * d.K);
        q.slot = c.take<int32_t>(2 * B);
        q.n_u = c.take<int32_t>(1);
    }
    S.staging = c.take<float>(2 * B * d.M);
    S.emb_u = c.take<float>(R * d.E);
    S.dec_a = c.take<float>(R * d.Ep);
    S.dec_b = c.take<float>(R * d.Ep);
    for (int i = 0; i < 2; ++i) {
        S.win[i] = c.take<WinDesc>(2 * B + 32);  // the overwrite reads a few descriptors past the count
        S.n_win[i] = c.take<int32_t>(1);
        S.flags[i] = c.take<uint8_t>(2 * B);
    }
    uint32_t slots = 1024;
    while (slots < 8 * B)  // four slots per (event, role) entry
        slots *= 2;
    S.tab_slots = slots;
    S.tab = c.take<unsigned long long>(slots);
    S.bytes = c.off;
    return S;
}

// raw fp32 weights staged in scratch during tig_init
struct RawWeights {
    tig_weights w;
    size_t bytes;
};

struct WeightField {
    const float *tig_weights::*member;
    size_t count;
};

int weight_fields(const Dims &d, WeightField *f)
{
    const size_t M = d.M, T = d.T, E = d.E, da = d.da, dkv = d.dkv, D = d.Dmsg;
    int n = 0;
    f[n++] = {&tig_weights::time_w, T};
    f[n++] = {&tig_weights::time_b, T};
    f[n++] = {&tig_weights::W_i, 3 * M * D};
    f[n++] = {&tig_weights::b_i, 3 * M};
    f[n++] = {&tig_weights::W_h, 3 * M * M};
    f[n++] = {&tig_weights::b_h, 3 * M};
    f[n++] = {&tig_weights::W_Q, da * da};
    f[n++] = {&tig_weights::b_Q, da};
    f[n++] = {&tig_weights::W_K, da * dkv};
    f[n++] = {&tig_weights::b_K, da};
    f[n++] = {&tig_weights::W_V, da * dkv};
    f[n++] = {&tig_weights::b_V, da};
    f[n++] = {&tig_weights::W_O, da * da};
    f[n++] = {&tig_weights::b_O, da};
    f[n++] = {&tig_weights::W_m1, E * (da + M)};
    f[n++] = {&tig_weights::b_m1, E};
    f[n++] = {&tig_weights::W_m2, E * E};
    f[n++] = {&tig_weights::b_m2, E};
    f[n++] = {&tig_weights::W_d1, E * 2 * E};
    f[n++] = {&tig_weights::b_d1, E};
    f[n++] = {&tig_weights::w_d2, E};
    f[n++] = {&tig_weights::b_d2, 1};
    return n;
}

RawWeights raw_weights_layout(const Dims &d, void *base)
{
    Carver c(base);
    RawWeights R;
    memset(&R.w, 0, sizeof(R.w));
    R.w.struct_size = sizeof(tig_weights);
    WeightField f[32];
    const int n = weight_fields(d, f);
    for (int i = 0; i < n; ++i)
        R.w.*(f[i].member) = c.take<float>(f[i].count);
    R.bytes = c.off;
    return R;
}

size_t init_scratch_bytes(const Dims &d, int64_t N, int64_t E)
{
    // [flags | raw weights | fold scratch]  and, after that is consumed, the adjacency sort
    const size_t a = 256 + raw_weights_layout(d, nullptr).bytes + pack_scratch_bytes(d);
    const size_t b = csr_build_scratch_bytes(E, N);
    return a > b ? a : b;
}

int fail(tig_ctx *ctx, int status, const char *what, hipError_t e = hipSuccess)
{
    if (ctx) {
        if (e != hipSuccess)
            snprintf(ctx->err, sizeof(ctx->err), "%s: %s", what, hipGetErrorString(e));
        else
            snprintf(ctx->err, sizeof(ctx->err), "%s", what);
    }
    return status;
}

thread_local char g_init_err[256] = "";

}  // namespace

namespace tig {
int fail_global(const char *what, hipError_t e)
{
    snprintf(g_init_err, sizeof(g_init_err), "%s: %s", what, hipGetErrorString(e));
    return TIG_EHIP;
}
}  // namespace tig

extern "C" {

int tig_workspace_bytes(const tig_config *cfg, const tig_graph *graph, size_t *persistent_bytes,
                        size_t *scratch_bytes)
{
    int rc = check_config(cfg);
    if (rc != TIG_OK)
        return rc;
    if (!graph || graph->struct_size != sizeof(tig_graph) || !persistent_bytes || !scratch_bytes)
        return TIG_EINVAL;
    if (graph->num_nodes < 1 || graph->num_nodes > 0x7FFFFFFF || graph->num_events < 0 ||
        graph->num_events >= ((int64_t)1 << 30))
        return TIG_EINVAL;
    const Dims d = make_dims(*cfg);
    LaunchPlan plan;
    if (!plan_launch(d, kLdsLimit, &plan))
        return TIG_EINVAL;
    *persistent_bytes = persistent_layout(d, graph->num_nodes, graph->num_events, nullptr).bytes;
    const size_t a = init_scratch_bytes(d, graph->num_nodes, graph->num_events);
    const size_t b = step_scratch(d, nullptr).bytes;
    *scratch_bytes = a > b ? a : b;
    return TIG_OK;
}

int tig_init(const tig_config *cfg, const tig_graph *graph, const tig_weights *weights,
             void *persistent, size_t persistent_bytes, void *scratch, size_t scratch_bytes,
             void *hip_stream, tig_ctx **out)
{
    if (!out)
        return TIG_EINVAL;
    *out = nullptr;
    size_t need_p = 0, need_s = 0;
    int rc = tig_workspace_bytes(cfg, graph, &need_p, &need_s);
    if (rc != TIG_OK)
        return rc;
    if ((weights && weights->struct_size != sizeof(tig_weights)) || !persistent || !scratch)
        return TIG_EINVAL;
    const int64_t N = graph->num_nodes, E = graph->num_events;
    if (E > 0 && (!graph->src || !graph->dst || !graph->ts || !graph->edge_feat))
        return TIG_EINVAL;
    if (persistent_bytes < need_p || scratch_bytes < need_s)
        return TIG_ENOSPACE;
    if (((uintptr_t)persistent & 255) || ((uintptr_t)scratch & 255))
        return TIG_EINVAL;
    const Dims d = make_dims(*cfg);
    WeightField wf[32];
    const int nwf = weight_fields(d, wf);
    for (int i = 0; weights && i < nwf; ++i)
        if (!(weights->*(wf[i].member)))
            return TIG_EINVAL;

    tig_ctx *ctx = new (std::nothrow) tig_ctx;
    if (!ctx)
        return TIG_ENOMEM;
    memset(ctx, 0, sizeof(*ctx));
    ctx->d = d;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->num_nodes = N;
    ctx->num_events = E;
    hipStream_t s = ctx->stream;

#define INIT_TRY(expr, what)                                                                \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            snprintf(g_init_err, sizeof(g_init_err), "%s: %s", what, hipGetErrorString(e_)); \
            delete ctx;                                                                     \
            return TIG_EHIP;                                                                \
        }                                                                                   \
    } while (0)

    if (!plan_launch(d, kLdsLimit, &ctx->plan)) {
        delete ctx;
        return TIG_EINVAL;
    }
    INIT_TRY(prepare_kernels(d, ctx->plan), "hipFuncSetAttribute");
    {
        int dev = 0;
        INIT_TRY(hipGetDevice(&dev), "hipGetDevice");
        INIT_TRY(hipDeviceGetAttribute(&ctx->num_cus, hipDeviceAttributeMultiprocessorCount, dev), "compute unit count");
        ctx->plan.num_cus = ctx->num_cus;
        INIT_TRY(static_scratch_of(dev, &ctx->static_scratch), "hipGetSymbolAddress(static scratch)");
    }

    const PersistentLayout L = persistent_layout(d, N, E, persistent);
    ctx->src = L.src;
    ctx->dst = L.dst;
    ctx->ts = L.ts;
    ctx->edge_feat = L.edge_feat;
    ctx->indptr = L.indptr;
    ctx->csr = L.csr;
    ctx->pos = L.pos;
    ctx->mem = L.mem;
    ctx->lu = L.lu;
    ctx->key[0] = L.key[0];
    ctx->key[1] = L.key[1];
    ctx->packed = L.packed;

    // graph copy (host or device source)
    if (E > 0) {
        INIT_TRY(hipMemcpyAsync(L.src, graph->src, sizeof(int32_t) * (size_t)E, hipMemcpyDefault, s), "copy src");
        INIT_TRY(hipMemcpyAsync(L.dst, graph->dst, sizeof(int32_t) * (size_t)E, hipMemcpyDefault, s), "copy dst");
        INIT_TRY(hipMemcpyAsync(L.ts, graph->ts, sizeof(double) * (size_t)E, hipMemcpyDefault, s), "copy ts");
        INIT_TRY(hipMemcpyAsync(L.edge_feat, graph->edge_feat, sizeof(float) * (size_t)E * d.F,
                                hipMemcpyDefault, s), "copy edge_feat");
    }
    // validation on the device
    int32_t *flags = (int32_t *)scratch;
    INIT_TRY(launch_fill_zero(flags, 256, s), "clear flags");
    INIT_TRY(launch_validate_graph(L.src, L.dst, L.ts, E, N, flags, s), "validate");
    int32_t hflags[4] = {0, 0, 0, 0};
    INIT_TRY(hipMemcpyAsync(hflags, flags, sizeof(hflags), hipMemcpyDeviceToHost, s), "read flags");
    INIT_TRY(hipStreamSynchronize(s), "sync");
    if (hflags[0] || hflags[1] || hflags[2]) {
        delete ctx;
        return hflags[0] ? TIG_ERANGE : (hflags[1] ? TIG_EUNSORTED : TIG_ESELFLOOP);
    }

    // weights: stage raw fp32 copies, then fold / pad / reorder
    ctx->has_model = weights != nullptr;
    if (weights) {
        char *wbase = (char *)scratch + 256;
        RawWeights R = raw_weights_layout(d, wbase);
        for (int i = 0; i < nwf; ++i)
            INIT_TRY(hipMemcpyAsync((void *)(R.w.*(wf[i].member)), weights->*(wf[i].member),
                                    sizeof(float) * wf[i].count, hipMemcpyDefault, s), "copy weights");
        INIT_TRY(pack_weights(d, R.w, L.packed, wbase + R.bytes, &ctx->pw, s), "pack weights");
        INIT_TRY(hipStreamSynchronize(s), "sync");
    }

    // temporal adjacency
    INIT_TRY(csr_build(L.src, L.dst, L.ts, E, N, L.indptr, L.csr, L.pos, scratch, scratch_bytes, s), "adjacency build");

    // state after a reset
    INIT_TRY(launch_fill_zero(L.mem, sizeof(float) * (size_t)N * d.M, s), "zero memory");
    INIT_TRY(launch_fill_zero(L.lu, sizeof(double) * (size_t)N, s), "zero last_update");
    INIT_TRY(launch_fill_zero(L.key[0], sizeof(unsigned long long) * (size_t)N, s), "zero keys");
    INIT_TRY(launch_fill_zero(L.key[1], sizeof(unsigned long long) * (size_t)N, s), "zero keys");
    INIT_TRY(hipStreamSynchronize(s), "sync");

    // per-step intermediates: counters and the claim table start from zero
    ctx->S = step_scratch(d, scratch);
    ctx->scratch = scratch;
    for (int i = 0; i < 2; ++i) {
        INIT_TRY(launch_fill_zero(ctx->S.n_win[i], 4, s), "clear counters");
        INIT_TRY(launch_fill_zero(ctx->S.qs[i].n_u, 4, s), "clear counters");
    }
    INIT_TRY(launch_fill_zero(ctx->S.tab, sizeof(unsigned long long) * (size_t)ctx->S.tab_slots, s), "clear claim table");
    INIT_TRY(hipStreamSynchronize(s), "sync");
#undef INIT_TRY
    if (hipHostMalloc((void **)&ctx->rows_seen_host, 64, hipHostMallocMapped) == hipSuccess) {
        ctx->rows_seen_host[0] = ctx->rows_seen_host[1] = 0;
        if (hipHostGetDevicePointer((void **)&ctx->rows_seen_dev, ctx->rows_seen_host, 0) != hipSuccess) {
            (void)hipHostFree(ctx->rows_seen_host);
            ctx->rows_seen_host = ctx->rows_seen_dev = nullptr;
        }
    } else {
        (void)hipGetLastError();
        ctx->rows_seen_host = ctx->rows_seen_dev = nullptr;
    }
    *out = ctx;
    return TIG_OK;
}

// A query preparation job for batch (first_eid, count) into query set `qs`.
static DedupJob make_dedup(const StepScratch &S, const QuerySet &qs, int64_t first_eid, int32_t count,
                           uint32_t epoch, bool shared)
{
    DedupJob j;
    j.first_eid = first_eid;
    j.count = count;
    j.qs = qs;
    j.tab = S.tab;
    j.tab_mask = S.tab_slots - 1;
    j.epoch = epoch;
    j.n_wgs = prepare_workgroups(count, shared);
    return j;
}

// `use_static`: every per-step intermediate lives in this device's static scratch array instead of
// the context's scratch workspace, the call prepares everything itself (winners, queries), and
// nothing is kept there for a later call.
struct TrainCall {
    float lr;
    float *loss_out;
};

static int step_impl(tig_ctx *ctx, const tig_batch *batch, const tig_out *out, hipEvent_t *marks,
                     bool use_static = false, const TrainCall *train = nullptr)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!batch || batch->struct_size != sizeof(tig_batch) || !out || out->struct_size != sizeof(tig_out))
        return fail(ctx, TIG_EINVAL, "tig_step: NULL argument or wrong struct_size");
    if (batch->count < 1 || batch->count > ctx->d.max_batch)
        return fail(ctx, TIG_EINVAL, "tig_step: count outside 1..max_batch");
    if (batch->first_eid < 0 || batch->first_eid + batch->count > ctx->num_events)
        return fail(ctx, TIG_ERANGE, "tig_step: event range leaves the graph");
    if (!out->emb || !out->score_pos || (batch->neg_dst && !out->score_neg))
        return fail(ctx, TIG_EINVAL, "tig_step: required output pointer is NULL");
    if (batch->first_eid < ctx->cursor)
        return fail(ctx, TIG_EORDER, "tig_step: batch starts before the end of the previous one");
    const bool general = ctx->mods_ws != nullptr;
    if (!general && !ctx->has_model)
        return fail(ctx, TIG_EINVAL, "tig_step: the context was created without weights and no module selection is attached");
    if (general && (use_static || train))
        return fail(ctx, TIG_EINVAL, "tig_step_static / tig_train_step: the context runs an attached module selection");
    // a training step or a step of a module selection has no embedding launch to carry a later
    // step's preparation (a training step runs it on its second stream instead, see side_prep)
    const bool solo = train || general;
    const bool wants_queries = !general || ctx->mods.emb == TIG_EMB_ATTENTION;
    StepScratch st = ctx->S;
    if (use_static) {
        if (ctx->d.deferred)
            return fail(ctx, TIG_EINVAL, "tig_step_static: the context runs the deferred message order");
        if (step_scratch(ctx->d, nullptr).bytes > (size_t)TIG_STATIC_SCRATCH_BYTES)
            return fail(ctx, TIG_ENOSPACE, "tig_step_static: the per-step intermediates of this configuration "
                                           "exceed TIG_STATIC_SCRATCH_BYTES");
        st = step_scratch(ctx->d, ctx->static_scratch);
    }
    const Dims &d = ctx->d;
    const int64_t first = batch->first_eid;
    const int32_t count = batch->count;

    StepArgs a;
    memset(&a, 0, sizeof(a));
    a.src = ctx->src;
    a.dst = ctx->dst;
    a.ts = ctx->ts;
    a.edge_feat = ctx->edge_feat;
    a.indptr = ctx->indptr;
    a.csr = ctx->csr;
    a.pos = ctx->pos;
    a.num_nodes = ctx->num_nodes;
    a.mem = ctx->mem;
    a.lu = ctx->lu;
    a.first_eid = first;
    a.count = count;
    a.roles = batch->neg_dst ? 3 : 2;
    a.neg = batch->neg_dst;
    a.staging = st.staging;
    a.emb_u = st.emb_u;
    a.dec_a = st.dec_a;
    a.dec_b = st.dec_b;
    a.emb = out->emb;
    a.score_pos = out->score_pos;
    a.score_neg = out->score_neg;
    if (wants_queries) {
        a.out_nbr_node = out->nbr_node;
        a.out_nbr_eid = out->nbr_eid;
        a.out_nbr_ts = out->nbr_ts;
        a.out_nbr_cnt = out->nbr_cnt;
    }
    a.out_is_winner = out->is_winner;
    a.rows_seen = ctx->rows_seen_dev;
    if (ctx->rows_seen_host) {
        // distinct rows of a recent step, with a margin of one eighth
        const int32_t seen = ((volatile int32_t *)ctx->rows_seen_host)[0];
        const int32_t wins = ((volatile int32_t *)ctx->rows_seen_host)[1];
        a.rows_est = seen > 0 ? seen + seen / 8 : 0;
        a.wins_est = wins > 0 ? wins + wins / 8 : 0;
    }

    // What the embedding launch can do on the side for a later step (never for a static call).
    const bool one_wg = winners_in_one_launch(count);
    const int spare = use_static || solo ? 0 : embed_spare_workgroups(d, ctx->plan, a.roles, count);
    uint32_t epoch = ctx->epoch;
    bool clear_tab = use_static;  // the static array's table holds claims of unknown epochs
    auto next_epoch = [&]() -> uint32_t {
        if (use_static)
            return 1u;
        if (++epoch == 0u) {  // wrapped: claims of 2^32 jobs ago would read as current
            clear_tab = true;
            epoch = 1u;
        }
        return epoch;
    };

    StepPlan sp = {};
    SelectJob sel_now = {}, sel_side = {};
    DedupJob ded_now = {}, ded_side = {};
    // a training step has no embedding launch to carry such work: it goes to the step's second stream
    const bool side_prep = train && ctx->have_train_side;
    int launches = 2;  // embedding, closing

    // ---- the distinct queries of this batch: prepared by the previous step's embedding launch if
    // that step guessed this batch (it reads the event stream and the adjacency only), else now
    const bool q_ready = !use_static && !general && ctx->ahead_q_valid && ctx->ahead_q_first == first &&
                         ctx->ahead_q_count == count;
    const int qi = use_static ? 0 : (q_ready ? ctx->qcur ^ 1 : ctx->qcur);
    a.qs = st.qs[qi];
    a.finish_here = !(q_ready && ctx->ahead_q_finished);
    if (!q_ready && wants_queries) {
        ded_now = make_dedup(st, st.qs[qi], first, count, next_epoch(), one_wg);
        sp.prep_ded = &ded_now;
    }

    // ---- the winners the GRU and the memory overwrite apply
    int wi;  // list applied by this step
    bool w_ready = false;
    if (!d.deferred) {
        // this batch's: selected ahead like the queries, else now
        w_ready = !use_static && !solo && ctx->ahead_w_valid && ctx->ahead_w_first == first &&
                  ctx->ahead_w_count == count;
        wi = use_static ? 0 : (w_ready ? ctx->wcur ^ 1 : ctx->wcur);
        a.msg_first_eid = first;
        a.msg_count = count;
        a.win_flags = st.flags[wi];
        if (!w_ready) {
            sel_now = SelectJob{first, count, st.win[wi], st.n_win[wi], st.flags[wi], ctx->key[wi]};
            (one_wg ? sp.prep_sel : sp.big_sel) = &sel_now;
        }
    } else {
        // Deferred order: the winners kept by the previous step.  This batch's go to the other list,
        // selected by one workgroup of the embedding launch when it can carry it, else up front
        // (each list has a key array of its own, so the row references of this step, which need
        // the applied batch's keys, are not disturbed).
        wi = ctx->wcur;
        a.msg_first_eid = ctx->pend_first;
        a.msg_count = ctx->pend_valid ? ctx->pend_count : 0;
        a.win_flags = st.flags[wi ^ 1];
        const SelectJob mine = SelectJob{first, count, st.win[wi ^ 1], st.n_win[wi ^ 1], st.flags[wi ^ 1],
                                         ctx->key[wi ^ 1]};
        if (spare > 0 && one_wg) {
            a.sel = mine;
        } else if (side_prep && one_wg) {
            sel_side = mine;
            sp.side_sel = &sel_side;
        } else {
            sel_now = mine;
            (one_wg ? sp.prep_sel : sp.big_sel) = &sel_now;
        }
    }
    a.win = st.win[wi];
    a.n_win = st.n_win[wi];
    a.msg_key = ctx->key[wi];
    // ---- the GRU of the applied batch: run by the previous step's closing launch if that step knew
    // the batch (and the memory has not changed since), else now, together with what is left of
    // this step's query preparation
    // (a training step runs it itself: its backward pass reads the gates that this launch leaves)
    const bool g_ready = !use_static && !general && !train && ctx->ahead_g_valid && a.msg_count > 0 && ctx->ahead_g_first == a.msg_first_eid &&
                         ctx->ahead_g_count == a.msg_count && !a.finish_here && (d.deferred || w_ready);
    sp.gru_now = !general && !g_ready && (a.msg_count > 0 || a.finish_here);
    if (general) {
        sp.mods = &ctx->mods;
        launches += ctx->mods.fused_embed ? 2 : (wants_queries ? 4 : 2);  // update[, overwrite][, finishing pass], embedding, decoder / closing
    }
    if (sp.big_sel)
        launches += 2;
    if (sp.prep_sel || sp.prep_ded)
        launches += 1;
    if (sp.gru_now)
        launches += 1;
    sp.clear_tab = clear_tab && sp.prep_ded;

    // ---- Chronological training and evaluation pass consecutive batches of one size: guess that
    // the next call continues where this one ends, and let the embedding launch prepare that batch
    // (its queries; in the update-first order also its winners) on compute units it leaves idle.
    const int64_t next_first = first + count;
    if (spare > 0 && next_first < ctx->num_events) {
        const int64_t left = ctx->num_events - next_first;
        const int32_t guess = left < count ? (int32_t)left : count;
        if (winners_in_one_launch(guess)) {
            a.ded = make_dedup(st, st.qs[qi ^ 1], next_first, guess, next_epoch(), true);
            // that set's counter was cleared by the closing launch of the step that used the set,
            // unless this step did not take the set prepared for it
            if (!q_ready)
                sp.clear_first = st.qs[qi ^ 1].n_u;
            if (!d.deferred)
                a.sel = SelectJob{next_first, guess, st.win[wi ^ 1], st.n_win[wi ^ 1], st.flags[wi ^ 1],
                                  ctx->key[wi ^ 1]};
            // The decode launch finishes that preparation: row references against the batch the NEXT
            // step applies -- the guessed batch itself, or in the deferred order this step's batch
            // (selected into the other list by now, by the embedding launch or up front).
            a.fin_count = guess;
            a.fin_msg_first_eid = d.deferred ? first : next_first;
            a.fin_msg_count = d.deferred ? count : guess;
            a.fin_msg_key = ctx->key[wi ^ 1];
        }
    }
    if (side_prep && next_first < ctx->num_events) {
        const int64_t left = ctx->num_events - next_first;
        const int32_t guess = left < count ? (int32_t)left : count;
        if (winners_in_one_launch(guess)) {
            // (the step that takes the set finishes it: slots, row references)
            ded_side = make_dedup(st, st.qs[qi ^ 1], next_first, guess, next_epoch(), true);
            sp.side_ded = &ded_side;
            if (!q_ready)
                sp.clear_first = st.qs[qi ^ 1].n_u;
        }
    }
    if (sp.side_sel || sp.side_ded)
        launches += 1;
    // ---- The closing launch also runs the GRU of the batch the next step applies, once that batch's
    // winners are known: in the update-first order the guessed batch (selected by this step's
    // embedding launch), in the deferred order this step's own batch (whatever comes next).
    if (!use_static && !solo) {
        if (!d.deferred && a.sel.count > 0)
            sp.ahead = GruAhead{a.sel.first_eid, a.sel.count, st.win[wi ^ 1], st.n_win[wi ^ 1]};
        else if (d.deferred)
            sp.ahead = GruAhead{first, count, st.win[wi ^ 1], st.n_win[wi ^ 1]};
    }
    if (clear_tab && !sp.prep_ded && (a.ded.count > 0 || sp.side_ded)) {
        // the epoch wrapped and only the side job uses the table: clear it ahead of everything
        const hipError_t e = launch_fill_zero(st.tab, sizeof(unsigned long long) * (size_t)st.tab_slots, ctx->stream);
        if (e != hipSuccess)
            return fail(ctx, TIG_EHIP, "tig_step: clearing the claim table", e);
    }

    if (!train && ctx->train_ws && ctx->embed_stale) {
        const hipError_t e = train_refold_embed(d, ctx->train_ws, ctx->packed, &ctx->pw, ctx->stream);
        if (e != hipSuccess)
            return fail(ctx, TIG_EHIP, "tig_step: re-folding the weights after training steps", e);
        ctx->embed_stale = false;
    }
    if (train) {
        sp.train = true;
        sp.train_ws = ctx->train_ws;
        sp.packed = ctx->packed;
        sp.pw_out = &ctx->pw;
        sp.lr = train->lr;
        sp.loss_out = train->loss_out;
        sp.train_side = ctx->have_train_side ? &ctx->train_side : nullptr;
        a.gru_gates = train_gates_buffer(d, ctx->train_ws);
    }
    const hipError_t e = launch_step(d, ctx->plan, ctx->pw, a, sp, ctx->stream, marks);
    // bit i: the interval between marks i and i + 1 held a kernel (a module selection's kernels fill
    // intervals 3 and 4)
    ctx->last_ran = (sp.big_sel ? 3u : 0u) | ((sp.prep_sel || sp.prep_ded) ? 4u : 0u) |
                    ((sp.mods || sp.gru_now) ? 8u : 0u) | 16u | ((sp.mods || (train && !wants_inspection(a))) ? 0u : 32u);
    if (e != hipSuccess) {
        // kernels of this step may already be enqueued: nothing prepared ahead is trusted any more,
        // and the model state is undefined until tig_reset / tig_state_import
        ctx->ahead_g_valid = false;
        if (!use_static) {
            ctx->ahead_w_valid = false;
            ctx->ahead_q_valid = false;
            ctx->epoch = epoch;
        }
        return fail(ctx, TIG_EHIP, "tig_step launch", e);
    }
    if (train && train->lr != 0.0f)
        ctx->embed_stale = true;
    ctx->cursor = next_first;
    ctx->last_launches = launches;
    ctx->ahead_g_valid = sp.ahead.count > 0;  // (never after a static call: the memory has changed)
    ctx->ahead_g_first = sp.ahead.first_eid;
    ctx->ahead_g_count = sp.ahead.count;
    if (use_static)
        return TIG_OK;  // the context's own lists and sets are untouched: winners and queries prepared ahead stay usable
    ctx->epoch = epoch;
    ctx->qcur = qi;
    const DedupJob &ded_ahead = sp.side_ded ? ded_side : a.ded;
    ctx->ahead_q_valid = ded_ahead.count > 0;
    ctx->ahead_q_finished = a.fin_count > 0;
    ctx->ahead_q_first = ded_ahead.first_eid;
    ctx->ahead_q_count = ded_ahead.count;
    if (d.deferred) {
        ctx->wcur = wi ^ 1;  // the list just selected is the one the next step applies
        ctx->pend_valid = true;
        ctx->pend_first = first;
        ctx->pend_count = count;
    } else {
        ctx->wcur = wi;
        ctx->ahead_w_valid = a.sel.count > 0;
        ctx->ahead_w_first = a.sel.first_eid;
        ctx->ahead_w_count = a.sel.count;
    }
    return TIG_OK;
}

int tig_step(tig_ctx *ctx, const tig_batch *batch, const tig_out *out)
{
    return step_impl(ctx, batch, out, nullptr);
}

int tig_step_static(tig_ctx *ctx, const tig_batch *batch, const tig_out *out)
{
    return step_impl(ctx, batch, out, nullptr, true);
}

// ---- training (Sec. II-C self-supervised signal; Alg. 2 "Backward and Optimize") ---------------

int tig_train_workspace_bytes(const tig_config *cfg, size_t *bytes)
{
    const int rc = check_config(cfg);
    if (rc != TIG_OK)
        return rc;
    if (!bytes)
        return TIG_EINVAL;
    const Dims d = make_dims(*cfg);
    if (!train_supported(d))
        return TIG_EINVAL;
    *bytes = train_workspace_bytes(d);
    return TIG_OK;
}

int tig_train_attach(tig_ctx *ctx, const tig_weights *weights, void *workspace, size_t workspace_bytes)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!weights || weights->struct_size != sizeof(tig_weights) || !workspace || ((uintptr_t)workspace & 255))
        return fail(ctx, TIG_EINVAL, "tig_train_attach: NULL / misaligned argument or wrong struct_size");
    WeightField wf[32];
    const int nwf = weight_fields(ctx->d, wf);
    for (int i = 0; i < nwf; ++i)
        if (!(weights->*(wf[i].member)))
            return fail(ctx, TIG_EINVAL, "tig_train_attach: a weight pointer is NULL");
    if (ctx->mods_ws || !ctx->has_model)
        return fail(ctx, TIG_EINVAL, "tig_train_attach: the context runs a module selection or has no model of its own");
    if (!train_supported(ctx->d))
        return fail(ctx, TIG_EINVAL, "tig_train_attach: training needs an fp32 context whose rows fit the backward kernels");
    if (workspace_bytes < train_workspace_bytes(ctx->d))
        return fail(ctx, TIG_ENOSPACE, "tig_train_attach: workspace too small");
    hipError_t e = prepare_train(ctx->d);
    if (e == hipSuccess && !ctx->have_train_side) {
        // (default priority; non-blocking: no implicit ordering against the legacy default stream)
        TrainSide ts = {};
        int made = 0;
        e = hipStreamCreateWithFlags(&ts.stream, hipStreamNonBlocking);
        for (; e == hipSuccess && made <= kTrainForks; ++made)
            e = hipEventCreateWithFlags(made < kTrainForks ? &ts.fork[made] : &ts.join, hipEventDisableTiming);
        if (e == hipSuccess) {
            ctx->train_side = ts;
            ctx->have_train_side = true;
        } else if (ts.stream) {
            for (int i = 0; i < made - 1; ++i)
                (void)hipEventDestroy(i < kTrainForks ? ts.fork[i] : ts.join);
            (void)hipStreamDestroy(ts.stream);
        }
    }
    if (e == hipSuccess)
        e = train_attach(ctx->d, *weights, workspace, ctx->packed, &ctx->pw, ctx->stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_train_attach", e);
    ctx->train_ws = workspace;
    ctx->ahead_g_valid = false;  // staged rows of another set of weights
    return TIG_OK;
}

int tig_train_step(tig_ctx *ctx, const tig_batch *batch, const tig_out *out, float lr, float *loss_out)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!ctx->train_ws)
        return fail(ctx, TIG_EINVAL, "tig_train_step: no training workspace attached (tig_train_attach)");
    if (!batch || batch->struct_size != sizeof(tig_batch) || !batch->neg_dst)
        return fail(ctx, TIG_EINVAL, "tig_train_step: the loss needs one negative per event");
    if (!(lr >= 0.0f))
        return fail(ctx, TIG_EINVAL, "tig_train_step: negative learning rate");
    const TrainCall tc = {lr, loss_out};
    return step_impl(ctx, batch, out, nullptr, false, &tc);
}

int tig_train_get(tig_ctx *ctx, int32_t what, const tig_weights *dst)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!ctx->train_ws || !dst || dst->struct_size != sizeof(tig_weights) || (what != 0 && what != 1))
        return fail(ctx, TIG_EINVAL, "tig_train_get: no workspace attached, NULL destination or unknown selector");
    const hipError_t e = train_copy_out(ctx->d, ctx->train_ws, what == 1, *dst, ctx->stream);
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_train_get", e);
    return TIG_OK;
}

// ---- other instances of the general architecture (Sec. II-C) -------------------------------------

static int check_modules(const tig_modules *m)
{
    if (!m || m->struct_size != sizeof(tig_modules))
        return TIG_EINVAL;
    if (m->aggregator != TIG_AGG_LAST && m->aggregator != TIG_AGG_MEAN)
        return TIG_EINVAL;
    if (m->updater != TIG_UPD_GRU && m->updater != TIG_UPD_RNN)
        return TIG_EINVAL;
    if (m->embedding != TIG_EMB_ATTENTION && m->embedding != TIG_EMB_IDENTITY && m->embedding != TIG_EMB_TIME_PROJECTION)
        return TIG_EINVAL;
    if (m->embedding == TIG_EMB_TIME_PROJECTION && !m->time_proj_w)
        return TIG_EINVAL;
    if (m->num_layers < 0 || m->num_layers > 2)
        return TIG_EINVAL;
    if (m->num_layers == 2) {
        const tig_layer_weights *l = m->layer2;
        if (m->embedding != TIG_EMB_ATTENTION || !l || l->struct_size != sizeof(tig_layer_weights) || !l->W_Q || !l->b_Q ||
            !l->W_K || !l->b_K || !l->W_V || !l->b_V || !l->W_O || !l->b_O || !l->W_m1 || !l->b_m1 || !l->W_m2 || !l->b_m2)
            return TIG_EINVAL;
    }
    return TIG_OK;
}

int tig_modules_workspace_bytes(const tig_config *cfg, const tig_modules *modules, int64_t num_nodes, size_t *bytes)
{
    int rc = check_config(cfg);
    if (rc == TIG_OK)
        rc = check_modules(modules);
    if (rc != TIG_OK)
        return rc;
    if (!bytes || num_nodes < 1 || num_nodes > 0x7FFFFFFF)
        return TIG_EINVAL;
    const Dims d = make_dims(*cfg);
    if (!modules_supported(d, *modules))
        return TIG_EINVAL;
    *bytes = modules_workspace_bytes(d, *modules, num_nodes);
    return TIG_OK;
}

int tig_modules_attach(tig_ctx *ctx, const tig_modules *modules, const tig_weights *weights, void *workspace,
                       size_t workspace_bytes)
{
    if (!ctx)
        return TIG_EINVAL;
    if (check_modules(modules) != TIG_OK || !weights || weights->struct_size != sizeof(tig_weights) || !workspace ||
        ((uintptr_t)workspace & 255))
        return fail(ctx, TIG_EINVAL, "tig_modules_attach: NULL / misaligned argument, wrong struct_size or unknown selector");
    if (ctx->train_ws)
        return fail(ctx, TIG_EINVAL, "tig_modules_attach: the context has a training workspace");
    if (!modules_supported(ctx->d, *modules))
        return fail(ctx, TIG_EINVAL, "tig_modules_attach: needs an fp32 context (emb_dim == mem_dim unless the embedding is "
                                     "attention; two layers: emb_dim + time_dim divisible by num_heads) whose rows fit the kernels");
    const tig_weights &w = *weights;
    const bool attn = modules->embedding == TIG_EMB_ATTENTION;
    if (!w.time_w || !w.time_b || !w.W_i || !w.b_i || !w.W_h || !w.b_h || !w.W_d1 || !w.b_d1 || !w.w_d2 || !w.b_d2 ||
        (attn && (!w.W_Q || !w.b_Q || !w.W_K || !w.b_K || !w.W_V || !w.b_V || !w.W_O || !w.b_O || !w.W_m1 || !w.b_m1 ||
                  !w.W_m2 || !w.b_m2)))
        return fail(ctx, TIG_EINVAL, "tig_modules_attach: a weight pointer the selection needs is NULL");
    if (workspace_bytes < modules_workspace_bytes(ctx->d, *modules, ctx->num_nodes))
        return fail(ctx, TIG_ENOSPACE, "tig_modules_attach: workspace too small");
    hipError_t e = hipStreamSynchronize(ctx->stream);
    ModParams mp;
    if (e == hipSuccess)
        e = modules_attach(ctx->d, *modules, w, ctx->num_nodes, workspace, &mp, ctx->stream);
    if (e == hipSuccess && mp.fused_embed) {
        // the fused embedding / closing kernels run this selection's attention: their prepared weights
        // are folded from `weights` as in tig_init (staged through the scratch workspace, whose
        // per-step counters and claim table are then put back to their resting state)
        hipStream_t s = ctx->stream;
        char *wbase = (char *)ctx->scratch + 256;
        RawWeights R = raw_weights_layout(ctx->d, wbase);
        WeightField wf[32];
        const int nwf = weight_fields(ctx->d, wf);
        for (int i = 0; i < nwf && e == hipSuccess; ++i) {
            if (wf[i].member == &tig_weights::W_i || wf[i].member == &tig_weights::b_i ||
                wf[i].member == &tig_weights::W_h || wf[i].member == &tig_weights::b_h)
                continue;  // the state update has kernels of its own
            e = hipMemcpyAsync((void *)(R.w.*(wf[i].member)), w.*(wf[i].member), sizeof(float) * wf[i].count,
                               hipMemcpyDefault, s);
        }
        if (e == hipSuccess)
            e = pack_weights(ctx->d, R.w, ctx->packed, wbase + R.bytes, &ctx->pw, s, kPackEmbed);
        for (int i = 0; i < 2 && e == hipSuccess; ++i) {
            e = launch_fill_zero(ctx->S.n_win[i], 4, s);
            if (e == hipSuccess)
                e = launch_fill_zero(ctx->S.qs[i].n_u, 4, s);
        }
        if (e == hipSuccess)
            e = launch_fill_zero(ctx->S.tab, sizeof(unsigned long long) * (size_t)ctx->S.tab_slots, s);
        if (e == hipSuccess)
            e = hipStreamSynchronize(s);
    }
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_modules_attach", e);
    ctx->mods = mp;
    ctx->mods_ws = workspace;
    // nothing prepared by earlier steps of another model is trusted
    ctx->ahead_g_valid = false;
    ctx->ahead_w_valid = false;
    ctx->ahead_q_valid = false;
    ctx->pend_valid = false;  // (a deferred step's kept winners lived in the scratch workspace)
    return TIG_OK;
}

int tig_step_profiled(tig_ctx *ctx, const tig_batch *batch, const tig_out *out, float *kernel_ms)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!kernel_ms)
        return fail(ctx, TIG_EINVAL, "tig_step_profiled: kernel_ms is NULL");
    if (!ctx->have_marks) {
        for (int i = 0; i <= kNumStepKernels; ++i) {
            const hipError_t e = hipEventCreate(&ctx->marks[i]);
            if (e != hipSuccess) {
                for (int j = 0; j < i; ++j)
                    (void)hipEventDestroy(ctx->marks[j]);
                return fail(ctx, TIG_EHIP, "hipEventCreate", e);
            }
        }
        ctx->have_marks = true;
    }
    const int rc = step_impl(ctx, batch, out, ctx->marks);
    if (rc != TIG_OK)
        return rc;
    hipError_t e = hipEventSynchronize(ctx->marks[kNumStepKernels]);
    for (int i = 0; i < kNumStepKernels && e == hipSuccess; ++i)
        e = hipEventElapsedTime(&kernel_ms[i], ctx->marks[i], ctx->marks[i + 1]);
    for (int i = 0; i < kNumStepKernels; ++i)
        if (!((ctx->last_ran >> i) & 1u))
            kernel_ms[i] = 0.0f;  // (an empty interval still reads a few microseconds)
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_step_profiled timing", e);
    return TIG_OK;
}

// The cursor is rewound: forget the winners kept for the next step (deferred order) and the ones
// selected ahead, and clear the key arrays (a selection of more than 4096 events merges its keys
// into them with atomicMax and needs every older key to be smaller; the keys of a list selected
// ahead go with them, so that list is dropped too).  Queries prepared ahead stay valid.
static hipError_t drop_pending(tig_ctx *ctx)
{
    hipError_t e = launch_fill_zero(ctx->key[0], sizeof(unsigned long long) * (size_t)ctx->num_nodes, ctx->stream);
    if (e == hipSuccess)
        e = launch_fill_zero(ctx->key[1], sizeof(unsigned long long) * (size_t)ctx->num_nodes, ctx->stream);
    if (ctx->d.deferred && ctx->pend_valid)
        ctx->ahead_q_finished = false;  // its row references point at the pending batch's staged rows
    ctx->pend_valid = false;
    ctx->ahead_w_valid = false;
    ctx->ahead_g_valid = false;  // computed from the memory that has just been replaced
    return e;
}

int tig_reset(tig_ctx *ctx)
{
    if (!ctx)
        return TIG_EINVAL;
    hipError_t e = launch_fill_zero(ctx->mem, sizeof(float) * (size_t)ctx->num_nodes * ctx->d.M, ctx->stream);
    if (e == hipSuccess)
        e = launch_fill_zero(ctx->lu, sizeof(double) * (size_t)ctx->num_nodes, ctx->stream);
    if (e == hipSuccess)
        e = drop_pending(ctx);
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_reset", e);
    ctx->cursor = 0;
    return TIG_OK;
}

int tig_state_export(tig_ctx *ctx, float *mem_out, double *last_update_out)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!mem_out || !last_update_out)
        return fail(ctx, TIG_EINVAL, "tig_state_export: NULL pointer");
    hipError_t e = hipMemcpyAsync(mem_out, ctx->mem, sizeof(float) * (size_t)ctx->num_nodes * ctx->d.M,
                                  hipMemcpyDefault, ctx->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(last_update_out, ctx->lu, sizeof(double) * (size_t)ctx->num_nodes,
                           hipMemcpyDefault, ctx->stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_state_export", e);
    return TIG_OK;
}

int tig_state_import(tig_ctx *ctx, const float *mem_in, const double *last_update_in)
{
    if (!ctx)
        return TIG_EINVAL;
    if (!mem_in || !last_update_in)
        return fail(ctx, TIG_EINVAL, "tig_state_import: NULL pointer");
    hipError_t e = hipMemcpyAsync(ctx->mem, mem_in, sizeof(float) * (size_t)ctx->num_nodes * ctx->d.M,
                                  hipMemcpyDefault, ctx->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ctx->lu, last_update_in, sizeof(double) * (size_t)ctx->num_nodes,
                           hipMemcpyDefault, ctx->stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess)
        e = drop_pending(ctx);
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_state_import", e);
    ctx->cursor = 0;
    return TIG_OK;
}

// ---- epoch machinery on one GPU (Sec. II-C "Distributed Parallel Training", Alg. 2) -------------

int tig_pac_epoch(tig_pac_part *parts, int32_t n_parts, int64_t *steps_out)
{
    if (!parts || n_parts < 1)
        return TIG_EINVAL;
    int64_t most = 0;
    for (int k = 0; k < n_parts; ++k) {
        tig_pac_part &p = parts[k];
        if (p.struct_size != sizeof(tig_pac_part) || !p.ctx || !p.out || !p.backup_mem || !p.backup_lu)
            return TIG_EINVAL;
        if (p.batch < 1 || p.batch > p.ctx->d.max_batch || p.num_events < 1 || p.num_events > p.ctx->num_events)
            return fail(p.ctx, TIG_EINVAL, "tig_pac_epoch: batch or num_events outside the context's limits");
        const int64_t nb = (p.num_events + p.batch - 1) / p.batch;
        most = nb > most ? nb : most;
    }
    // Every partition cycles over its own batches until the one with the most batches has finished a
    // data cycle: memory reset at the start of a cycle, backup at its end (Alg. 2).
    for (int64_t step = 0; step < most; ++step) {
        for (int k = 0; k < n_parts; ++k) {
            tig_pac_part &p = parts[k];
            const int64_t nb = (p.num_events + p.batch - 1) / p.batch;
            const int64_t i = step % nb;
            int rc = TIG_OK;
            if (i == 0)
                rc = tig_reset(p.ctx);
            if (rc != TIG_OK)
                return rc;
            tig_batch b;
            b.struct_size = sizeof(tig_batch);
            b.first_eid = i * p.batch;
            const int64_t left = p.num_events - b.first_eid;
            b.count = (int32_t)(left < p.batch ? left : p.batch);
            b.neg_dst = p.neg_dst ? p.neg_dst + b.first_eid : nullptr;
            if ((rc = step_impl(p.ctx, &b, p.out, nullptr)) != TIG_OK)
                return rc;
            if (i == nb - 1 && (rc = tig_state_export(p.ctx, p.backup_mem, p.backup_lu)) != TIG_OK)
                return rc;
        }
    }
    // end of the epoch: every memory goes back to its latest backup, the end of a complete cycle
    for (int k = 0; k < n_parts; ++k) {
        const int rc = tig_state_import(parts[k].ctx, parts[k].backup_mem, parts[k].backup_lu);
        if (rc != TIG_OK)
            return rc;
    }
    if (steps_out)
        *steps_out = most;
    return TIG_OK;
}

int tig_pac_sync_shared(tig_ctx *const *ctxs, int32_t n_parts, const int32_t *const *local_ids, int64_t n_shared,
                        int32_t mode)
{
    if (!ctxs || n_parts < 1 || n_parts > kMaxSyncParts || !local_ids || n_shared < 0 || (mode != 0 && mode != 1))
        return TIG_EINVAL;
    SyncArgs a;
    memset(&a, 0, sizeof(a));
    for (int k = 0; k < n_parts; ++k) {
        if (!ctxs[k] || !local_ids[k])
            return TIG_EINVAL;
        if (ctxs[k]->d.M != ctxs[0]->d.M || ctxs[k]->stream != ctxs[0]->stream)
            return fail(ctxs[k], TIG_EINVAL, "tig_pac_sync_shared: contexts differ in memory width or stream");
        for (int j = 0; j < k; ++j)
            if (ctxs[j] == ctxs[k])
                return TIG_EINVAL;
        a.mem[k] = ctxs[k]->mem;
        a.lu[k] = ctxs[k]->lu;
        a.ids[k] = local_ids[k];
        a.num_nodes[k] = ctxs[k]->num_nodes;
    }
    a.n_parts = n_parts;
    a.M = ctxs[0]->d.M;
    a.mode = mode;
    a.n_shared = n_shared;
    const hipError_t e = launch_sync_shared(a, ctxs[0]->stream);
    for (int k = 0; k < n_parts; ++k)
        ctxs[k]->ahead_g_valid = false;  // staged GRU rows were computed from the memory before the exchange
    if (e != hipSuccess)
        return fail(ctxs[0], TIG_EHIP, "tig_pac_sync_shared", e);
    return TIG_OK;
}

void tig_destroy(tig_ctx *ctx)
{
    if (!ctx)
        return;
    if (ctx->have_marks)
        for (int i = 0; i <= kNumStepKernels; ++i)
            (void)hipEventDestroy(ctx->marks[i]);
    if (ctx->rows_seen_host)
        (void)hipHostFree(ctx->rows_seen_host);
    if (ctx->have_train_side) {
        (void)hipStreamSynchronize(ctx->train_side.stream);
        for (int i = 0; i < kTrainForks; ++i)
            (void)hipEventDestroy(ctx->train_side.fork[i]);
        (void)hipEventDestroy(ctx->train_side.join);
        (void)hipStreamDestroy(ctx->train_side.stream);
    }
    delete ctx;
}

const char *tig_strerror(int status)
{
    switch (status) {
    case TIG_OK: return "success";
    case TIG_EINVAL: return "invalid argument";
    case TIG_ERANGE: return "node or event id out of range";
    case TIG_EUNSORTED: return "event times are not non-decreasing";
    case TIG_ESELFLOOP: return "event with src == dst";
    case TIG_ENOSPACE: return "workspace too small";
    case TIG_EHIP: return "HIP runtime error";
    case TIG_ENOMEM: return "out of host memory";
    case TIG_EORDER: return "batch out of chronological order";
    default: return "unknown status";
    }
}

const char *tig_last_error(const tig_ctx *ctx) { return ctx ? ctx->err : g_init_err; }

int tig_launch_info(const tig_ctx *ctx, int32_t *kernels_per_step, int32_t *gru_lds_bytes,
                    int32_t *embed_lds_bytes)
{
    if (!ctx)
        return TIG_EINVAL;
    if (kernels_per_step)
        *kernels_per_step = ctx->last_launches;
    if (gru_lds_bytes)
        *gru_lds_bytes = ctx->plan.gru_lds;
    if (embed_lds_bytes)
        *embed_lds_bytes = ctx->plan.emb_lds;
    return TIG_OK;
}

}  // extern "C"
