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
    float *mem;
    double *lu;
    unsigned long long *key;
    void *packed;
    // scratch (per step)
    int32_t *nbr_node, *nbr_eid, *nbr_cnt;
    double *nbr_ts;
    float *staging;
    WinDesc *win[2];   // winner lists: this step's, and the one selected ahead for the next
    int32_t *n_win[2];
    int cur;           // list used by the last step
    bool ahead_valid;  // win[cur ^ 1] holds the winners of batch (ahead_first, ahead_count)
    int64_t ahead_first;
    int32_t ahead_count;
    int num_cus;
    int64_t cursor;    // end of the last batch stepped since the last reset / import
    int last_launches; // kernels enqueued by the last tig_step
    // deferred order: win[cur] holds the winners of batch (pend_first, pend_count), not yet applied
    bool pend_valid;
    int64_t pend_first;
    int32_t pend_count;
    int32_t *pos;
    void *static_scratch;  // this device's copy of g_static_scratch
    hipEvent_t marks[kNumStepKernels + 1];
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
    unsigned long long *key;
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
    L.key = c.take<unsigned long long>((size_t)N);
    L.packed = c.take<char>(packed_weights_bytes(d));
    L.bytes = c.off;
    return L;
}

struct StepScratch {
    int32_t *nbr_node, *nbr_eid, *nbr_cnt;
    double *nbr_ts;
    float *staging;
    WinDesc *win[2];
    int32_t *n_win[2];
    size_t bytes;
};

StepScratch step_scratch(const Dims &d, void *base)
{
    Carver c(base);
    StepScratch S;
    const size_t Q = (size_t)3 * d.max_batch;
    S.nbr_node = c.take<int32_t>(Q * d.K);
    S.nbr_eid = c.take<int32_t>(Q * d.K);
    S.nbr_ts = c.take<double>(Q * d.K);
    S.nbr_cnt = c.take<int32_t>(Q);
    S.staging = c.take<float>((size_t)2 * d.max_batch * d.M);
    for (int i = 0; i < 2; ++i) {
        S.win[i] = c.take<WinDesc>((size_t)2 * d.max_batch + 32);  // GRU tiles read whole 32-row slices
        S.n_win[i] = c.take<int32_t>(1);
    }
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
    if (!weights || weights->struct_size != sizeof(tig_weights) || !persistent || !scratch)
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
    for (int i = 0; i < nwf; ++i)
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
    ctx->key = L.key;
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
    {
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
    INIT_TRY(launch_fill_zero(L.key, sizeof(unsigned long long) * (size_t)N, s), "zero keys");
    INIT_TRY(hipStreamSynchronize(s), "sync");
#undef INIT_TRY

    const StepScratch S = step_scratch(d, scratch);
    ctx->nbr_node = S.nbr_node;
    ctx->nbr_eid = S.nbr_eid;
    ctx->nbr_ts = S.nbr_ts;
    ctx->nbr_cnt = S.nbr_cnt;
    ctx->staging = S.staging;
    for (int i = 0; i < 2; ++i) {
        ctx->win[i] = S.win[i];
        ctx->n_win[i] = S.n_win[i];
    }
    ctx->cur = 0;
    ctx->ahead_valid = false;
    {
        hipError_t e = launch_fill_zero(S.n_win[0], 256, s);
        if (e == hipSuccess)
            e = launch_fill_zero(S.n_win[1], 256, s);
        const hipError_t e2 = e == hipSuccess ? hipStreamSynchronize(s) : e;
        if (e2 != hipSuccess) {
            snprintf(g_init_err, sizeof(g_init_err), "clear counters: %s", hipGetErrorString(e2));
            delete ctx;
            return TIG_EHIP;
        }
    }
    *out = ctx;
    return TIG_OK;
}

// `use_static`: every per-step intermediate lives in this device's static scratch array instead of
// the context's scratch workspace, the winners are selected up front by the call itself, and
// nothing is kept there for a later call.
static int step_impl(tig_ctx *ctx, const tig_batch *batch, const tig_out *out, hipEvent_t *marks,
                     bool use_static = false)
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
    StepScratch st;
    if (use_static) {
        if (ctx->d.deferred)
            return fail(ctx, TIG_EINVAL, "tig_step_static: the context runs the deferred message order");
        if (step_scratch(ctx->d, nullptr).bytes > (size_t)TIG_STATIC_SCRATCH_BYTES)
            return fail(ctx, TIG_ENOSPACE, "tig_step_static: the per-step intermediates of this configuration "
                                           "exceed TIG_STATIC_SCRATCH_BYTES");
        st = step_scratch(ctx->d, ctx->static_scratch);
    }

    StepArgs a;
    a.src = ctx->src;
    a.dst = ctx->dst;
    a.ts = ctx->ts;
    a.edge_feat = ctx->edge_feat;
    a.indptr = ctx->indptr;
    a.csr = ctx->csr;
    a.num_nodes = ctx->num_nodes;
    a.mem = ctx->mem;
    a.lu = ctx->lu;
    a.key = ctx->key;
    a.first_eid = batch->first_eid;
    a.count = batch->count;
    a.roles = batch->neg_dst ? 3 : 2;
    a.neg = batch->neg_dst;
    a.nbr_node = out->nbr_node ? out->nbr_node : (use_static ? st.nbr_node : ctx->nbr_node);
    a.nbr_eid = out->nbr_eid ? out->nbr_eid : (use_static ? st.nbr_eid : ctx->nbr_eid);
    a.nbr_ts = out->nbr_ts ? out->nbr_ts : (use_static ? st.nbr_ts : ctx->nbr_ts);
    a.nbr_cnt = out->nbr_cnt ? out->nbr_cnt : (use_static ? st.nbr_cnt : ctx->nbr_cnt);
    a.staging = use_static ? st.staging : ctx->staging;
    a.pos = ctx->pos;
    a.is_winner = out->is_winner;
    a.emb = out->emb;
    a.score_pos = out->score_pos;
    a.score_neg = out->score_neg;

    a.next_is_winner = nullptr;
    const bool one_launch = 2 * batch->count <= 8192;  // selection in one workgroup
    StepArgs sel;
    const StepArgs *selp = nullptr;
    int launches = 0;
    int new_cur = ctx->cur;
    if (use_static) {
        // everything in the static array; this batch's winners are selected first, none ahead
        a.win = st.win[0];
        a.n_win = st.n_win[0];
        a.msg_first_eid = batch->first_eid;
        a.msg_count = batch->count;
        a.next_first_eid = batch->first_eid + batch->count;
        a.next_count = 0;
        a.next_win = st.win[1];
        a.next_n_win = st.n_win[1];
        selp = &a;
        launches += (one_launch ? 1 : 2) + 3;
    } else if (ctx->d.deferred) {
        // Deferred order: the GRU and the memory overwrite apply the winners kept by the previous
        // step; this step's winners go to the other list, selected by one extra workgroup of the
        // embedding launch when it can carry it, else by a selection of its own up front (it
        // reads the event stream only).
        a.win = ctx->win[ctx->cur];
        a.n_win = ctx->n_win[ctx->cur];
        a.msg_first_eid = ctx->pend_first;
        a.msg_count = ctx->pend_valid ? ctx->pend_count : 0;
        a.is_winner = nullptr;
        a.next_first_eid = batch->first_eid;
        a.next_count = 0;
        a.next_win = ctx->win[ctx->cur ^ 1];
        a.next_n_win = ctx->n_win[ctx->cur ^ 1];
        a.next_is_winner = out->is_winner;
        if (!marks && embed_can_select_ahead(ctx->d, ctx->plan, a.roles, batch->count, batch->count)) {
            a.next_count = batch->count;
        } else {
            sel = a;
            sel.win = a.next_win;
            sel.n_win = a.next_n_win;
            sel.is_winner = out->is_winner;
            selp = &sel;
            launches += one_launch ? 1 : 2;
        }
        launches += a.msg_count > 0 ? 3 : 2;
    } else {
        // Winner list of this batch: selected ahead by the previous step's embedding launch if that
        // step guessed this batch (the selection depends on the event stream only, so state changes
        // in between do not matter).  A caller that asks for the per-entry flags gets a fresh run.
        const bool ready = ctx->ahead_valid && ctx->ahead_first == batch->first_eid &&
                           ctx->ahead_count == batch->count && !out->is_winner && !marks;
        new_cur = ready ? ctx->cur ^ 1 : ctx->cur;  // takes effect once the launches have succeeded
        a.win = ctx->win[new_cur];
        a.n_win = ctx->n_win[new_cur];
        a.msg_first_eid = batch->first_eid;
        a.msg_count = batch->count;
        // Chronological training and evaluation pass consecutive batches of one size: guess that the
        // next call continues where this one ends, and let the embedding launch select its winners.
        // (The profiled step keeps every kernel to its own work.)
        a.next_first_eid = batch->first_eid + batch->count;
        a.next_count = 0;
        a.next_win = ctx->win[new_cur ^ 1];
        a.next_n_win = ctx->n_win[new_cur ^ 1];
        if (!marks && a.next_first_eid < ctx->num_events) {
            const int64_t left = ctx->num_events - a.next_first_eid;
            const int32_t guess = left < batch->count ? (int32_t)left : batch->count;
            if (embed_can_select_ahead(ctx->d, ctx->plan, a.roles, batch->count, guess))
                a.next_count = guess;
        }
        if (!ready) {
            selp = &a;
            launches += one_launch ? 1 : 2;
        }
        launches += 3;
    }
    const hipError_t e = launch_step(ctx->d, ctx->plan, ctx->pw, a, selp, ctx->stream, marks);
    if (e != hipSuccess) {
        // kernels of this step may already be enqueued: the list bookkeeping stays as it was, the
        // model state is undefined until tig_reset / tig_state_import
        if (!use_static)
            ctx->ahead_valid = false;
        return fail(ctx, TIG_EHIP, "tig_step launch", e);
    }
    if (!use_static) {
        ctx->ahead_valid = false;
        ctx->cur = new_cur;
    }
    ctx->cursor = batch->first_eid + batch->count;
    if (!marks)
        ctx->last_launches = launches;
    if (use_static) {
        // the context's own lists are untouched: a list selected ahead stays usable
    } else if (ctx->d.deferred) {
        ctx->cur ^= 1;  // the list just selected is the one the next step applies
        ctx->pend_valid = true;
        ctx->pend_first = batch->first_eid;
        ctx->pend_count = batch->count;
    } else if (a.next_count > 0) {
        ctx->ahead_valid = true;
        ctx->ahead_first = a.next_first_eid;
        ctx->ahead_count = a.next_count;
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
    if (e != hipSuccess)
        return fail(ctx, TIG_EHIP, "tig_step_profiled timing", e);
    return TIG_OK;
}

// Deferred order: forgets the winners kept for the next step.  A selection of more than 4096 events
// left its keys in the per-node array (the overwrite that would have cleared them never runs).
static hipError_t drop_pending(tig_ctx *ctx)
{
    hipError_t e = hipSuccess;
    if (ctx->pend_valid && 2 * ctx->pend_count > 8192)
        e = launch_fill_zero(ctx->key, sizeof(unsigned long long) * (size_t)ctx->num_nodes, ctx->stream);
    ctx->pend_valid = false;
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

void tig_destroy(tig_ctx *ctx)
{
    if (!ctx)
        return;
    if (ctx->have_marks)
        for (int i = 0; i <= kNumStepKernels; ++i)
            (void)hipEventDestroy(ctx->marks[i]);
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
