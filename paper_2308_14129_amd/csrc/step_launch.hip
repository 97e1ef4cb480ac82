// Launch plan and launch sequence of one batch step (host side).
#include <hip/hip_runtime.h>

#include "tig_internal.h"

namespace tig {

bool plan_launch(const Dims &d, int lds_limit, LaunchPlan *plan)
{
    if (d.dkvp > 512)
        return false;
    if (gru_lds_bytes(d) > lds_limit)
        return false;
    plan->emb_mt = 0;
    plan->num_cus = 0;
    for (int mt = 3; mt >= 1; --mt)
        if (embed_lds_bytes(d, mt) <= lds_limit) {
            plan->emb_mt = mt;
            break;
        }
    if (!plan->emb_mt)
        return false;
    plan->gru_lds = gru_lds_bytes(d);
    plan->emb_lds = embed_lds_bytes(d, plan->emb_mt);
    return true;
}

hipError_t prepare_kernels(const Dims &d, const LaunchPlan &plan)
{
    hipError_t e = prepare_small();
    if (e == hipSuccess)
        e = prepare_gru(d, plan);
    return e != hipSuccess ? e : prepare_embed(d, plan);
}

hipError_t launch_step(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw,
                       const StepArgs &a, const StepPlan &sp, hipStream_t s, hipEvent_t *marks)
{
    hipError_t e;
    int mark = 0;
    auto stamp = [&]() -> hipError_t { return marks ? hipEventRecord(marks[mark++], s) : hipSuccess; };

    // the counter of a query set this step's embedding launch fills, if no closing launch cleared it
    if (sp.clear_first && (e = launch_fill_zero(sp.clear_first, 4, s)) != hipSuccess)
        return e;
    if ((e = stamp()) != hipSuccess)
        return e;
    if (sp.big_sel && (e = launch_scatter(a, *sp.big_sel, s)) != hipSuccess)
        return e;
    if ((e = stamp()) != hipSuccess)
        return e;
    if (sp.big_sel && (e = launch_select(a, *sp.big_sel, s)) != hipSuccess)
        return e;
    if ((e = stamp()) != hipSuccess)
        return e;
    if (sp.prep_sel || sp.prep_ded) {
        if (sp.prep_ded) {
            // a preparation of its own starts from an empty query set (and, if the table may hold
            // claims of an unknown epoch, from an empty table)
            if (sp.clear_tab)
                e = launch_fill_zero(sp.prep_ded->tab, ((size_t)sp.prep_ded->tab_mask + 1) * 8, s);
            if (e == hipSuccess)
                e = launch_fill_zero(sp.prep_ded->qs.n_u, 4, s);
            if (e != hipSuccess)
                return e;
        }
        const SelectJob no_sel = {};
        const DedupJob no_ded = {};
        if ((e = launch_prepare(a, sp.prep_sel ? *sp.prep_sel : no_sel, sp.prep_ded ? *sp.prep_ded : no_ded, d.K,
                                s)) != hipSuccess)
            return e;
    }
    if ((e = stamp()) != hipSuccess)
        return e;
    if (sp.mods) {
        if ((e = launch_modules(d, plan, pw, a, *sp.mods, s, marks ? marks + mark : nullptr)) != hipSuccess)
            return e;
        mark += marks ? 2 : 0;
        return stamp();
    }
    if (sp.train && sp.train_side && (sp.side_sel || sp.side_ded)) {
        // beside the step, ordered after whatever this step prepared for itself (the jobs share the
        // claim table); the step's stream waits for the side stream ahead of its update
        const TrainSide &ts = *sp.train_side;
        const SelectJob no_sel = {};
        const DedupJob no_ded = {};
        if ((e = hipEventRecord(ts.fork[kTrainForks - 1], s)) != hipSuccess ||
            (e = hipStreamWaitEvent(ts.stream, ts.fork[kTrainForks - 1], 0)) != hipSuccess ||
            (e = launch_prepare(a, sp.side_sel ? *sp.side_sel : no_sel, sp.side_ded ? *sp.side_ded : no_ded, d.K,
                                ts.stream)) != hipSuccess)
            return e;
    }
    if (sp.gru_now && (e = launch_gru(d, plan, pw, a, s)) != hipSuccess)
        return e;
    if ((e = stamp()) != hipSuccess)
        return e;
    if (sp.train) {
        if ((e = launch_train(d, a, sp.train_ws, sp.packed, sp.pw_out, sp.lr, sp.loss_out, s, sp.train_side)) != hipSuccess ||
            (e = stamp()) != hipSuccess)
            return e;
        // inspection outputs, if any are asked for (the training step has cleared its query set's counter)
        if (wants_inspection(a) && (e = launch_closing(d, plan, *sp.pw_out, a, GruAhead{}, s, false)) != hipSuccess)
            return e;
        return stamp();
    }
    if ((e = launch_embed(d, plan, pw, a, s)) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    if ((e = launch_closing(d, plan, pw, a, sp.ahead, s)) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    return hipSuccess;
}

}  // namespace tig
