// Launch plan and launch sequence of one batch step (host side).
#include <hip/hip_runtime.h>

#include "tig_internal.h"

namespace tig {

bool plan_launch(const Dims &d, int lds_limit, LaunchPlan *plan)
{
    if (d.dkvp > 512)
        return false;
    plan->gru_mt = 0;
    for (int mt = 1; mt >= 1; --mt)
        if (gru_lds_bytes(d, mt) <= lds_limit) {
            plan->gru_mt = mt;
            break;
        }
    plan->emb_mt = 0;
    plan->num_cus = 0;
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
    hipError_t e = prepare_small();
    if (e == hipSuccess)
        e = prepare_gru(d, plan);
    return e != hipSuccess ? e : prepare_embed(d, plan);
}

hipError_t launch_step(const Dims &d, const LaunchPlan &plan, const PackedWeights &pw,
                       const StepArgs &a, const StepArgs *sel, hipStream_t s, hipEvent_t *marks)
{
    hipError_t e;
    int mark = 0;
    auto stamp = [&]() -> hipError_t { return marks ? hipEventRecord(marks[mark++], s) : hipSuccess; };

    if ((e = stamp()) != hipSuccess)
        return e;
    bool needs_select = false;
    if (sel && (e = launch_scatter(*sel, s, &needs_select)) != hipSuccess)
        return e;
    if ((e = stamp()) != hipSuccess)
        return e;
    if (needs_select && (e = launch_select(*sel, s)) != hipSuccess)
        return e;
    if ((e = stamp()) != hipSuccess)
        return e;
    if ((e = launch_gru(d, plan, pw, a, s)) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    if ((e = launch_commit(a, d.M, s)) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    if ((e = launch_embed(d, plan, pw, a, s)) != hipSuccess || (e = stamp()) != hipSuccess)
        return e;
    return hipSuccess;
}

}  // namespace tig
