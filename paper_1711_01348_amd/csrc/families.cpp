// Pattern recognition: which kernel family evaluates the forward pass and each gradient.
// Every plan can run on the plan-driven generic kernels; a specialised family is chosen only
// when body, index matrices and dtype match its template exactly.
#include "plan.hpp"

namespace tad {

void select_families(tad_plan &plan) {
    plan.fwd_family = TAD_FAMILY_GENERIC;
    for (auto &ap : plan.ap) ap.family = TAD_FAMILY_GENERIC;
    plan.ws_bytes = 0;
    if (plan.flags & TAD_PLAN_GENERIC_ONLY) return;
}

}  // namespace tad
