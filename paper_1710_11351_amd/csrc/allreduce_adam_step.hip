// Entry points of the fused aggregation + update step with Adam in place of MomentumSGD,
// over the whole tensor list or a range of it: the same kernels as allreduce_step.hip,
// instantiated for the second optimizer.
#include <cmath>

#include "step_kernel.hpp"

using namespace cmn;

extern "C" int cmn_allreduce_adam_step_range(const cmn_plan *plan, int tensor_begin, int tensor_end, float alpha,
                                             float beta1, float beta2, float eps, float wd, int t, int mean_dest,
                                             void *stream) {
    if (t < 1) return plan ? CMN_EINVAL : CMN_ENULL;
    const OptArgs o{adam_step_size(alpha, beta1, beta2, t), 1.0f - beta1, 1.0f - beta2, eps, wd};
    return launch_fused<OPT_ADAM>(plan, tensor_begin, tensor_end, mean_dest, o, stream);
}

extern "C" int cmn_allreduce_adam_step(const cmn_plan *plan, float alpha, float beta1, float beta2, float eps,
                                       float wd, int t, int mean_dest, void *stream) {
    if (!plan) return CMN_ENULL;
    return cmn_allreduce_adam_step_range(plan, 0, plan->T, alpha, beta1, beta2, eps, wd, t, mean_dest, stream);
}
