// Entry points of the fused aggregation + update step (S1..S5 in one pass over HBM)
// with MomentumSGD, over the whole tensor list or a range of it.  (The Adam entry points
// live in allreduce_adam_step.hip so that the two sets of kernel variants build in parallel.)
// HBM traffic per element: K gradient reads + parameter and optimizer state read and
// written (+ the averaged gradient, once or K times, if asked for).
#include <cmath>

#include "step_kernel.hpp"

using namespace cmn;

extern "C" int cmn_allreduce_step_range(const cmn_plan *plan, int tensor_begin, int tensor_end, float lr, float mu,
                                        float wd, int mean_dest, void *stream) {
    const OptArgs o{lr, mu, 0.0f, 0.0f, wd};
    return launch_fused<OPT_SGD>(plan, tensor_begin, tensor_end, mean_dest, o, stream);
}

extern "C" int cmn_allreduce_step(const cmn_plan *plan, float lr, float mu, float wd, int mean_dest, void *stream) {
    if (!plan) return CMN_ENULL;
    return cmn_allreduce_step_range(plan, 0, plan->T, lr, mu, wd, mean_dest, stream);
}
