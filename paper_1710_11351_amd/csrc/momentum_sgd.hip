// cmn_momentum_sgd and cmn_adam: the optimizer step on its own.  They read the bound
// mean gradients and update the parameters and optimizer state in place, through the
// same tile table and kernel template as the fused step (the ring start rank stored in a
// tile is simply not used).  HBM traffic per element: 3 reads + 2 writes (MomentumSGD),
// 4 reads + 3 writes (Adam).
#include <cmath>

#include "step_kernel.hpp"

using namespace cmn;

extern "C" int cmn_momentum_sgd(const cmn_plan *plan, float lr, float mu, float wd, void *stream) {
    const OptArgs o{lr, mu, 0.0f, 0.0f, wd};
    return launch_optimizer<OPT_SGD>(plan, o, stream);
}

extern "C" int cmn_adam(const cmn_plan *plan, float alpha, float beta1, float beta2, float eps, float wd, int t,
                        void *stream) {
    if (t < 1) return plan ? CMN_EINVAL : CMN_ENULL;
    const OptArgs o{adam_step_size(alpha, beta1, beta2, t), 1.0f - beta1, 1.0f - beta2, eps, wd};
    return launch_optimizer<OPT_ADAM>(plan, o, stream);
}
