// cmn_momentum_sgd: the optimizer step on its own.  Reads the bound mean
// gradients, updates p and v in place.  Driven by the same tile table as the
// fused step (a tile = a run of elements of one tensor); the ring start rank
// stored in a tile is not used here.  HBM traffic per element: 3 reads, 2 writes.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "plan.hpp"

#pragma clang fp contract(off)

namespace cmn {

__global__ __launch_bounds__(kBlock) void k_momentum_sgd(
    const cmn_tile *__restrict__ tiles, float *const *__restrict__ mean_ptrs,
    float *const *__restrict__ param_ptrs, float *const *__restrict__ vel_ptrs, float lr, float mu, float wd) {
    const cmn_tile tl = tiles[blockIdx.x];
    const int t = tl.tensor, len = tl.len;
    const float *g = mean_ptrs[t] + tl.e0;
    float *p = param_ptrs[t] + tl.e0;
    float *v = vel_ptrs[t] + tl.e0;

    int head = tl.head_sgd;
    if (head < 0 || head > len) head = len;
    const int nvec = (len - head) / 4;
    const int tail0 = head + nvec * 4;
    const __amdgpu_buffer_rsrc_t p_out = make_rsrc(p, unsigned(len) * 4u);
    const __amdgpu_buffer_rsrc_t v_out = make_rsrc(v, unsigned(len) * 4u);

    for (int vi = threadIdx.x; vi < nvec; vi += kBlock) {
        const unsigned e = unsigned(head + vi * 4);
        const f32x4 gv = load_vec<f32x4>(g + e);
        f32x4 pv = load_vec<f32x4>(p + e);
        f32x4 vv = load_vec<f32x4>(v + e);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float pi = pv[i], vi2 = vv[i];
            sgd_update(gv[i], pi, vi2, lr, mu, wd);
            pv[i] = pi; vv[i] = vi2;
        }
        store_through(v_out, e * 4u, vv);
        store_through(p_out, e * 4u, pv);
    }
    const int n_single = head + (len - tail0);
    for (int i = threadIdx.x; i < n_single; i += kBlock) {
        const int e = i < head ? i : tail0 + (i - head);
        float pi = p[e], vi2 = v[e];
        sgd_update(g[e], pi, vi2, lr, mu, wd);
        v[e] = vi2;
        p[e] = pi;
    }
}

}  // namespace cmn

using namespace cmn;

extern "C" int cmn_momentum_sgd(const cmn_plan *plan, float lr, float mu, float wd, void *stream) {
    if (int rc = check_launch(plan)) return rc;
    if (!plan->have_opt || !plan->have_mean) return CMN_EUNBOUND;
    if (plan->n_tiles == 0) return CMN_OK;
    hipLaunchKernelGGL(k_momentum_sgd, dim3(unsigned(plan->n_tiles)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), ws_ptr<const cmn_tile>(plan, plan->ws.tiles),
                       ws_ptr<float *const>(plan, plan->ws.mean_ptrs), ws_ptr<float *const>(plan, plan->ws.param_ptrs),
                       ws_ptr<float *const>(plan, plan->ws.vel_ptrs), lr, mu, wd);
    return hipGetLastError() == hipSuccess ? CMN_OK : CMN_EHIP;
}
