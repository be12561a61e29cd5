// cmn_allreduce_step: pack, ring-order sum, scale, unpack and MomentumSGD in one
// pass over HBM.  No packed buffer exists: a tile names a run of elements of one
// tensor inside one ring chunk, every thread owns one 16-byte vector of it, reads
// the K replicas' vectors in the chunk's fold order, and updates p and v in place.
// HBM traffic per element: K gradient reads + p, v read + p, v written.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "plan.hpp"

#pragma clang fp contract(off)

namespace cmn {

// U = gradient vectors requested back to back before the first one is consumed.
template <int DT, int U, bool WRITE_MEAN>
__global__ __launch_bounds__(kBlock) void k_allreduce_step(
    const cmn_tile *__restrict__ tiles, const void *const *__restrict__ grad_cols,
    float *const *__restrict__ param_ptrs, float *const *__restrict__ vel_ptrs,
    float *const *__restrict__ mean_ptrs, int K, float inv_k, float lr, float mu, float wd) {
    using G = GradT<DT>;
    using elem = typename G::elem;
    using raw = typename G::raw;
    constexpr int VEC = G::VEC;

    const cmn_tile tl = tiles[blockIdx.x];
    const int t = tl.tensor, s = tl.start_rank, len = tl.len;
    const void *const *gcol = grad_cols + size_t(t) * size_t(K);
    float *p = param_ptrs[t] + tl.e0;
    float *v = vel_ptrs[t] + tl.e0;
    float *m = WRITE_MEAN ? mean_ptrs[t] + tl.e0 : nullptr;

    int head = WRITE_MEAN ? tl.head_step_mean : tl.head_step;
    if (head < 0 || head > len) head = len;
    const int nvec = (len - head) / VEC;
    const int tail0 = head + nvec * VEC;
    const __amdgpu_buffer_rsrc_t p_out = make_rsrc(p, unsigned(len) * 4u);
    const __amdgpu_buffer_rsrc_t v_out = make_rsrc(v, unsigned(len) * 4u);
    const __amdgpu_buffer_rsrc_t m_out = make_rsrc(m, WRITE_MEAN ? unsigned(len) * 4u : 0u);

    for (int vi = threadIdx.x; vi < nvec; vi += kBlock) {
        const unsigned e = unsigned(head + vi * VEC);
        f32x4 pv[VEC / 4], vv[VEC / 4];
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            pv[q] = load_vec<f32x4>(p + e + 4 * q);
            vv[q] = load_vec<f32x4>(v + e + 4 * q);
        }
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = sum_identity();

        int j = 0;
        for (; j + U <= K; j += U) {
            raw g[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                g[u] = load_stream<raw>(static_cast<const elem *>(gcol[ring_rank(s, j + u, K)]) + tl.e0 + e);
#pragma unroll
            for (int u = 0; u < U; ++u) G::accumulate(acc, g[u]);
        }
        for (; j < K; ++j) {
            const raw g = load_stream<raw>(static_cast<const elem *>(gcol[ring_rank(s, j, K)]) + tl.e0 + e);
            G::accumulate(acc, g);
        }

#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            f32x4 gb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                gb[i] = acc[4 * q + i] * inv_k;
                float pi = pv[q][i], vi2 = vv[q][i];
                sgd_update(gb[i], pi, vi2, lr, mu, wd);
                pv[q][i] = pi; vv[q][i] = vi2;
            }
            if (WRITE_MEAN) store_through(m_out, (e + 4 * q) * 4u, gb);
            store_through(v_out, (e + 4 * q) * 4u, vv[q]);
            store_through(p_out, (e + 4 * q) * 4u, pv[q]);
        }
    }

    // ragged head and tail of the tile (or the whole tile when its streams share no alignment)
    const int n_single = head + (len - tail0);
    for (int i = threadIdx.x; i < n_single; i += kBlock) {
        const int e = i < head ? i : tail0 + (i - head);
        float acc = sum_identity();
        for (int j = 0; j < K; ++j)
            acc = acc + G::decode(static_cast<const elem *>(gcol[ring_rank(s, j, K)])[tl.e0 + e]);
        const float gb = acc * inv_k;
        float pi = p[e], vi2 = v[e];
        sgd_update(gb, pi, vi2, lr, mu, wd);
        if (WRITE_MEAN) m[e] = gb;
        v[e] = vi2;
        p[e] = pi;
    }
}

template <int DT, bool WM>
static void launch_step(const cmn_plan *p, float lr, float mu, float wd, hipStream_t s) {
    constexpr int U = 16;
    hipLaunchKernelGGL((k_allreduce_step<DT, U, WM>), dim3(unsigned(p->n_tiles)), dim3(kBlock), 0, s,
                       ws_ptr<const cmn_tile>(p, p->ws.tiles), ws_ptr<const void *const>(p, p->ws.grad_cols),
                       ws_ptr<float *const>(p, p->ws.param_ptrs), ws_ptr<float *const>(p, p->ws.vel_ptrs),
                       ws_ptr<float *const>(p, p->ws.mean_ptrs), p->K, 1.0f / float(p->K), lr, mu, wd);
}

}  // namespace cmn

using namespace cmn;

extern "C" int cmn_allreduce_step(const cmn_plan *plan, float lr, float mu, float wd, int write_mean_grad,
                                  void *stream) {
    if (int rc = check_launch(plan)) return rc;
    if (!plan->have_grads || !plan->have_opt || (write_mean_grad && !plan->have_mean)) return CMN_EUNBOUND;
    if (plan->n_tiles == 0) return CMN_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->dtype == CMN_F32) {
        if (write_mean_grad) launch_step<CMN_F32, true>(plan, lr, mu, wd, s);
        else launch_step<CMN_F32, false>(plan, lr, mu, wd, s);
    } else {
        if (write_mean_grad) launch_step<CMN_F16, true>(plan, lr, mu, wd, s);
        else launch_step<CMN_F16, false>(plan, lr, mu, wd, s);
    }
    return hipGetLastError() == hipSuccess ? CMN_OK : CMN_EHIP;
}
