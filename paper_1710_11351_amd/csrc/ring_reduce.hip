// cmn_ring_reduce: K packed replica buffers [K][L] -> one float32 sum [L].
// A workgroup works on one tile of one ring chunk at a time, so the fold order (which
// replica is read first) is uniform over the workgroup and every output vector is
// produced once by one thread: K streaming reads, one streaming write.  Two kernels:
// one-pass (a workgroup per tile) and, from K = 8 on, two-phase persistent (a workgroup
// folds many tiles into registers, then writes them), which keeps the write stream out
// of the read stream's way on MI355X.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "plan.hpp"

#pragma clang fp contract(off)

namespace cmn {

constexpr int kReduceIters = 1;  // 16-byte vectors per thread per stream

template <int DT, int U>
__global__ __launch_bounds__(kBlock) void k_ring_reduce(const void *__restrict__ packed,
                                                        float *__restrict__ reduced,
                                                        const float *const *__restrict__ scale_ptrs, long long L,
                                                        long long chunk_elems, int tiles_per_chunk, int K,
                                                        int ring_rotate) {
    using G = GradT<DT>;
    using elem = typename G::elem;
    constexpr int VEC = G::VEC;
    constexpr int TILE = kBlock * VEC * kReduceIters;

    const int c = blockIdx.x / tiles_per_chunk;
    const int tile = blockIdx.x - c * tiles_per_chunk;
    const int s = ring_rotate ? c % K : 0;
    const long long chunk_begin = c * chunk_elems;
    const int in_chunk = int(min((long long)TILE, chunk_elems - (long long)tile * TILE));
    const elem *src = static_cast<const elem *>(packed) + chunk_begin + (long long)tile * TILE;
    float *dst = reduced + chunk_begin + (long long)tile * TILE;
    const __amdgpu_buffer_rsrc_t out = make_rsrc(dst, unsigned(in_chunk) * 4u);

    // chunk_elems is a multiple of the alignment, hence of VEC: no ragged vectors
    constexpr int Q = VEC / 4;
    __shared__ f32x4 deal_buf[deal_buffer_vectors<Q>()];
    const int e = threadIdx.x * VEC;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = sum_identity();
    if (e < in_chunk)
        fold_all<DT, U>(
            acc, K, [&](int j) { return src + (long long)ring_rank(s, j, K) * L + e; },
            [&](int j) { return load_uniform(scale_ptrs[ring_rank(s, j, K)] + c); });
    f32x4 o[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) o[q] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    wave_deal<Q>(o, deal_buf);                       // fp32 stores that cover whole cache lines
#pragma unroll
    for (int q = 0; q < Q; ++q)                      // past in_chunk the buffer bounds drop the store
        store_vec<kStoreReducedOnePass>(out, dealt_offset<Q>(q) * 4u, o[q]);
}

template <int DT, int U>
__global__ __launch_bounds__(kBlock, 2) void k_ring_reduce_two_phase(
    const void *__restrict__ packed, float *__restrict__ reduced, const float *const *__restrict__ scale_ptrs,
    long long L, long long chunk_elems, int tiles_per_chunk, int K, int ring_rotate, int tile_begin, int n_tiles) {
    using G = GradT<DT>;
    using elem = typename G::elem;
    constexpr int VEC = G::VEC;
    constexpr int TILE = kBlock * VEC;
    constexpr int M = kStashFloats / VEC;
    constexpr int Q = VEC / 4;
    __shared__ f32x4 deal_buf[deal_buffer_vectors<Q>()];
    const int W = gridDim.x;
    const int e = threadIdx.x * VEC;
    // this launch owns the (chunk, tile) pairs numbered [tile_begin, n_tiles)
    for (int tile0 = tile_begin + blockIdx.x; tile0 < n_tiles; tile0 += W * M) {
        f32x4 stash[M][VEC / 4];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int g = tile0 + m * W;
            if (g < n_tiles) {
                const int c = g / tiles_per_chunk, tile = g - c * tiles_per_chunk;
                const int s = ring_rotate ? c % K : 0;
                const int in_chunk = int(min((long long)TILE, chunk_elems - (long long)tile * TILE));
                const elem *src = static_cast<const elem *>(packed) + c * chunk_elems + (long long)tile * TILE;
                float acc[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = sum_identity();
                if (e < in_chunk)
                    fold_all<DT, U, true>(
                        acc, K, [&](int j) { return src + (long long)ring_rank(s, j, K) * L + e; },
                        [&](int j) { return load_uniform(scale_ptrs[ring_rank(s, j, K)] + c); });
#pragma unroll
                for (int q = 0; q < Q; ++q) stash[m][q] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
                wave_deal<Q>(stash[m], deal_buf);
            }
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int g = tile0 + m * W;
            if (g < n_tiles) {
                const int c = g / tiles_per_chunk, tile = g - c * tiles_per_chunk;
                const int in_chunk = int(min((long long)TILE, chunk_elems - (long long)tile * TILE));
                float *dst = reduced + c * chunk_elems + (long long)tile * TILE;
                const __amdgpu_buffer_rsrc_t out = make_rsrc(dst, unsigned(in_chunk) * 4u);
#pragma unroll
                for (int q = 0; q < Q; ++q)              // past in_chunk the buffer bounds drop the store
                    store_vec<kStoreReducedPhase2>(out, dealt_offset<Q>(q) * 4u, stash[m][q]);
            }
        }
    }
}

}  // namespace cmn

using namespace cmn;

extern "C" int cmn_ring_reduce(const cmn_plan *plan, const void *packed, float *reduced, void *stream) {
    if (!plan) return CMN_ENULL;
    if (plan->L == 0) return CMN_OK;
    if (!packed || !reduced) return CMN_ENULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256 || reinterpret_cast<uintptr_t>(reduced) % 256) return CMN_EALIGN;
    const int tile = kBlock * vec_elems(plan->dtype) * kReduceIters;
    const long long tpc = (plan->chunk_elems + tile - 1) / tile;
    if (tpc * plan->C > 0x7fffffffLL) return CMN_ESIZE;
    const dim3 grid(unsigned(tpc * plan->C));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t err = hipSuccess;
#define CMN_LAUNCH_REDUCE(DT)                                                                              \
    err = launch_kernel(k_ring_reduce<DT, 16>, grid, dim3(kBlock), 0, s, packed, reduced, scales, (long long)plan->L, \
                        (long long)plan->chunk_elems, int(tpc), plan->K, plan->ring_rotate)
    const float *const *scales = nullptr;
    if (plan->dtype == CMN_I8S) {
        if (!plan->bound || !plan->have_scales) return CMN_EUNBOUND;
        scales = ws_ptr<const float *const>(plan, plan->ws.scale_ptrs);
    }
    // (a launch of the persistent kernel only pays off over a few thousand tiles)
    if (prefer_two_phase_reduce(plan) && kReduceIters == 1 &&
        (tpc * plan->C >= kMinTwoPhaseTiles || plan->step_mode == STEP_TWO_PHASE)) {
        // one launch per round of the persistent grid, tiles spread evenly (a kernel boundary
        // realigns the phases of the workgroups)
        const long long n_tiles = tpc * plan->C, resident = two_phase_grid(plan);
        const long long per_launch = two_phase_launches(plan, n_tiles).second;
#define CMN_LAUNCH_REDUCE2(DT)                                                                                  \
    for (long long b0 = 0; b0 < n_tiles && err == hipSuccess; b0 += per_launch) {                               \
        const long long e0 = b0 + per_launch < n_tiles ? b0 + per_launch : n_tiles, cnt = e0 - b0;              \
        err = launch_kernel(k_ring_reduce_two_phase<DT, 8>, dim3(unsigned(cnt < resident ? cnt : resident)),    \
                            dim3(kBlock), 0, s, packed, reduced, scales, (long long)plan->L,                    \
                            (long long)plan->chunk_elems, int(tpc), plan->K, plan->ring_rotate, int(b0), int(e0)); \
    }
        if (plan->dtype == CMN_F32) CMN_LAUNCH_REDUCE2(CMN_F32)
        else if (plan->dtype == CMN_F16) CMN_LAUNCH_REDUCE2(CMN_F16)
        else CMN_LAUNCH_REDUCE2(CMN_BF16)
#undef CMN_LAUNCH_REDUCE2
    } else if (plan->dtype == CMN_F32) CMN_LAUNCH_REDUCE(CMN_F32);
    else if (plan->dtype == CMN_F16) CMN_LAUNCH_REDUCE(CMN_F16);
    else if (plan->dtype == CMN_BF16) CMN_LAUNCH_REDUCE(CMN_BF16);
    else CMN_LAUNCH_REDUCE(CMN_I8S);
#undef CMN_LAUNCH_REDUCE
    return err == hipSuccess ? CMN_OK : CMN_EHIP;
}
