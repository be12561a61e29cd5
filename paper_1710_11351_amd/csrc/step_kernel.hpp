// The tensor-space kernels behind cmn_allreduce_step, cmn_allreduce_adam_step, their
// _range forms, cmn_momentum_sgd and cmn_adam.  A tile names a run of elements of one
// tensor inside one ring chunk; every thread owns one 16-byte gradient vector of it.
//   SRC_FOLD: read the K replicas' vectors in the chunk's fold order, sum, scale by 1/K
//   SRC_MEAN: read the averaged gradient from the bound mean-gradient tensor
// then apply the optimizer to p and its state in place.  No packed buffer exists.
// TileView holds the per-tile work (fold, apply, ragged elements); k_step does it in one
// pass with a workgroup per tile, k_step_two_phase with a persistent grid that reads
// first and writes afterwards.  Both give identical bits.
#pragma once

#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "plan.hpp"

#pragma clang fp contract(off)

namespace cmn {

enum { SRC_FOLD = 0, SRC_MEAN = 1 };

template <int SRC, int MEAN, int OPT>
__device__ __forceinline__ constexpr int head_index() {
    return SRC == SRC_MEAN ? (OPT == OPT_ADAM ? CMN_HEAD_ADAM_OPT : CMN_HEAD_SGD)
           : OPT == OPT_ADAM ? (MEAN == CMN_MEAN_TO_MEAN_GRADS ? CMN_HEAD_ADAM_MEAN : CMN_HEAD_ADAM)
                             : (MEAN == CMN_MEAN_TO_MEAN_GRADS ? CMN_HEAD_STEP_MEAN : CMN_HEAD_STEP);
}

// A table entry as the sixteen 32-bit words it occupies: read as words it travels through one
// scalar load (a byte-sized field on its own would need a vector load and a broadcast).
struct TileWords {
    uint32_t w[16];
    template <typename T> __device__ __forceinline__ T *ptr(int i) const {
        return reinterpret_cast<T *>((unsigned long long)w[2 * i + 1] << 32 | w[2 * i]);
    }
    __device__ __forceinline__ float *p() const { return ptr<float>(0); }
    __device__ __forceinline__ float *s1() const { return ptr<float>(1); }
    __device__ __forceinline__ float *s2() const { return ptr<float>(2); }
    __device__ __forceinline__ float *m() const { return ptr<float>(3); }
    __device__ __forceinline__ long long e0() const { return (long long)(((unsigned long long)w[9] << 32) | w[8]); }
    __device__ __forceinline__ int len() const { return int(w[10]); }
    __device__ __forceinline__ int tensor() const { return int(w[11]); }
    __device__ __forceinline__ int start_rank() const { return int(w[12]); }
    __device__ __forceinline__ int chunk() const { return int(w[13]); }
    __device__ __forceinline__ int head(int i) const { return int(int8_t((w[14 + i / 4] >> (8 * (i % 4))) & 0xffu)); }
};
static_assert(sizeof(DeviceTile) == sizeof(TileWords) && offsetof(DeviceTile, p) == 0 && offsetof(DeviceTile, s1) == 8 &&
                  offsetof(DeviceTile, s2) == 16 && offsetof(DeviceTile, m) == 24 && offsetof(DeviceTile, e0) == 32 &&
                  offsetof(DeviceTile, len) == 40 && offsetof(DeviceTile, tensor) == 44 &&
                  offsetof(DeviceTile, start_rank) == 48 && offsetof(DeviceTile, chunk) == 52 &&
                  offsetof(DeviceTile, head) == 56,
              "TileWords mirrors DeviceTile");
__device__ __forceinline__ TileWords load_tile(const DeviceTile *tiles, int i) {
    return *reinterpret_cast<const TileWords *>(tiles + i);
}

// Everything a kernel needs to know about one tile, derived from its table entry.
template <int DT, int SRC, int MEAN, int OPT>
struct TileView {
    using G = GradT<DT>;
    using elem = typename G::elem;
    static constexpr int VEC = SRC == SRC_MEAN ? 4 : G::VEC;
    static constexpr int Q = VEC / 4;   // float4s per thread and tile
    static constexpr bool ADAM = OPT == OPT_ADAM;
    static constexpr bool USE_MEAN_TENSOR = SRC == SRC_MEAN || MEAN == CMN_MEAN_TO_MEAN_GRADS;

    long long e0;
    int len, s, chunk, head, nvec, tail0;
    const void *const *gcol;
    float *p, *s1, *s2, *m;

    __device__ __forceinline__ TileView(const TileWords &tl, const void *const *grad_cols, int K) {
        e0 = tl.e0(); len = tl.len(); s = tl.start_rank(); chunk = tl.chunk();
        gcol = grad_cols + size_t(tl.tensor()) * size_t(K);
        p = tl.p();
        s1 = tl.s1();
        s2 = ADAM ? tl.s2() : nullptr;
        m = USE_MEAN_TENSOR ? tl.m() : nullptr;
        head = tl.head(head_index<SRC, MEAN, OPT>());
        if (head < 0 || head > len) head = len;
        nvec = (len - head) / VEC;
        tail0 = head + nvec * VEC;
    }

    // Averaged gradient of the thread's run of VEC elements (vector number vi of the tile): fold of
    // the K replicas, times 1/K, then dealt over the wavefront so that the fp32 side coalesces.
    // Every thread of the workgroup calls this; a thread without a vector contributes zeros.
    template <int U, bool ONE_TAIL = false>
    __device__ __forceinline__ void averaged(f32x4 (&out)[Q], int vi, const float *const *scale_ptrs, int K,
                                             float inv_k, f32x4 *deal_buf) const {
        float gb[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) gb[i] = 0.0f;
        if (vi < nvec) {
            const unsigned e = unsigned(head + vi * VEC);
#pragma unroll
            for (int i = 0; i < VEC; ++i) gb[i] = sum_identity();
            fold_all<DT, U, ONE_TAIL>(
                gb, K, [&](int j) { return static_cast<const elem *>(gcol[ring_rank(s, j, K)]) + e0 + e; },
                [&](int j) { return load_uniform(scale_ptrs[ring_rank(s, j, K)] + chunk); });
#pragma unroll
            for (int i = 0; i < VEC; ++i) gb[i] = gb[i] * inv_k;
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) out[q] = f32x4{gb[4 * q], gb[4 * q + 1], gb[4 * q + 2], gb[4 * q + 3]};
        wave_deal<Q>(out, deal_buf);
    }

    // The same from the bound mean-gradient tensor (optimizer-only kernels, Q = 1).
    template <bool STREAM>
    __device__ __forceinline__ void averaged_from_mean(f32x4 (&out)[Q], int vi) const {
        static_assert(SRC != SRC_MEAN || Q == 1, "the mean gradient is fp32");
        out[0] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (vi < nvec) out[0] = STREAM ? load_stream<f32x4>(m + head + vi * 4) : load_vec<f32x4>(m + head + vi * 4);
    }

    // Optimizer on the thread's Q float4s in dealt order (g from averaged() of the same round,
    // vi0 = number of the round's first vector): parameter and state fetched here; results, and
    // the averaged gradient where asked for, stored with the policy of the calling kernel's kind.
    // STREAM: parameters and state are too large to stay in the memory-side cache until the next
    // step, so they are read and written as streaming data.
    template <bool ONE_PASS = true, bool STREAM = false>
    __device__ __forceinline__ void apply(const f32x4 (&g)[Q], int vi0, int K, const OptArgs &o, f32x4 *deal_buf) const {
        const unsigned bytes = unsigned(len) * 4u;
        const __amdgpu_buffer_rsrc_t p_out = make_rsrc(p, bytes);
        const __amdgpu_buffer_rsrc_t s1_out = make_rsrc(s1, bytes);
        const __amdgpu_buffer_rsrc_t s2_out = make_rsrc(s2, ADAM ? bytes : 0u);
        const __amdgpu_buffer_rsrc_t m_out = make_rsrc(m, MEAN == CMN_MEAN_TO_MEAN_GRADS ? bytes : 0u);
        constexpr int ST = STREAM ? kStoreStateStream : ONE_PASS ? kStoreStateOnePass : kStoreStatePhase2;
        const unsigned end = unsigned(nvec) * VEC;             // floats of the tile covered by whole vectors
        unsigned x[Q];
        f32x4 pv[Q], s1v[Q], s2v[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            x[q] = unsigned(vi0) * VEC + dealt_offset<Q>(q);   // multiple of 4, like end
            if (x[q] < end) {
                pv[q] = STREAM ? load_stream<f32x4>(p + head + x[q]) : load_vec<f32x4>(p + head + x[q]);
                s1v[q] = STREAM ? load_stream<f32x4>(s1 + head + x[q]) : load_vec<f32x4>(s1 + head + x[q]);
                if (ADAM) s2v[q] = STREAM ? load_stream<f32x4>(s2 + head + x[q]) : load_vec<f32x4>(s2 + head + x[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (x[q] < end) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float pi = pv[q][i], a = s1v[q][i], b = ADAM ? s2v[q][i] : 0.0f;
                    opt_update<OPT>(g[q][i], pi, a, b, o);
                    pv[q][i] = pi; s1v[q][i] = a;
                    if (ADAM) s2v[q][i] = b;
                }
                const unsigned off = (unsigned(head) + x[q]) * 4u;
                if (SRC == SRC_FOLD && MEAN == CMN_MEAN_TO_MEAN_GRADS) store_vec<kStoreAverage>(m_out, off, g[q]);
                if (ADAM) store_vec<ST>(s2_out, off, s2v[q]);
                store_vec<ST>(s1_out, off, s1v[q]);
                store_vec<ST>(p_out, off, pv[q]);
            }
        }
        if constexpr (SRC == SRC_FOLD && MEAN == CMN_MEAN_TO_ALL_REPLICAS) {
            // every gradient of these vectors has been read before; hand the average to each replica,
            // encoded from run order (one 16-byte vector per thread again)
            f32x4 r[Q];
#pragma unroll
            for (int q = 0; q < Q; ++q) r[q] = g[q];
            wave_undeal<Q>(r, deal_buf);
            const int vi = vi0 + int(threadIdx.x);
            if (vi < nvec) {
                float gb[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) gb[i] = r[i / 4][i % 4];
                const typename G::raw avg = G::encode_vec(gb);
                const unsigned e = unsigned(head + vi * VEC);
                for (int k = 0; k < K; ++k) {
                    elem *dst = static_cast<elem *>(const_cast<void *>(gcol[k])) + e0;
                    store_vec<kStoreAverage>(make_rsrc(dst, unsigned(len) * unsigned(sizeof(elem))), e * unsigned(sizeof(elem)), avg);
                }
            }
        }
    }

    // The one-pass step of a list with few fp32 replicas, where parameter and state fetches are a large share
    // of a tile's reads: they are requested before the fold, so that they travel together with the gradients,
    // and everything is stored afterwards (Q = 1: run order and dealt order coincide).
    template <int U>
    __device__ __forceinline__ void state_first_step(int vi0, const float *const *scale_ptrs, int K, float inv_k,
                                                     const OptArgs &o, f32x4 *deal_buf) const {
        static_assert(Q == 1 && SRC == SRC_FOLD && MEAN != CMN_MEAN_TO_ALL_REPLICAS, "fp32 gradients, average stored at most once");
        const unsigned x = (unsigned(vi0) + threadIdx.x) * 4u, end = unsigned(nvec) * 4u;
        f32x4 pv = {}, s1v = {}, s2v = {};
        if (x < end) {
            pv = load_vec<f32x4>(p + head + x);
            s1v = load_vec<f32x4>(s1 + head + x);
            if (ADAM) s2v = load_vec<f32x4>(s2 + head + x);
        }
        f32x4 g[1];
        averaged<U>(g, vi0 + int(threadIdx.x), scale_ptrs, K, inv_k, deal_buf);
        if (x < end) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float pi = pv[i], a = s1v[i], b = ADAM ? s2v[i] : 0.0f;
                opt_update<OPT>(g[0][i], pi, a, b, o);
                pv[i] = pi; s1v[i] = a;
                if (ADAM) s2v[i] = b;
            }
            const unsigned bytes = unsigned(len) * 4u, off = (unsigned(head) + x) * 4u;
            if (MEAN == CMN_MEAN_TO_MEAN_GRADS) store_vec<kStoreAverage>(make_rsrc(m, bytes), off, g[0]);
            if (ADAM) store_vec<kStoreStateOnePass>(make_rsrc(s2, bytes), off, s2v);
            store_vec<kStoreStateOnePass>(make_rsrc(s1, bytes), off, s1v);
            store_vec<kStoreStateOnePass>(make_rsrc(p, bytes), off, pv);
        }
    }

    // ragged head and tail of the tile (or the whole tile when its streams share no alignment):
    // one element per thread, start to finish
    __device__ __forceinline__ void ragged(const float *const *scale_ptrs, int K, float inv_k, const OptArgs &o) const {
        const int n_single = head + (len - tail0);
        for (int i = threadIdx.x; i < n_single; i += kBlock) {
            const int e = i < head ? i : tail0 + (i - head);
            float gb;
            if (SRC == SRC_MEAN) {
                gb = m[e];
            } else {
                float acc = sum_identity();
                for (int j = 0; j < K; ++j) {
                    const int r = ring_rank(s, j, K);
                    acc = acc + G::decode(static_cast<const elem *>(gcol[r])[e0 + e],
                                          DT == CMN_I8S ? load_uniform(scale_ptrs[r] + chunk) : 1.0f);
                }
                gb = acc * inv_k;
            }
            float pi = p[e], a = s1[e], b = ADAM ? s2[e] : 0.0f;
            opt_update<OPT>(gb, pi, a, b, o);
            if (SRC == SRC_FOLD && MEAN == CMN_MEAN_TO_MEAN_GRADS) m[e] = gb;
            if (ADAM) s2[e] = b;
            s1[e] = a;
            p[e] = pi;
            if (SRC == SRC_FOLD && MEAN == CMN_MEAN_TO_ALL_REPLICAS) {
                const elem avg = G::encode(gb);
                for (int k = 0; k < K; ++k) static_cast<elem *>(const_cast<void *>(gcol[k]))[e0 + e] = avg;
            }
        }
    }
};

// Streaming kernel: one workgroup per tile, everything in one go.
// U = gradient vectors requested back to back before the first one is consumed.
template <int DT, int U, int SRC, int MEAN, int OPT>
__global__ __launch_bounds__(kBlock) void k_step(
    const DeviceTile *__restrict__ tiles, const void *const *__restrict__ grad_cols,
    const float *const *__restrict__ scale_ptrs, int K, float inv_k, OptArgs o, int stream_state) {
    using TV = TileView<DT, SRC, MEAN, OPT>;
    constexpr int Q = TV::Q;
    __shared__ f32x4 deal_buf[deal_buffer_vectors<Q>()];
    const TV tv(load_tile(tiles, blockIdx.x), grad_cols, K);
    for (int vi0 = 0; vi0 < tv.nvec; vi0 += kBlock) {          // same trip count for the whole workgroup
        f32x4 g[Q];
        if constexpr (SRC == SRC_MEAN) {
            if (stream_state) tv.template averaged_from_mean<true>(g, vi0 + int(threadIdx.x));
            else tv.template averaged_from_mean<false>(g, vi0 + int(threadIdx.x));
        } else {
            tv.template averaged<U>(g, vi0 + int(threadIdx.x), scale_ptrs, K, inv_k, deal_buf);
        }
        if (stream_state) tv.template apply<true, true>(g, vi0, K, o, deal_buf);
        else tv.template apply<true, false>(g, vi0, K, o, deal_buf);
    }
    tv.ragged(scale_ptrs, K, inv_k, o);
}

// The same for lists of at most kStateFirstReplicas fp32 replicas whose state stays in the memory-side cache:
// parameters and state are requested ahead of the gradients (ResNet-50, K = 4: 118 -> 116 us, with Adam
// 170 -> 165 us).  From about 8 replicas on that only delays the gradient loads (K = 12 cold: 272 -> 276 us), and
// narrow storage types would pay for holding their 2 or 4 float4s per stream across the fold with occupancy.
template <int U, int MEAN, int OPT>
__global__ __launch_bounds__(kBlock) void k_step_state_first(
    const DeviceTile *__restrict__ tiles, const void *const *__restrict__ grad_cols, int K, float inv_k, OptArgs o) {
    using TV = TileView<CMN_F32, SRC_FOLD, MEAN, OPT>;
    __shared__ f32x4 deal_buf[1];
    const TV tv(load_tile(tiles, blockIdx.x), grad_cols, K);
    for (int vi0 = 0; vi0 < tv.nvec; vi0 += kBlock) tv.template state_first_step<U>(vi0, nullptr, K, inv_k, o, deal_buf);
    tv.ragged(nullptr, K, inv_k, o);
}

// Two-phase persistent kernel for the fused step.  Mixing even a few stores into a saturated
// read stream slows the reads on MI355X by far more than the stores' byte share, so the
// work is ordered to keep them apart in time: a workgroup first folds the gradients of up
// to M of its tiles (pure reads) and parks the averaged gradients in registers, then
// updates the parameters and optimizer state of those tiles (a short in-place read+write
// burst).  All workgroups start together and run at the same rate, so the phases separate
// chip-wide without any barrier; results do not depend on it.  A tile is exactly one
// 16-byte vector per thread here (tile_elems == kBlock * VEC).
template <int DT, int U, int MEAN, int OPT>
__global__ __launch_bounds__(kBlock, 2) void k_step_two_phase(
    const DeviceTile *__restrict__ tiles, const void *const *__restrict__ grad_cols,
    const float *const *__restrict__ scale_ptrs, int K, float inv_k, OptArgs o, int n_tiles, int stream_state) {
    using TV = TileView<DT, SRC_FOLD, MEAN, OPT>;
    constexpr int Q = TV::Q;
    constexpr int M = kStashFloats / TV::VEC;
    __shared__ f32x4 deal_buf[deal_buffer_vectors<Q>()];
    const int W = gridDim.x;
    for (int tile0 = blockIdx.x; tile0 < n_tiles; tile0 += W * M) {
        f32x4 gbar[M][Q];                                      // dealt order
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int ti = tile0 + m * W;
            if (ti < n_tiles) {
                const TV tv(load_tile(tiles, ti), grad_cols, K);
                tv.template averaged<U, true>(gbar[m], int(threadIdx.x), scale_ptrs, K, inv_k, deal_buf);
                tv.ragged(scale_ptrs, K, inv_k, o);
            }
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int ti = tile0 + m * W;
            if (ti < n_tiles) {
                const TV tv(load_tile(tiles, ti), grad_cols, K);
                if (stream_state) tv.template apply<false, true>(gbar[m], 0, K, o, deal_buf);
                else tv.template apply<false, false>(gbar[m], 0, K, o, deal_buf);
            }
        }
    }
}

// Parameters and optimizer state of a large model cannot stay in the memory-side cache from one
// kernel to the next: then they are streamed (VGG-16, 1.1-1.7 GB: fused step 1785 -> 1730 us,
// cmn_momentum_sgd 525 -> 480 us).  The write phase of the fused step keeps the cached policy up to
// twice the cache size (ResNet-50 with Adam, 306 MB: 570 vs 585 us on cache-swept launches).  The
// optimizer-only kernels, which run behind cmn_scale_unpack and also read the mean gradient, gain
// from streaming as soon as mean gradient + parameters + state exceed the cache by a quarter
// (behind a cache sweep and the unpack kernel, cached vs streamed: MomentumSGD 20 M elements, 240 MB:
// 62 vs 63 us, 32 M, 384 MB: 96 vs 92, 50 M: 166 vs 145; Adam 16 M, 256 MB: 67 vs 70, 25.6 M, 409 MB:
// 113 vs 110, 50 M: 245 vs 207 us).
template <int SRC, int OPT>
inline int stream_state(const cmn_plan *p) {
    const double state = double(p->N) * (OPT == OPT_ADAM ? 12.0 : 8.0);
    if (SRC == SRC_MEAN) return int(state + 4.0 * double(p->N) > 1.25 * 256.0 * 1024.0 * 1024.0);
    return int(beyond_cache(state));
}

template <int DT, int SRC, int MEAN, int OPT>
inline hipError_t launch_k_step(const cmn_plan *p, const char *ws, int64_t tile_begin, int64_t tile_count,
                                const OptArgs &o, hipStream_t s) {
    constexpr int U = 16;
    if constexpr (DT == CMN_F32 && SRC == SRC_FOLD && MEAN != CMN_MEAN_TO_ALL_REPLICAS) {
        if (state_first_step(p, OPT == OPT_ADAM ? 12 : 8, MEAN))
            return launch_kernel(k_step_state_first<U, MEAN, OPT>, dim3(unsigned(tile_count)), dim3(kBlock), 0, s,
                                 ws_ptr<const DeviceTile>(ws, p->ws.tiles) + tile_begin,
                                 ws_ptr<const void *const>(ws, p->ws.grad_cols), p->K, 1.0f / float(p->K), o);
    }
    return launch_kernel(k_step<DT, U, SRC, MEAN, OPT>, dim3(unsigned(tile_count)), dim3(kBlock), 0, s,
                       ws_ptr<const DeviceTile>(ws, p->ws.tiles) + tile_begin,
                       ws_ptr<const void *const>(ws, p->ws.grad_cols), ws_ptr<const float *const>(ws, p->ws.scale_ptrs),
                       p->K, 1.0f / float(p->K), o, stream_state<SRC, OPT>(p));
}

template <int DT, int MEAN, int OPT>
inline hipError_t launch_k_two_phase(const cmn_plan *p, const char *ws, int64_t tile_begin, int64_t tile_count,
                                     const OptArgs &o, hipStream_t s) {
    constexpr int U = 8;
    const int64_t resident = two_phase_grid(p);
    const unsigned grid = unsigned(tile_count < resident ? tile_count : resident);
    return launch_kernel(k_step_two_phase<DT, U, MEAN, OPT>, dim3(grid), dim3(kBlock), 0, s,
                       ws_ptr<const DeviceTile>(ws, p->ws.tiles) + tile_begin,
                       ws_ptr<const void *const>(ws, p->ws.grad_cols), ws_ptr<const float *const>(ws, p->ws.scale_ptrs),
                       p->K, 1.0f / float(p->K), o, int(tile_count), stream_state<SRC_FOLD, OPT>(p));
}

// Fused step (SRC_FOLD) over tensors [t0, t1) with the tables at device address ws (the workspace a
// plan was bound to, or any other image of the same layout); `have` says which tensor lists those
// tables hold.  Validation shared by the SGD and Adam entry points.
template <int OPT>
inline int launch_fused_at(const cmn_plan *plan, const char *ws, const BoundLists &have, int t0, int t1, int mean_dest,
                           const OptArgs &o, void *stream) {
    if (t0 < 0 || t1 < t0 || t1 > plan->T) return CMN_EINVAL;
    if (mean_dest != CMN_MEAN_NONE && mean_dest != CMN_MEAN_TO_MEAN_GRADS && mean_dest != CMN_MEAN_TO_ALL_REPLICAS)
        return CMN_EINVAL;
    if (!have.grads || !have.opt || (mean_dest == CMN_MEAN_TO_MEAN_GRADS && !have.mean)) return CMN_EUNBOUND;
    if (OPT == OPT_ADAM && !have.state2) return CMN_EUNBOUND;
    if (plan->dtype == CMN_I8S) {
        if (mean_dest == CMN_MEAN_TO_ALL_REPLICAS) return CMN_EINVAL;
        if (!have.scales) return CMN_EUNBOUND;
    }
    const int64_t b = plan->first_tile[size_t(t0)], n = plan->first_tile[size_t(t1)] - b;
    if (n == 0) return CMN_OK;
    if (n > 0x7fffffffLL) return CMN_ESIZE;            // one workgroup per tile must fit a grid
    hipStream_t s = static_cast<hipStream_t>(stream);
    // A launch of the persistent kernel costs about 8 us more than one of the one-pass kernel (its
    // workgroups start and drain together) and repays that only over a few thousand tiles: small
    // layer groups of a bucketed step take the one-pass kernel (ResNet-50, K = 32, 16 groups:
    // 739 -> 651 us per step).
    const bool two_phase = fused_range_kernel_kind(plan, OPT == OPT_ADAM, mean_dest, n) == 2;
    const int64_t per_launch = two_phase_launches(plan, n).second;   // one launch per round of the persistent grid
    hipError_t err = hipSuccess;      // of this call's launches only: the runtime's sticky last error is not consulted
#define CMN_STEP_CASE(DT, MEAN)                                                                          \
    do {                                                                                                 \
        if constexpr (DT != CMN_I8S) {      /* int8 storage never takes the two-phase kernel */          \
            if (two_phase) {                                                                             \
                for (int64_t b0 = 0; b0 < n && err == hipSuccess; b0 += per_launch)                      \
                    err = launch_k_two_phase<DT, MEAN, OPT>(plan, ws, b + b0, n - b0 < per_launch ? n - b0 : per_launch, o, s); \
                break;                                                                                   \
            }                                                                                            \
        }                                                                                                \
        err = launch_k_step<DT, SRC_FOLD, MEAN, OPT>(plan, ws, b, n, o, s);                              \
    } while (0)
#define CMN_STEP_DTYPE(DT)                                                                  \
    do {                                                                                    \
        if (mean_dest == CMN_MEAN_NONE) CMN_STEP_CASE(DT, CMN_MEAN_NONE);                   \
        else if (mean_dest == CMN_MEAN_TO_MEAN_GRADS) CMN_STEP_CASE(DT, CMN_MEAN_TO_MEAN_GRADS); \
        else CMN_STEP_CASE(DT, CMN_MEAN_TO_ALL_REPLICAS);                                   \
    } while (0)
    if (plan->dtype == CMN_F32) CMN_STEP_DTYPE(CMN_F32);
    else if (plan->dtype == CMN_F16) CMN_STEP_DTYPE(CMN_F16);
    else if (plan->dtype == CMN_BF16) CMN_STEP_DTYPE(CMN_BF16);
    else if (mean_dest == CMN_MEAN_NONE) CMN_STEP_CASE(CMN_I8S, CMN_MEAN_NONE);
    else CMN_STEP_CASE(CMN_I8S, CMN_MEAN_TO_MEAN_GRADS);
#undef CMN_STEP_DTYPE
#undef CMN_STEP_CASE
    return err == hipSuccess ? CMN_OK : CMN_EHIP;
}

// The same on the workspace the plan is bound to.
template <int OPT>
inline int launch_fused(const cmn_plan *plan, int t0, int t1, int mean_dest, const OptArgs &o, void *stream) {
    if (int rc = check_launch(plan)) return rc;
    return launch_fused_at<OPT>(plan, plan->dev_ws, bound_lists(plan), t0, t1, mean_dest, o, stream);
}

// Optimizer alone (SRC_MEAN) over all tensors.
template <int OPT>
inline int launch_optimizer(const cmn_plan *plan, const OptArgs &o, void *stream) {
    if (int rc = check_launch(plan)) return rc;
    if (!plan->have_opt || !plan->have_mean) return CMN_EUNBOUND;
    if (OPT == OPT_ADAM && !plan->have_state2) return CMN_EUNBOUND;
    if (plan->n_tiles == 0) return CMN_OK;
    if (plan->n_tiles > 0x7fffffffLL) return CMN_ESIZE;
    const hipError_t err = launch_k_step<CMN_F32, SRC_MEAN, CMN_MEAN_NONE, OPT>(plan, plan->dev_ws, 0, plan->n_tiles, o,
                                                                                static_cast<hipStream_t>(stream));
    return err == hipSuccess ? CMN_OK : CMN_EHIP;
}

// lr_t of Adam: the bias corrections of both moments folded into the step size.
inline float adam_step_size(float alpha, float beta1, float beta2, int t) {
    const double c1 = 1.0 - std::pow(double(beta1), double(t));
    const double c2 = 1.0 - std::pow(double(beta2), double(t));
    return float(double(alpha) * std::sqrt(c2) / c1);
}

}  // namespace cmn
