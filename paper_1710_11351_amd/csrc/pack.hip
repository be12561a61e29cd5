// cmn_pack (gather) and cmn_scale_unpack (scatter): the two kernels that work in
// packed coordinates.  Both are driven by the prefix-sum offsets table of the
// tensor list, copied into LDS together with the row of T tensor pointers the
// workgroup needs; a thread finds the tensor of its 16-byte vector by binary
// search in LDS and falls back to element-wise access only where a vector
// crosses a tensor edge or a tensor is not 16-byte aligned relative to the packed
// buffer.  Lists too long for LDS are searched in global memory instead.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "plan.hpp"

#pragma clang fp contract(off)

namespace cmn {

// 16-byte vectors per thread of k_pack: all of them are loaded before the first is stored.  Two or three beat
// one, four and eight on MI355X (1 GiB copy: 6.1, 6.3, 6.2, 6.1, 5.5 TB/s for 1, 2, 3, 4, 8; ResNet-50 x 32
// replicas: 1202, 1108, 1057 us for 1, 2, 3), and four taken one after the other reach 5.9 TB/s.
constexpr int kPackIters = 3;
// 16-byte vectors per thread of k_scale_unpack, taken one after the other (loading them all first, before or
// after the table fill, was slower: 41 vs 37 us on ResNet-50); two beat four by 1-4 %.
constexpr int kUnpackIters = 2;
constexpr size_t kLdsTableBudget = 48 * 1024;  // bytes of LDS the two tables may take

// Largest t with off[t] <= i; since i < off[T] that tensor is not empty.
template <typename OffFn>
__device__ __forceinline__ int find_tensor(OffFn off, int T, long long i) {
    int lo = 0, hi = T;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off(mid) <= i) lo = mid; else hi = mid;
    }
    return lo;
}

template <int DT, bool LDS>
__global__ __launch_bounds__(kBlock) void k_pack(const long long *__restrict__ off_g,
                                                 const void *const *__restrict__ grad_rows,
                                                 void *__restrict__ packed, int T, long long N, long long L) {
    using G = GradT<DT>;
    using elem = typename G::elem;
    using raw = typename G::raw;
    constexpr int VEC = G::VEC;
    constexpr int TILE = kBlock * VEC * kPackIters;
    extern __shared__ long long lds[];  // [T+1] offsets, then [T] pointers of this replica

    const int k = blockIdx.y;
    const void *const *row_g = grad_rows + size_t(k) * size_t(T);
    if (LDS) {
        for (int i = threadIdx.x; i <= T; i += kBlock) lds[i] = off_g[i];
        for (int i = threadIdx.x; i < T; i += kBlock) lds[T + 1 + i] = reinterpret_cast<long long>(row_g[i]);
        __syncthreads();
    }
    auto off = [&](int i) -> long long { return LDS ? lds[i] : off_g[i]; };
    auto ptr = [&](int i) -> const elem * {
        return LDS ? reinterpret_cast<const elem *>(lds[T + 1 + i]) : static_cast<const elem *>(row_g[i]);
    };

    elem *dst = static_cast<elem *>(packed) + (long long)k * L;
    const long long tile_begin = (long long)blockIdx.x * TILE;
    int t = -1;
    raw out[kPackIters];
#pragma unroll
    for (int it = 0; it < kPackIters; ++it) {
        const long long i = tile_begin + (long long)(it * kBlock + threadIdx.x) * VEC;
        out[it] = raw{};                                 // padding [N, L) is +0
        if (i < N) {
            if (t < 0 || i >= off(t + 1)) t = find_tensor(off, T, i);
            const elem *src = ptr(t) + (i - off(t));
            if (i + VEC <= off(t + 1) && (reinterpret_cast<uintptr_t>(src) & 15) == 0) {
                out[it] = load_stream<raw>(src);
            } else {
                int tt = t;
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const long long idx = i + j;
                    if (idx < N) {
                        while (idx >= off(tt + 1)) ++tt;  // steps over empty tensors too
                        out[it][j] = ptr(tt)[idx - off(tt)];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int it = 0; it < kPackIters; ++it) {
        const long long i = tile_begin + (long long)(it * kBlock + threadIdx.x) * VEC;
        // the packed buffer is far larger than any cache: streaming store (4 % faster than a plain one)
        if (i < L) __builtin_nontemporal_store(out[it], reinterpret_cast<raw *>(dst + i));
    }
}

template <bool LDS, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_scale_unpack(const long long *__restrict__ off_g,
                                                         float *const *__restrict__ mean_g,
                                                         const float *__restrict__ reduced, int T, long long N,
                                                         float inv_k) {
    constexpr int TILE = kBlock * 4 * kUnpackIters;
    extern __shared__ long long lds[];
    if (LDS) {
        for (int i = threadIdx.x; i <= T; i += kBlock) lds[i] = off_g[i];
        for (int i = threadIdx.x; i < T; i += kBlock) lds[T + 1 + i] = reinterpret_cast<long long>(mean_g[i]);
        __syncthreads();
    }
    auto off = [&](int i) -> long long { return LDS ? lds[i] : off_g[i]; };
    auto ptr = [&](int i) -> float * { return LDS ? reinterpret_cast<float *>(lds[T + 1 + i]) : mean_g[i]; };

    const long long tile_begin = (long long)blockIdx.x * TILE;
    int t = -1;
    for (int it = 0; it < kUnpackIters; ++it) {
        const long long i = tile_begin + (long long)(it * kBlock + threadIdx.x) * 4;
        if (i >= N) break;
        f32x4 g = load_stream<f32x4>(reduced + i);         // i + 4 <= L: L is a multiple of 4
#pragma unroll
        for (int j = 0; j < 4; ++j) g[j] = g[j] * inv_k;
        if (t < 0 || i >= off(t + 1)) t = find_tensor(off, T, i);
        float *d = ptr(t) + (i - off(t));
        if (i + 4 <= off(t + 1) && (reinterpret_cast<uintptr_t>(d) & 15) == 0) {
            // plain: the optimizer reads it next, out of the memory-side cache (unless the model outgrows it)
            if (STREAM) __builtin_nontemporal_store(g, reinterpret_cast<f32x4 *>(d));
            else *reinterpret_cast<f32x4 *>(d) = g;
        } else {
            int tt = t;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const long long idx = i + j;
                if (idx < N) {
                    while (idx >= off(tt + 1)) ++tt;
                    ptr(tt)[idx - off(tt)] = g[j];
                }
            }
        }
    }
}

static bool tables_fit_lds(int T) { return (2 * size_t(T) + 1) * 8 <= kLdsTableBudget; }

}  // namespace cmn

using namespace cmn;

extern "C" int cmn_pack(const cmn_plan *plan, void *packed, void *stream) {
    if (int rc = check_launch(plan)) return rc;
    if (!plan->have_grads) return CMN_EUNBOUND;
    if (plan->L == 0) return CMN_OK;
    if (!packed) return CMN_ENULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256) return CMN_EALIGN;
    const int T = plan->T;
    const long long tile = kBlock * vec_elems(plan->dtype) * kPackIters;
    const long long nx = (plan->L + tile - 1) / tile;
    if (nx > 0x7fffffffLL || plan->K > 65535) return CMN_ESIZE;
    const dim3 grid(unsigned(nx), unsigned(plan->K));
    const bool lds = tables_fit_lds(T);
    const size_t shm = lds ? (2 * size_t(T) + 1) * 8 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long *off = ws_ptr<const long long>(plan, plan->ws.off_table);
    const void *const *rows = ws_ptr<const void *const>(plan, plan->ws.grad_rows);
    const long long N = plan->N, L = plan->L;
    hipError_t err;
#define CMN_LAUNCH_PACK(DT, LDS) \
    err = launch_kernel(k_pack<DT, LDS>, grid, dim3(kBlock), shm, s, off, rows, packed, T, N, L)
    if (plan->dtype == CMN_F32) { if (lds) CMN_LAUNCH_PACK(CMN_F32, true); else CMN_LAUNCH_PACK(CMN_F32, false); }
    else if (plan->dtype == CMN_I8S) { if (lds) CMN_LAUNCH_PACK(CMN_I8S, true); else CMN_LAUNCH_PACK(CMN_I8S, false); }
    else /* any 16-bit type: a bit copy */ { if (lds) CMN_LAUNCH_PACK(CMN_F16, true); else CMN_LAUNCH_PACK(CMN_F16, false); }
#undef CMN_LAUNCH_PACK
    return err == hipSuccess ? CMN_OK : CMN_EHIP;
}

extern "C" int cmn_scale_unpack(const cmn_plan *plan, const float *reduced, void *stream) {
    if (int rc = check_launch(plan)) return rc;
    if (!plan->have_mean) return CMN_EUNBOUND;
    if (plan->N == 0) return CMN_OK;
    if (!reduced) return CMN_ENULL;
    if (reinterpret_cast<uintptr_t>(reduced) % 256) return CMN_EALIGN;
    const int T = plan->T;
    const long long tile = kBlock * 4 * kUnpackIters;
    const long long nx = (plan->N + tile - 1) / tile;
    if (nx > 0x7fffffffLL) return CMN_ESIZE;
    const bool lds = tables_fit_lds(T);
    const size_t shm = lds ? (2 * size_t(T) + 1) * 8 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long *off = ws_ptr<const long long>(plan, plan->ws.off_table);
    float *const *mean = ws_ptr<float *const>(plan, plan->ws.mean_ptrs);
    const float inv_k = 1.0f / float(plan->K);
    const bool big = beyond_cache(4.0 * double(plan->N));
    hipError_t err;
#define CMN_LAUNCH_UNPACK(LDS, STREAM)                                                                       \
    err = launch_kernel(k_scale_unpack<LDS, STREAM>, dim3(unsigned(nx)), dim3(kBlock), shm, s, off, mean, reduced, T, \
                        (long long)plan->N, inv_k)
    if (lds) { if (big) CMN_LAUNCH_UNPACK(true, true); else CMN_LAUNCH_UNPACK(true, false); }
    else { if (big) CMN_LAUNCH_UNPACK(false, true); else CMN_LAUNCH_UNPACK(false, false); }
#undef CMN_LAUNCH_UNPACK
    return err == hipSuccess ? CMN_OK : CMN_EHIP;
}
