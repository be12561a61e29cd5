// Device-side helpers shared by the kernels: 16-byte vector access, exact
// decoding of stored gradients to float32, and the element-wise arithmetic of
// the scale and MomentumSGD steps.  Every float operation rounds once: the
// translation units are built with contraction off and the pragma repeats it.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <tuple>
#include <utility>

#include "../../include/cmn.h"
#include "plan.hpp"

#pragma clang fp contract(off)

namespace cmn {

// Kernel launch that hands back the launch's own status.  (The <<<>>> form reports failures only
// through the runtime's sticky last-error slot, which may hold an error of the caller's earlier
// HIP calls and which reading would clear.)  Arguments are converted to the kernel's exact
// parameter types first, since the runtime copies them by address.
template <typename... P, size_t... I>
inline hipError_t launch_kernel_impl(void (*kernel)(P...), dim3 grid, dim3 block, size_t shm, hipStream_t s,
                                     std::tuple<P...> &vals, std::index_sequence<I...>) {
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))..., nullptr};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, shm, s);
}
template <typename... P, typename... A>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t shm, hipStream_t s, A &&...a) {
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> vals{static_cast<P>(std::forward<A>(a))...};
    return launch_kernel_impl(kernel, grid, block, shm, s, vals, std::index_sequence_for<P...>{});
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef signed char i8x16 __attribute__((ext_vector_type(16)));

// Storage traits of the gradient element type.
template <int DT> struct GradT;

template <> struct GradT<CMN_F32> {
    using elem = float;
    using raw = f32x4;                 // one 16-byte load
    static constexpr int VEC = 4;      // elements per 16-byte vector
    static __device__ __forceinline__ void accumulate(float (&acc)[4], const raw &r, float /*scale*/) {
        acc[0] = acc[0] + r.x; acc[1] = acc[1] + r.y; acc[2] = acc[2] + r.z; acc[3] = acc[3] + r.w;
    }
    static __device__ __forceinline__ float decode(elem x, float /*scale*/) { return x; }
    static __device__ __forceinline__ elem encode(float x) { return x; }
    static __device__ __forceinline__ raw encode_vec(const float (&g)[4]) { return raw{g[0], g[1], g[2], g[3]}; }
};

template <> struct GradT<CMN_F16> {
    using elem = _Float16;
    using raw = f16x8;
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void accumulate(float (&acc)[8], const raw &r, float /*scale*/) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = acc[i] + static_cast<float>(r[i]);  // exact widening
    }
    static __device__ __forceinline__ float decode(elem x, float /*scale*/) { return static_cast<float>(x); }
    static __device__ __forceinline__ elem encode(float x) { return static_cast<elem>(x); }  // nearest even
    static __device__ __forceinline__ raw encode_vec(const float (&g)[8]) {
        raw r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = static_cast<elem>(g[i]);
        return r;
    }
};

template <> struct GradT<CMN_BF16> {
    using elem = unsigned short;        // raw bfloat16 bit pattern
    using raw = u16x8;
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float decode(elem x, float /*scale*/ = 1.0f) {
        return __builtin_bit_cast(float, static_cast<unsigned>(x) << 16);   // exact
    }
    static __device__ __forceinline__ elem encode(float x) {                 // nearest, ties to even
        const unsigned u = __builtin_bit_cast(unsigned, x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<elem>((u >> 16) | 0x40u);   // NaN stays NaN
        return static_cast<elem>((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
    static __device__ __forceinline__ void accumulate(float (&acc)[8], const raw &r, float /*scale*/) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = acc[i] + decode(r[i]);
    }
    static __device__ __forceinline__ raw encode_vec(const float (&g)[8]) {
        raw r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = encode(g[i]);
        return r;
    }
};

template <> struct GradT<CMN_I8S> {
    using elem = signed char;
    using raw = i8x16;
    static constexpr int VEC = 16;
    static __device__ __forceinline__ float decode(elem q, float scale) {
        const float f = static_cast<float>(q);   // exact
        return f * scale;                        // rounded once
    }
    static __device__ __forceinline__ void accumulate(float (&acc)[16], const raw &r, float scale) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = acc[i] + decode(r[i], scale);
    }
    // the average is never written back in this format
    static __device__ __forceinline__ elem encode(float) { return 0; }
    static __device__ __forceinline__ raw encode_vec(const float (&)[16]) { return raw{}; }
};

// Read of a value that no kernel of this library writes and that is the same for the whole
// wavefront (an int8 scale): through the constant address space, so that it becomes a scalar
// load instead of a vector memory instruction with 64 equal addresses.
__device__ __forceinline__ float load_uniform(const float *p) {
    return *(const __attribute__((address_space(4))) float *)(p);
}

template <typename V>
__device__ __forceinline__ V load_vec(const void *p) {
    return *reinterpret_cast<const V *>(p);
}

// Load of data that is read exactly once per launch (gradients, packed buffers):
// the non-temporal hint keeps it from displacing reusable lines in L2 and in the
// memory-side cache, and measurably raises streaming read bandwidth on MI355X.
template <typename V>
__device__ __forceinline__ V load_stream(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const V *>(p));
}

// Raw buffer descriptor over [base, base + bytes): the hardware drops stores and
// zero-fills loads that fall outside it.  base must be uniform over the wavefront.
typedef unsigned int u32x4v __attribute__((__vector_size__(16)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(void *base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, int(bytes), 0x00020000 /* 32-bit data format */);
}

// 16-byte store at byte_off with an explicit cache policy (the auxiliary operand of the
// buffer store: bit 1 = nt, bit 4 = sc1).  The data written is the same under every policy;
// which one is cheapest depends on what else the kernel has in flight, so each store site
// names its policy.
//   ST_BACK     default write-back: the line lingers dirty in L2 until evicted
//   ST_THROUGH  sc1: written through towards memory at once
//   ST_STREAM   nt: streaming data nobody re-reads soon
enum { ST_BACK = 0, ST_STREAM = 2, ST_THROUGH = 16, ST_STREAM_THROUGH = 18 };
template <int POLICY, class V>
__device__ __forceinline__ void store_vec(__amdgpu_buffer_rsrc_t r, unsigned byte_off, V v) {
    static_assert(sizeof(V) == 16, "one 16-byte vector");
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4v, v), r, int(byte_off), 0, POLICY);
}

// Per-site policies, each chosen by A/B measurement on MI355X (ResNet-50 list):
//  - p and optimizer state are read again by the next step and fit the memory-side cache:
//    streaming them out (nt) costs the one-pass kernel 17 % at K = 4.  One-pass kernels write
//    them through (2 % better than write-back while reads are in flight); the write phase of
//    the two-phase kernel is a pure burst and does best with plain write-back.
//  - the averaged gradient handed to the mean tensors or back to the K replicas is not read
//    again by this library: nt + sc1 (K = 32: 586 -> 557 us with the mean stored, 1258 -> 1089 us
//    with all replicas overwritten; K = 4: 228 -> 174 us).
constexpr int kStoreStateOnePass = ST_THROUGH;
constexpr int kStoreStatePhase2 = ST_BACK;
constexpr int kStoreStateStream = ST_STREAM_THROUGH;   // optimizer-only kernels on models larger than the cache
constexpr int kStoreAverage = ST_STREAM_THROUGH;
constexpr int kStoreReducedOnePass = ST_THROUGH;   // ring reduce, one-pass
constexpr int kStoreReducedPhase2 = ST_BACK;       // ring reduce, two-phase (scale+unpack reads it next; nt: no gain)

// Re-dealing the floats of a wavefront so that fp32 accesses coalesce.  A thread that loads one
// 16-byte vector of a narrow type owns 4Q consecutive elements (Q = 2 for 16-bit, 4 for int8
// gradients), so its Q float4s lie 16Q bytes from the next lane's and every fp32 load or store
// instruction would touch only half or a quarter of each cache line (measured: the int8 ring
// reduce at K = 4 takes 88 us that way and 33 us dealt).  A wavefront's 64 runs form one block
// of 256Q consecutive floats.
//   run order:   v[q] = floats [4q, 4q + 4) of lane l's run, which starts at float 4Q*l
//   dealt order: v[q] = floats [256q + 4l, 256q + 4l + 4) of the block: instruction q covers 1 KB
// buf holds kBlock * Q float4s of LDS; each wavefront uses its own part, so the exchange needs
// no workgroup barrier.  Every lane of the wavefront must call these (inactive ones pass zeros).
template <int Q>
__device__ __forceinline__ void wave_exchange(f32x4 (&v)[Q], f32x4 *buf, bool to_dealt) {
    if constexpr (Q > 1) {
        const int lane = threadIdx.x & 63;
        f32x4 *w = buf + (threadIdx.x >> 6) * 64 * Q;
#pragma unroll
        for (int q = 0; q < Q; ++q) w[to_dealt ? lane * Q + q : q * 64 + lane] = v[q];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int q = 0; q < Q; ++q) v[q] = w[to_dealt ? q * 64 + lane : lane * Q + q];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the next exchange must not overtake these reads
        __builtin_amdgcn_wave_barrier();
    }
}
template <int Q> __device__ __forceinline__ void wave_deal(f32x4 (&v)[Q], f32x4 *buf) { wave_exchange<Q>(v, buf, true); }
template <int Q> __device__ __forceinline__ void wave_undeal(f32x4 (&v)[Q], f32x4 *buf) { wave_exchange<Q>(v, buf, false); }

// Float offset, inside the 256Q * 4 floats the workgroup's 256 runs cover, of this thread's
// q-th float4 in dealt order.  For Q = 1 it is the thread's own run: 4 * threadIdx.x.
template <int Q>
__device__ __forceinline__ unsigned dealt_offset(int q) {
    return (threadIdx.x >> 6) * 256u * Q + unsigned(q) * 256u + (threadIdx.x & 63) * 4u;
}
template <int Q> constexpr int deal_buffer_vectors() { return Q > 1 ? kBlock * Q : 1; }

// The K-term sum starts from -0.0f because x + (-0.0f) == x for every x, signed
// zeros included, so the first addition reproduces the first gradient exactly.
__device__ __forceinline__ constexpr float sum_identity() { return -0.0f; }

// Replica visited at position j of the fold that starts at replica s.
__device__ __forceinline__ int ring_rank(int s, int j, int K) {
    const int r = s + j;
    return r >= K ? r - K : r;
}

// Fold replicas [j, j + B) of the fixed order into acc: B vector loads are issued back to
// back, then added strictly in order.  ptr_of(j) yields the address of replica j's vector,
// scale_of(j) its scale (only int8 storage uses it).
template <int DT, int B, typename PtrFn, typename ScaleFn>
__device__ __forceinline__ void fold_batch(float (&acc)[GradT<DT>::VEC], int j, PtrFn ptr_of, ScaleFn scale_of) {
    using G = GradT<DT>;
    typename G::raw g[B];
    float sc[B];
#pragma unroll
    for (int u = 0; u < B; ++u) {
        g[u] = load_stream<typename G::raw>(ptr_of(j + u));
        sc[u] = DT == CMN_I8S ? scale_of(j + u) : 1.0f;
    }
#pragma unroll
    for (int u = 0; u < B; ++u) G::accumulate(acc, g[u], sc[u]);
}

// The last n < B replicas of the order as one batch: the loads that exist are requested together
// (n is uniform over the workgroup, so the conditions are scalar branches).
template <int DT, int B, typename PtrFn, typename ScaleFn>
__device__ __forceinline__ void fold_tail(float (&acc)[GradT<DT>::VEC], int j, int n, PtrFn ptr_of, ScaleFn scale_of) {
    using G = GradT<DT>;
    typename G::raw g[B];
    float sc[B];
#pragma unroll
    for (int u = 0; u < B; ++u)
        if (u < n) {
            g[u] = load_stream<typename G::raw>(ptr_of(j + u));
            sc[u] = DT == CMN_I8S ? scale_of(j + u) : 1.0f;
        }
#pragma unroll
    for (int u = 0; u < B; ++u)
        if (u < n) G::accumulate(acc, g[u], sc[u]);
}

// The whole K-term fold: batches of U, then the remainder.  ONE_TAIL: the remainder goes out as one batch
// (what the two-phase kernels want: at two waves per SIMD every extra round trip shows, K = 13: 290 -> 261 us,
// K = 15: 318 -> 292 us).  Otherwise it goes out in halving batches of 8, 4, 2, 1, which costs the one-pass
// kernels nothing at their occupancy and keeps their register count (the single batch would raise it by 10-30,
// for int8 to 256, and slow K = 4 by 3 %).
template <int DT, int U, bool ONE_TAIL = false, typename PtrFn, typename ScaleFn>
__device__ __forceinline__ void fold_all(float (&acc)[GradT<DT>::VEC], int K, PtrFn ptr_of, ScaleFn scale_of) {
    int j = 0;
    for (; j + U <= K; j += U) fold_batch<DT, U>(acc, j, ptr_of, scale_of);
    if constexpr (ONE_TAIL) {
        if (j < K) fold_tail<DT, U>(acc, j, K - j, ptr_of, scale_of);
    } else {
        if (U > 8 && j + 8 <= K) { fold_batch<DT, 8>(acc, j, ptr_of, scale_of); j += 8; }
        if (U > 4 && j + 4 <= K) { fold_batch<DT, 4>(acc, j, ptr_of, scale_of); j += 4; }
        if (U > 2 && j + 2 <= K) { fold_batch<DT, 2>(acc, j, ptr_of, scale_of); j += 2; }
        if (j < K) fold_batch<DT, 1>(acc, j, ptr_of, scale_of);
    }
}

// Optimizer hyper-parameters as the kernels receive them (by value).
//   MomentumSGD: a = lr, b = mu.        Adam: a = lr_t, b = 1 - beta1, c = 1 - beta2, d = eps.
struct OptArgs {
    float a, b, c, d, wd;
};

enum { OPT_SGD = 0, OPT_ADAM = 1 };

// One element of the optimizer step; gbar is the averaged gradient, s1 the velocity
// (MomentumSGD) or first moment (Adam), s2 Adam's second moment.  Every operation
// rounds to float32 once; sqrt and the division are the correctly rounded ones.
template <int OPT>
__device__ __forceinline__ void opt_update(float gbar, float &p, float &s1, float &s2, const OptArgs &o) {
    float g = gbar;
    if (o.wd != 0.0f) {
        const float dec = o.wd * p;
        g = g + dec;
    }
    if (OPT == OPT_SGD) {
        const float t1 = o.b * s1;
        const float t2 = o.a * g;
        s1 = t1 - t2;
        p = p + s1;
    } else {
        const float t1 = g - s1;
        const float t2 = o.b * t1;
        s1 = s1 + t2;
        const float t3 = g * g;
        const float t4 = t3 - s2;
        const float t5 = o.c * t4;
        s2 = s2 + t5;
        const float root = sqrtf(s2);
        const float den = root + o.d;
        const float q = s1 / den;
        const float u = o.a * q;
        p = p - u;
    }
}

}  // namespace cmn
