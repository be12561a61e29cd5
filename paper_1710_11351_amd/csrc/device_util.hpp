// Device-side helpers shared by the kernels: 16-byte vector access, exact
// decoding of stored gradients to float32, and the element-wise arithmetic of
// the scale and MomentumSGD steps.  Every float operation rounds once: the
// translation units are built with contraction off and the pragma repeats it.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/cmn.h"

#pragma clang fp contract(off)

namespace cmn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Storage traits of the gradient element type.
template <int DT> struct GradT;

template <> struct GradT<CMN_F32> {
    using elem = float;
    using raw = f32x4;                 // one 16-byte load
    static constexpr int VEC = 4;      // elements per 16-byte vector
    static __device__ __forceinline__ void accumulate(float (&acc)[4], const raw &r) {
        acc[0] = acc[0] + r.x; acc[1] = acc[1] + r.y; acc[2] = acc[2] + r.z; acc[3] = acc[3] + r.w;
    }
    static __device__ __forceinline__ float decode(elem x) { return x; }
};

template <> struct GradT<CMN_F16> {
    using elem = _Float16;
    using raw = f16x8;
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void accumulate(float (&acc)[8], const raw &r) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = acc[i] + static_cast<float>(r[i]);  // exact widening
    }
    static __device__ __forceinline__ float decode(elem x) { return static_cast<float>(x); }
};

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

// 16-byte store at byte_off that is written through L2 towards memory at once
// (cache-policy bit sc1, aux value 16) instead of lingering as a dirty line until
// evicted.  On MI355X the write traffic of a read-dominated kernel is cheaper this way
// (measured: about 2 % of the fused step's time); the data written is the same.
__device__ __forceinline__ void store_through(__amdgpu_buffer_rsrc_t r, unsigned byte_off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4v, v), r, int(byte_off), 0, 16);
}

// The K-term sum starts from -0.0f because x + (-0.0f) == x for every x, signed
// zeros included, so the first addition reproduces the first gradient exactly.
__device__ __forceinline__ constexpr float sum_identity() { return -0.0f; }

// Replica visited at position j of the fold that starts at replica s.
__device__ __forceinline__ int ring_rank(int s, int j, int K) {
    const int r = s + j;
    return r >= K ? r - K : r;
}

// MomentumSGD on one element; gbar is the averaged gradient.
__device__ __forceinline__ void sgd_update(float gbar, float &p, float &v, float lr, float mu, float wd) {
    float g = gbar;
    if (wd != 0.0f) {
        const float d = wd * p;
        g = g + d;
    }
    const float t1 = mu * v;
    const float t2 = lr * g;
    v = t1 - t2;
    p = p + v;
}

}  // namespace cmn
