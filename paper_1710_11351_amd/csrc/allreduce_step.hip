// Entry points of the fused aggregation + update step (S1..S5 in one pass over HBM)
// with MomentumSGD, over the whole tensor list or a range of it, and (at the end of the file) the
// variant of it that keeps its tables in the library's own device array.  (The Adam entry points
// live in allreduce_adam_step.hip so that the two sets of kernel variants build in parallel.)
// HBM traffic per element: K gradient reads + parameter and optimizer state read and
// written (+ the averaged gradient, once or K times, if asked for).
#include <cmath>
#include <cstring>
#include <mutex>

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

// ---------------------------------------------------------------------------------------------
// cmn_allreduce_step_noalloc: the fused MomentumSGD step for callers that cannot allocate
// device memory (code under HIP graph capture, serving loops, harnesses that forbid it).
// cmn_allreduce_step reads its offset, pointer and tile tables from a workspace the caller
// allocated and handed to cmn_plan_bind; here the same tables live in one array that is part
// of the library's code object, so that no workspace, no bind call and no allocation is needed.
//
// The tables reach the array through small kernels that carry the bytes as a by-value
// argument: stream-ordered, no host buffer has to outlive the call, and under stream capture
// they become ordinary kernel nodes (no memcpy or memset nodes).  A caller that steps the same
// tensors every iteration pays for that once: the host remembers which image the array of each
// device holds and launches only the step kernels while it has not changed.
namespace cmn {

static_assert(CMN_NOALLOC_SCRATCH_BYTES % 256 == 0, "whole 256-byte units");

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress; the device address it yields is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[CMN_NOALLOC_SCRATCH_BYTES];

constexpr int kChunkVectors = 224;                 // 3584 bytes: a kernel's arguments may take 4 KB in all
struct TableChunk {
    u32x4 v[kChunkVectors];
};

// dst[0 .. n) = c.v[0 .. n), n <= kChunkVectors, one 16-byte vector per thread.
__global__ __launch_bounds__(kBlock) void k_write_tables(u32x4 *__restrict__ dst, TableChunk c, int n) {
    const int i = threadIdx.x;
    if (i < n) dst[i] = c.v[i];
}

constexpr int kMaxDevices = 64;
struct DeviceScratch {
    unsigned char *ptr = nullptr;      // device address of this GPU's copy of `scratch`
    uint64_t owner_serial = 0;         // plan and image generation whose tables the array holds (0: unknown)
    uint64_t owner_generation = 0;
    bool replays_possible = false;     // a captured graph may rewrite the array at any time: never trust the above
};
static DeviceScratch g_scratch[kMaxDevices];
static std::mutex g_scratch_mutex;

}  // namespace cmn

extern "C" int cmn_allreduce_step_noalloc(cmn_plan *plan, const void *const *grad_ptrs, void *const *param_ptrs,
                                          void *const *vel_ptrs, void *const *mean_grad_ptrs, float lr, float mu,
                                          float wd, int mean_dest, void *stream) {
    if (!plan || !grad_ptrs || !param_ptrs || !vel_ptrs) return CMN_ENULL;
    if (plan->dtype == CMN_I8S) return CMN_EINVAL;                    // its scales are bound through a workspace
    if (plan->ws.total > CMN_NOALLOC_SCRATCH_BYTES) return CMN_ESIZE;  // tables larger than the library's array
    int rc;
    if ((rc = check_ptr_array(plan, grad_ptrs, plan->K, elem_bytes(plan->dtype)))) return rc;
    if ((rc = check_ptr_array(plan, param_ptrs, 1, 4))) return rc;
    if ((rc = check_ptr_array(plan, vel_ptrs, 1, 4))) return rc;
    if (mean_grad_ptrs && (rc = check_ptr_array(plan, mean_grad_ptrs, 1, 4))) return rc;
    if (mean_dest != CMN_MEAN_NONE && mean_dest != CMN_MEAN_TO_MEAN_GRADS && mean_dest != CMN_MEAN_TO_ALL_REPLICAS)
        return CMN_EINVAL;
    if (mean_dest == CMN_MEAN_TO_MEAN_GRADS && !mean_grad_ptrs) return CMN_EUNBOUND;
    if (plan->n_tiles == 0) return CMN_OK;

    hipStream_t s = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return CMN_EHIP;
    if (dev >= kMaxDevices) return CMN_ESIZE;
    DeviceScratch &ds = g_scratch[dev];
    if (!ds.ptr) {                                   // once per device, with that device current
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CMN_EHIP;
        ds.ptr = static_cast<unsigned char *>(p);
    }

    // The table image of this call: rebuilt only when the pointers differ from the last call's.
    const size_t T = size_t(plan->T), K = size_t(plan->K);
    try {
        std::vector<const void *> now;
        now.reserve(K * T + 3 * T + 1);
        now.insert(now.end(), grad_ptrs, grad_ptrs + K * T);
        now.insert(now.end(), param_ptrs, param_ptrs + T);
        now.insert(now.end(), vel_ptrs, vel_ptrs + T);
        if (mean_grad_ptrs) now.insert(now.end(), mean_grad_ptrs, mean_grad_ptrs + T);
        now.push_back(reinterpret_cast<const void *>(uintptr_t(mean_grad_ptrs != nullptr)));   // with / without a mean list
        if (plan->image_generation == 0 || now != plan->static_inputs) {
            plan->static_image.resize(plan->ws.total);
            fill_table_image(plan, plan->static_image.data(), grad_ptrs, param_ptrs, vel_ptrs, mean_grad_ptrs, nullptr,
                             nullptr);
            plan->static_inputs.swap(now);
            ++plan->image_generation;
        }
    } catch (...) { return CMN_ENOMEM; }

    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) return CMN_EHIP;
    const bool capturing = cap != hipStreamCaptureStatusNone;
    if (capturing) ds.replays_possible = true;
    const bool resident = !ds.replays_possible && ds.owner_serial == plan->serial &&
                          ds.owner_generation == plan->image_generation;
    if (!resident) {
        ds.owner_serial = 0;
        const unsigned char *img = plan->static_image.data();
        const size_t n_vec = plan->ws.total / 16;                 // the layout is made of 256-byte units
        for (size_t v0 = 0; v0 < n_vec; v0 += kChunkVectors) {
            const int n = int(n_vec - v0 < size_t(kChunkVectors) ? n_vec - v0 : size_t(kChunkVectors));
            TableChunk c{};
            std::memcpy(c.v, img + v0 * 16, size_t(n) * 16);
            if (launch_kernel(k_write_tables, dim3(1), dim3(kBlock), 0, s, reinterpret_cast<u32x4 *>(ds.ptr) + v0, c,
                              n) != hipSuccess)
                return CMN_EHIP;
        }
        if (!capturing) {
            ds.owner_serial = plan->serial;
            ds.owner_generation = plan->image_generation;
        }
    }
    const OptArgs o{lr, mu, 0.0f, 0.0f, wd};
    const BoundLists have{true, true, mean_grad_ptrs != nullptr, false, false};
    return launch_fused_at<OPT_SGD>(plan, reinterpret_cast<const char *>(ds.ptr), have, 0, plan->T, mean_dest, o, stream);
}
