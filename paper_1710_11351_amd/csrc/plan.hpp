// Internal: the plan object behind the opaque cmn_plan handle and the layout of
// its device-side tables.  Host code only; the kernels receive plain pointers.
#pragma once

#include <cstddef>
#include <cstdint>
#include <utility>
#include <vector>

#include "../../include/cmn.h"

namespace cmn {

constexpr int kMaxTensors = 1 << 20;
constexpr int kMaxReplicas = 4096;
constexpr int kBlock = 256;  // threads per workgroup of every kernel (4 wavefronts)

// Elements of one cmn_tile at most: kBlock threads x one 16-byte vector x kTileIters.
constexpr int kTileIters = 1;

// Floats a thread of a two-phase kernel parks in registers between its read phase and its
// write phase (leaves ~50 of the 256 registers available at two waves per SIMD for the fold).
constexpr int kStashFloats = 200;

enum { STEP_AUTO = 0, STEP_ONE_PASS = 1, STEP_TWO_PHASE = 2 };

// Up to this many fp32 replicas the one-pass fused step requests parameters and state ahead of the gradients.
constexpr int kStateFirstReplicas = 4;

// Fewer tiles than this in one launch of the fused step: the one-pass kernel, whatever the plan-wide choice.
constexpr int64_t kMinTwoPhaseTiles = 4096;

// What the tensor-space kernels read per tile: the fields of the public cmn_tile plus the tile's
// own addresses, so that one 64-byte scalar load yields everything but the gradient pointers
// (looking p, state and mean gradient up by tensor index would put three more dependent scalar
// loads in front of every tile's first vector load).
struct DeviceTile {
    float *p, *s1, *s2, *m;   // parameter, optimizer state (velocity or first moment), Adam's second moment,
                              // mean gradient, each at element e0 of the tensor; null where not bound
    int64_t e0;
    int32_t len, tensor, start_rank, chunk;
    int8_t head[8];
};
static_assert(sizeof(DeviceTile) == 64, "one scalar cache line");

// Whether a working set that one kernel writes and the next one reads is too large for the 256 MB
// memory-side cache to carry it over (measured boundary: 306 MB still profits from the cache,
// 1.7 GB profits from streaming loads and stores instead).
inline bool beyond_cache(double bytes) { return bytes > 2.0 * 256.0 * 1024.0 * 1024.0; }

inline int elem_bytes(int dtype) { return dtype == CMN_F32 ? 4 : dtype == CMN_I8S ? 1 : 2; }
inline int vec_elems(int dtype) { return 16 / elem_bytes(dtype); }

// Byte offsets of the tables inside the caller's device workspace (each 256-aligned).
struct WorkspaceLayout {
    size_t off_table = 0;    // int64 [T+1]   prefix sums of numel
    size_t grad_rows = 0;    // void* [K][T]  replica-major (rows go to LDS in pack)
    size_t grad_cols = 0;    // void* [T][K]  tensor-major (one tile reads K neighbours)
    size_t param_ptrs = 0;   // float* [T]
    size_t vel_ptrs = 0;     // float* [T]
    size_t mean_ptrs = 0;    // float* [T]
    size_t state2_ptrs = 0;  // float* [T]   Adam second moments
    size_t scale_ptrs = 0;   // float* [K]   per-replica arrays of n_chunks scales (int8 gradients)
    size_t tiles = 0;        // DeviceTile [n_tiles]        // cmn_tile [n_tiles]
    size_t total = 0;
};

}  // namespace cmn

struct cmn_plan {
    int T = 0, K = 1, C = 1, align_bytes = 256, dtype = CMN_F32, ring_rotate = 1;
    int tile_elems = 0;
    // launch-shape knobs, fixed at creation from the environment (results never depend on them)
    int step_mode = cmn::STEP_AUTO;      // CMN_STEP_KERNEL=stream | two_phase: force one kind of kernel where it applies
    int grid_limit = 0;                  // CMN_TWO_PHASE_GRID: at most this many persistent workgroups (0: 2 per CU)
    std::vector<int64_t> numel;  // [T]
    std::vector<int64_t> off;    // [T+1]
    int64_t N = 0, chunk_elems = 0, L = 0, n_tiles = 0;
    std::vector<int64_t> first_tile;  // [T+1] index of each tensor's first tile in the table
    cmn::WorkspaceLayout ws;

    // state set by cmn_plan_bind
    bool bound = false, have_grads = false, have_opt = false, have_mean = false, have_state2 = false, have_scales = false;
    char *dev_ws = nullptr;
    std::vector<unsigned char> staging;  // host image of the workspace

    // state of cmn_allreduce_step_noalloc: the pointer arrays of its last call on this plan, the table
    // image built from them, and a number that changes whenever the image does
    uint64_t serial = 0;                 // unique per plan created in this process (never reused)
    uint64_t image_generation = 0;
    std::vector<const void *> static_inputs;
    std::vector<unsigned char> static_image;
};

namespace cmn {

// Fills out[0..n_tiles) for the given pointer arrays (may be null: heads become -1).
void build_tiles(const cmn_plan &p, const void *const *grad_ptrs, void *const *param_ptrs,
                 void *const *vel_ptrs, void *const *mean_ptrs, void *const *state2_ptrs, cmn_tile *out);

// Shared argument checks of the kernel entry points.
int check_launch(const cmn_plan *p);

// Compute units of the current device (cached) and the kernel-choice rule measured on MI355X:
// the two-phase kernels win from K = 8 replicas on and lose for int8 storage.
// CMN_STEP_KERNEL=stream in the environment forces the one-pass kernels (A/B runs, tests).
int device_compute_units();
bool prefer_two_phase_reduce(const cmn_plan *p);
bool prefer_two_phase_step(const cmn_plan *p, int state_bytes_per_elem /* 8: p + velocity, 12: p + both Adam moments */,
                           int mean_dest);
bool state_first_step(const cmn_plan *p, int state_bytes_per_elem, int mean_dest);
int64_t two_phase_grid(const cmn_plan *p);
std::pair<int64_t, int64_t> two_phase_launches(const cmn_plan *p, int64_t n_tiles);   // (launches, tiles per launch)

// 1 (one pass), 3 (one pass, state first) or 2 (two-phase) for a fused-step launch over n_tiles tiles of this plan.
int fused_range_kernel_kind(const cmn_plan *p, bool adam, int mean_dest, int64_t n_tiles);

// Which tensor lists a table image holds.
struct BoundLists {
    bool grads, opt, mean, state2, scales;
};
inline BoundLists bound_lists(const cmn_plan *p) {
    return BoundLists{p->have_grads, p->have_opt, p->have_mean, p->have_state2, p->have_scales};
}

// Writes the plan's tables for these pointer arrays (each may be null) into img[0 .. ws.total):
// offsets, both gradient pointer tables, the [T] pointer tables, the scale pointers and the
// tile table.  Pure host work; throws std::bad_alloc only.
void fill_table_image(const cmn_plan *p, unsigned char *img, const void *const *grad_ptrs, void *const *param_ptrs,
                      void *const *vel_ptrs, void *const *mean_ptrs, void *const *state2_ptrs,
                      const float *const *scale_ptrs);

// Null / alignment check of a pointer array with `rows` rows of T entries (entries of empty tensors are ignored).
int check_ptr_array(const cmn_plan *p, const void *const *ptrs, int rows, unsigned elem_bytes);

template <typename T>
inline T *ws_ptr(const char *ws, size_t byte_off) {
    return reinterpret_cast<T *>(const_cast<char *>(ws) + byte_off);
}
template <typename T>
inline T *ws_ptr(const cmn_plan *p, size_t byte_off) {
    return ws_ptr<T>(p->dev_ws, byte_off);
}

}  // namespace cmn
