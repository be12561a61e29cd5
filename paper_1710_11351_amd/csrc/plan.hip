// Host side of libcmn: plan creation, geometry of the packed index space, the
// work-unit (tile) table of the tensor-space kernels, and binding of device
// tensors.  The geometry follows the contract stated at the top of cmn.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <new>

#include "plan.hpp"

namespace cmn {

static size_t round256(size_t x) { return (x + 255) & ~size_t(255); }

static WorkspaceLayout make_layout(int T, int K, int64_t n_tiles) {
    WorkspaceLayout w;
    size_t o = 0;
    w.off_table = o;  o = round256(o + sizeof(int64_t) * (size_t(T) + 1));
    w.grad_rows = o;  o = round256(o + sizeof(void *) * size_t(T) * size_t(K));
    w.grad_cols = o;  o = round256(o + sizeof(void *) * size_t(T) * size_t(K));
    w.param_ptrs = o; o = round256(o + sizeof(void *) * size_t(T));
    w.vel_ptrs = o;   o = round256(o + sizeof(void *) * size_t(T));
    w.mean_ptrs = o;  o = round256(o + sizeof(void *) * size_t(T));
    w.state2_ptrs = o; o = round256(o + sizeof(void *) * size_t(T));
    w.scale_ptrs = o;  o = round256(o + sizeof(void *) * size_t(K));
    w.tiles = o;      o = round256(o + sizeof(DeviceTile) * size_t(n_tiles));
    w.total = o < 256 ? 256 : o;
    return w;
}

// Walk the tiles in table order: tensors in list order, each tensor cut at ring-chunk
// edges (in packed coordinates) and at multiples of tile_elems (in tensor coordinates).
template <typename F>
static int64_t for_each_tile(const cmn_plan &p, F &&emit) {
    int64_t count = 0;
    if (p.chunk_elems == 0) return 0;
    for (int t = 0; t < p.T; ++t) {
        const int64_t n = p.numel[t], o = p.off[t];
        int64_t e = 0;
        while (e < n) {
            const int64_t c = (o + e) / p.chunk_elems;
            int64_t end = (c + 1) * p.chunk_elems - o;          // chunk edge, tensor coordinates
            if (end > n) end = n;
            const int64_t tile_end = (e / p.tile_elems + 1) * p.tile_elems;
            if (end > tile_end) end = tile_end;
            emit(t, e, int32_t(end - e), p.ring_rotate ? int32_t(c % p.K) : 0, int32_t(c));
            ++count;
            e = end;
        }
    }
    return count;
}

// Number of leading elements before element index 0 of a tensor reaches a 16-byte
// boundary on every stream, or -1 if the streams disagree.  `vec` is the vector width
// in elements of the narrowest stream (4 for float32, 8 for binary16 gradients).
static int common_head(const void *const *g, int n_g, int g_elem_bytes, int vec, const void *const *f32,
                       int n_f32) {
    int a = -1;
    for (int i = 0; i < n_g; ++i) {
        const uintptr_t idx = reinterpret_cast<uintptr_t>(g[i]) / unsigned(g_elem_bytes);
        const int ai = int((vec - int(idx % unsigned(vec))) % vec);
        if (a < 0) a = ai;
        else if (a != ai) return -1;
    }
    for (int i = 0; i < n_f32; ++i) {
        const uintptr_t idx = reinterpret_cast<uintptr_t>(f32[i]) / 4u;
        if (a < 0) a = int((vec - int(idx % unsigned(vec))) % vec);
        else if ((idx + unsigned(a)) % 4u != 0) return -1;
    }
    return a;
}

void build_tiles(const cmn_plan &p, const void *const *grad_ptrs, void *const *param_ptrs,
                 void *const *vel_ptrs, void *const *mean_ptrs, void *const *state2_ptrs, cmn_tile *out) {
    const int vec = vec_elems(p.dtype), geb = elem_bytes(p.dtype);
    std::vector<int8_t> h(size_t(p.T) * 8, int8_t(-1));   // per tensor: head of element 0 per variant
    std::vector<const void *> g(p.K);
    const bool opt = param_ptrs && vel_ptrs;
    for (int t = 0; t < p.T; ++t) {
        if (p.numel[t] == 0) continue;
        int8_t *ht = &h[size_t(t) * 8];
        const void *f32[5];
        if (grad_ptrs && opt) {
            for (int k = 0; k < p.K; ++k) g[k] = grad_ptrs[size_t(k) * p.T + t];
            f32[0] = param_ptrs[t]; f32[1] = vel_ptrs[t];
            ht[CMN_HEAD_STEP] = int8_t(common_head(g.data(), p.K, geb, vec, f32, 2));
            if (mean_ptrs) {
                f32[2] = mean_ptrs[t];
                ht[CMN_HEAD_STEP_MEAN] = int8_t(common_head(g.data(), p.K, geb, vec, f32, 3));
            }
            if (state2_ptrs) {
                f32[2] = state2_ptrs[t];
                ht[CMN_HEAD_ADAM] = int8_t(common_head(g.data(), p.K, geb, vec, f32, 3));
                if (mean_ptrs) {
                    f32[3] = mean_ptrs[t];
                    ht[CMN_HEAD_ADAM_MEAN] = int8_t(common_head(g.data(), p.K, geb, vec, f32, 4));
                }
            }
        }
        if (mean_ptrs && opt) {
            f32[0] = mean_ptrs[t]; f32[1] = param_ptrs[t]; f32[2] = vel_ptrs[t];
            ht[CMN_HEAD_SGD] = int8_t(common_head(nullptr, 0, 4, 4, f32, 3));
            if (state2_ptrs) {
                f32[3] = state2_ptrs[t];
                ht[CMN_HEAD_ADAM_OPT] = int8_t(common_head(nullptr, 0, 4, 4, f32, 4));
            }
        }
    }
    int64_t i = 0;
    for_each_tile(p, [&](int t, int64_t e0, int32_t len, int32_t start, int32_t chunk) {
        cmn_tile &tl = out[i++];
        tl.e0 = e0; tl.len = len; tl.tensor = t; tl.start_rank = start; tl.chunk = chunk;
        for (int v = 0; v < 8; ++v) {
            const int a = h[size_t(t) * 8 + v];
            const int w = (v == CMN_HEAD_SGD || v == CMN_HEAD_ADAM_OPT) ? 4 : vec;
            tl.head[v] = a < 0 ? int8_t(-1) : int8_t(((a - e0) % w + w) % w);
        }
    });
}

int device_compute_units() {
    static const int cached = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            return cus;
        return 256;
    }();
    return cached;
}

// Workgroups of a two-phase launch: two per compute unit (256 VGPRs each), fewer on request.
int64_t two_phase_grid(const cmn_plan *p) {
    const int64_t resident = int64_t(2) * device_compute_units();
    return p->grid_limit > 0 && p->grid_limit < resident ? p->grid_limit : resident;
}

// Which kernel serves a plan.  The two-phase kernels need one vector per thread and tile and
// are not built for int8 storage (its decode arithmetic wants the one-pass kernel's occupancy).
// Where both kinds apply the choice follows measurements on MI355X:
//  - ring reduce: two-phase from 8 replicas on;
//  - fused step: the stores of p and the optimizer state disturb the gradient reads less while
//    they end in the 256 MB memory-side cache, so with cache-resident state (ResNet-50 with
//    MomentumSGD, 204 MB) the one-pass kernel stays ahead until the replicas deliver about 44
//    bytes per element (fp32: 11 replicas, 16-bit: 22; cache-swept launches, K = 10: 232 vs
//    235 us, K = 11: 252 vs 244, K = 13: 290 vs 265; the same with Adam, 306 MB: K = 9: 250 vs
//    260, K = 11: 289 vs 281; 50 M elements, 400 MB: K = 8: 390 vs 408); with state beyond twice
//    the cache (75 M elements and more, VGG-16) the two-phase kernel wins from about 32 bytes
//    per element (K = 8: 633 vs 613 us), and likewise when the average is written back to all K
//    replicas.
static bool two_phase_possible(const cmn_plan *p) {
    return p->step_mode != STEP_ONE_PASS && p->dtype != CMN_I8S && p->tile_elems == kBlock * vec_elems(p->dtype);
}
bool prefer_two_phase_reduce(const cmn_plan *p) {
    return two_phase_possible(p) && (p->step_mode == STEP_TWO_PHASE || p->K >= 8);
}
bool prefer_two_phase_step(const cmn_plan *p, int state_bytes_per_elem, int mean_dest) {
    if (!two_phase_possible(p)) return false;
    if (p->step_mode == STEP_TWO_PHASE) return true;
    const bool cached = !beyond_cache(double(p->N) * state_bytes_per_elem);
    const bool light_stores = cached && mean_dest != CMN_MEAN_TO_ALL_REPLICAS;
    return p->K * elem_bytes(p->dtype) >= (light_stores ? 44 : 32);
}

// Few fp32 replicas, the average stored at most once, state that stays in the memory-side cache: the one-pass
// kernel that requests parameters and state ahead of the gradients (see k_step_state_first).
bool state_first_step(const cmn_plan *p, int state_bytes_per_elem, int mean_dest) {
    return p->dtype == CMN_F32 && p->K <= kStateFirstReplicas && mean_dest != CMN_MEAN_TO_ALL_REPLICAS &&
           !beyond_cache(double(p->N) * state_bytes_per_elem);
}

int check_ptr_array(const cmn_plan *p, const void *const *ptrs, int rows, unsigned elem_bytes) {
    for (int r = 0; r < rows; ++r)
        for (int t = 0; t < p->T; ++t) {
            if (p->numel[t] == 0) continue;
            const void *q = ptrs[size_t(r) * p->T + t];
            if (!q) return CMN_ENULL;
            if (reinterpret_cast<uintptr_t>(q) % elem_bytes) return CMN_EALIGN;
        }
    return CMN_OK;
}

// Rebuild the tile table inside a table image from the pointer tables the image holds.
static void fill_tile_table(const cmn_plan *p, unsigned char *img, const BoundLists &have) {
    auto tab = [&](size_t off) { return reinterpret_cast<void *const *>(img + off); };
    const void *const *gp = have.grads ? reinterpret_cast<const void *const *>(img + p->ws.grad_rows) : nullptr;
    void *const *pp = have.opt ? tab(p->ws.param_ptrs) : nullptr, *const *vp = have.opt ? tab(p->ws.vel_ptrs) : nullptr;
    void *const *mp = have.mean ? tab(p->ws.mean_ptrs) : nullptr, *const *sp = have.state2 ? tab(p->ws.state2_ptrs) : nullptr;
    std::vector<cmn_tile> table(size_t(p->n_tiles));
    build_tiles(*p, gp, pp, vp, mp, sp, table.data());
    DeviceTile *out = reinterpret_cast<DeviceTile *>(img + p->ws.tiles);
    auto at = [](void *const *base, const cmn_tile &tl) {
        return base ? static_cast<float *>(base[tl.tensor]) + tl.e0 : nullptr;
    };
    for (size_t i = 0; i < table.size(); ++i) {
        const cmn_tile &tl = table[i];
        DeviceTile &d = out[i];
        d.p = at(pp, tl); d.s1 = at(vp, tl); d.s2 = at(sp, tl); d.m = at(mp, tl);
        d.e0 = tl.e0; d.len = tl.len; d.tensor = tl.tensor; d.start_rank = tl.start_rank; d.chunk = tl.chunk;
        std::memcpy(d.head, tl.head, sizeof d.head);
    }
}

void fill_table_image(const cmn_plan *p, unsigned char *img, const void *const *grad_ptrs, void *const *param_ptrs,
                      void *const *vel_ptrs, void *const *mean_ptrs, void *const *state2_ptrs,
                      const float *const *scale_ptrs) {
    std::memset(img, 0, p->ws.total);
    std::memcpy(img + p->ws.off_table, p->off.data(), sizeof(int64_t) * (size_t(p->T) + 1));
    const size_t T = size_t(p->T), K = size_t(p->K);
    if (grad_ptrs) {
        auto **rows = reinterpret_cast<const void **>(img + p->ws.grad_rows);
        auto **cols = reinterpret_cast<const void **>(img + p->ws.grad_cols);
        for (size_t k = 0; k < K; ++k)
            for (size_t t = 0; t < T; ++t) {
                rows[k * T + t] = grad_ptrs[k * T + t];
                cols[t * K + k] = grad_ptrs[k * T + t];
            }
    }
    if (param_ptrs) std::memcpy(img + p->ws.param_ptrs, param_ptrs, sizeof(void *) * T);
    if (vel_ptrs) std::memcpy(img + p->ws.vel_ptrs, vel_ptrs, sizeof(void *) * T);
    if (mean_ptrs) std::memcpy(img + p->ws.mean_ptrs, mean_ptrs, sizeof(void *) * T);
    if (state2_ptrs) std::memcpy(img + p->ws.state2_ptrs, state2_ptrs, sizeof(void *) * T);
    if (scale_ptrs) std::memcpy(img + p->ws.scale_ptrs, scale_ptrs, sizeof(void *) * K);
    fill_tile_table(p, img, BoundLists{grad_ptrs != nullptr, param_ptrs && vel_ptrs, mean_ptrs != nullptr,
                                       state2_ptrs != nullptr, scale_ptrs != nullptr});
}

int fused_range_kernel_kind(const cmn_plan *p, bool adam, int mean_dest, int64_t n_tiles) {
    if (prefer_two_phase_step(p, adam ? 12 : 8, mean_dest) && (n_tiles >= kMinTwoPhaseTiles || p->step_mode == STEP_TWO_PHASE))
        return 2;
    return state_first_step(p, adam ? 12 : 8, mean_dest) ? 3 : 1;
}

// One launch of a two-phase kernel covers at most one round of the persistent grid (a kernel
// boundary realigns the workgroups' phases, which rounds drifting inside one launch would lose:
// VGG-16, 5.3 rounds: 1931 us in one launch, 1830 us in six).  Returns the number of launches
// for n_tiles tiles and the tiles per launch, spread evenly.
std::pair<int64_t, int64_t> two_phase_launches(const cmn_plan *p, int64_t n_tiles) {
    const int64_t slots = two_phase_grid(p) * (kStashFloats / vec_elems(p->dtype));
    const int64_t n_launch = (n_tiles + slots - 1) / slots;
    return {n_launch, n_launch ? (n_tiles + n_launch - 1) / n_launch : 0};
}

int check_launch(const cmn_plan *p) {
    if (!p) return CMN_ENULL;
    if (!p->bound) return CMN_EUNBOUND;
    return CMN_OK;
}

}  // namespace cmn

using namespace cmn;

extern "C" {

int cmn_plan_create(cmn_plan **out, int n_tensors, const int64_t *numel, int K, int n_chunks,
                    int align_bytes, int grad_dtype, int ring_rotate) {
    if (!out) return CMN_ENULL;
    *out = nullptr;
    if (n_tensors < 0 || K < 1 || n_chunks < 1) return CMN_EINVAL;
    if (n_tensors > 0 && !numel) return CMN_ENULL;
    if (grad_dtype < CMN_F32 || grad_dtype > CMN_I8S) return CMN_EINVAL;
    if (ring_rotate != 0 && ring_rotate != 1) return CMN_EINVAL;
    if (align_bytes < 16 || (align_bytes & (align_bytes - 1)) != 0) return CMN_EINVAL;
    if (n_tensors > kMaxTensors || K > kMaxReplicas || align_bytes > (1 << 20)) return CMN_ESIZE;

    cmn_plan *p = new (std::nothrow) cmn_plan;
    if (!p) return CMN_ENOMEM;
    static std::atomic<uint64_t> next_serial{1};
    p->serial = next_serial.fetch_add(1);
    try {
        p->T = n_tensors; p->K = K; p->C = n_chunks; p->align_bytes = align_bytes;
        p->dtype = grad_dtype; p->ring_rotate = ring_rotate;
        p->numel.assign(numel, numel + n_tensors);
        p->off.assign(size_t(n_tensors) + 1, 0);
    } catch (...) { delete p; return CMN_ENOMEM; }

    const int64_t kMaxElems = int64_t(1) << 46;  // keeps every byte offset far inside int64
    for (int t = 0; t < n_tensors; ++t) {
        if (numel[t] < 0) { delete p; return CMN_EINVAL; }
        if (numel[t] > kMaxElems || p->off[t] > kMaxElems) { delete p; return CMN_ESIZE; }
        p->off[t + 1] = p->off[t] + numel[t];
    }
    p->N = p->off[n_tensors];
    const int64_t A = align_bytes / elem_bytes(grad_dtype);
    const int64_t per = (p->N + n_chunks - 1) / n_chunks;
    p->chunk_elems = (per + A - 1) / A * A;
    p->L = p->chunk_elems * n_chunks;
    if (p->L > kMaxElems || p->L * K > (int64_t(1) << 50)) { delete p; return CMN_ESIZE; }

    p->tile_elems = kBlock * vec_elems(grad_dtype) * kTileIters;
    if (const char *k = std::getenv("CMN_STEP_KERNEL"))
        p->step_mode = std::strcmp(k, "stream") == 0 ? STEP_ONE_PASS : std::strcmp(k, "two_phase") == 0 ? STEP_TWO_PHASE : STEP_AUTO;
    if (const char *k = std::getenv("CMN_TWO_PHASE_GRID")) p->grid_limit = std::atoi(k) > 0 ? std::atoi(k) : 0;
    try {
        p->first_tile.assign(size_t(n_tensors) + 1, 0);
    } catch (...) { delete p; return CMN_ENOMEM; }
    {
        std::vector<int64_t> &ft = p->first_tile;
        p->n_tiles = for_each_tile(*p, [&ft](int t, int64_t, int32_t, int32_t, int32_t) { ++ft[size_t(t) + 1]; });
        for (int t = 0; t < n_tensors; ++t) ft[size_t(t) + 1] += ft[size_t(t)];
    }
    if (p->n_tiles > (int64_t(1) << 31) - 1) { delete p; return CMN_ESIZE; }
    p->ws = make_layout(p->T, p->K, p->n_tiles);
    *out = p;
    return CMN_OK;
}

int cmn_plan_destroy(cmn_plan *plan) {
    delete plan;
    return CMN_OK;
}

int64_t cmn_plan_total_elems(const cmn_plan *p) { return p ? p->N : -1; }
int64_t cmn_plan_padded_elems(const cmn_plan *p) { return p ? p->L : -1; }
int64_t cmn_plan_chunk_elems(const cmn_plan *p) { return p ? p->chunk_elems : -1; }
int64_t cmn_plan_tile_count(const cmn_plan *p) { return p ? p->n_tiles : -1; }
int cmn_plan_step_kernel_kind(const cmn_plan *p, int adam, int mean_dest) {
    return p ? fused_range_kernel_kind(p, adam != 0, mean_dest, p->n_tiles) : -1;
}
int cmn_plan_range_kernel_kind(const cmn_plan *p, int tensor_begin, int tensor_end, int adam, int mean_dest) {
    if (!p || tensor_begin < 0 || tensor_end < tensor_begin || tensor_end > p->T) return -1;
    return fused_range_kernel_kind(p, adam != 0, mean_dest,
                                   p->first_tile[size_t(tensor_end)] - p->first_tile[size_t(tensor_begin)]);
}
int cmn_plan_range_launch_count(const cmn_plan *p, int tensor_begin, int tensor_end, int adam, int mean_dest) {
    if (!p || tensor_begin < 0 || tensor_end < tensor_begin || tensor_end > p->T) return -1;
    const int64_t n = p->first_tile[size_t(tensor_end)] - p->first_tile[size_t(tensor_begin)];
    if (n == 0) return 0;
    if (fused_range_kernel_kind(p, adam != 0, mean_dest, n) != 2) return 1;
    return int(two_phase_launches(p, n).first);
}
size_t cmn_plan_workspace_bytes(const cmn_plan *p) { return p ? p->ws.total : 0; }

int cmn_plan_describe_tiles(const cmn_plan *plan, const void *const *grad_ptrs, void *const *param_ptrs,
                            void *const *vel_ptrs, void *const *mean_grad_ptrs, void *const *second_moment_ptrs,
                            cmn_tile *tiles) {
    if (!plan || (!tiles && plan->n_tiles > 0)) return CMN_ENULL;
    int rc;
    if (grad_ptrs && (rc = check_ptr_array(plan, grad_ptrs, plan->K, elem_bytes(plan->dtype)))) return rc;
    if (param_ptrs && (rc = check_ptr_array(plan, param_ptrs, 1, 4))) return rc;
    if (vel_ptrs && (rc = check_ptr_array(plan, vel_ptrs, 1, 4))) return rc;
    if (mean_grad_ptrs && (rc = check_ptr_array(plan, mean_grad_ptrs, 1, 4))) return rc;
    if (second_moment_ptrs && (rc = check_ptr_array(plan, second_moment_ptrs, 1, 4))) return rc;
    try {
        build_tiles(*plan, grad_ptrs, param_ptrs, vel_ptrs, mean_grad_ptrs, second_moment_ptrs, tiles);
    } catch (...) { return CMN_ENOMEM; }
    return CMN_OK;
}

// Copy the staging image to the device workspace and wait for the copy: the image is pageable
// host memory that the next bind call rewrites.
static int upload_image(cmn_plan *p, void *dev_workspace, hipStream_t s) {
    if (hipMemcpyAsync(dev_workspace, p->staging.data(), p->ws.total, hipMemcpyHostToDevice, s) != hipSuccess) return CMN_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return CMN_EHIP;
    return CMN_OK;
}

int cmn_plan_bind(cmn_plan *plan, void *dev_workspace, const void *const *grad_ptrs, void *const *param_ptrs,
                  void *const *vel_ptrs, void *const *mean_grad_ptrs, void *stream) {
    if (!plan || !dev_workspace) return CMN_ENULL;
    if (reinterpret_cast<uintptr_t>(dev_workspace) % 256) return CMN_EALIGN;
    if ((param_ptrs == nullptr) != (vel_ptrs == nullptr)) return CMN_ENULL;
    cmn_plan *p = plan;
    int rc;
    if (grad_ptrs && (rc = check_ptr_array(p, grad_ptrs, p->K, elem_bytes(p->dtype)))) return rc;
    if (param_ptrs && (rc = check_ptr_array(p, param_ptrs, 1, 4))) return rc;
    if (vel_ptrs && (rc = check_ptr_array(p, vel_ptrs, 1, 4))) return rc;
    if (mean_grad_ptrs && (rc = check_ptr_array(p, mean_grad_ptrs, 1, 4))) return rc;

    p->bound = false;
    try {
        p->staging.resize(p->ws.total);
        fill_table_image(p, p->staging.data(), grad_ptrs, param_ptrs, vel_ptrs, mean_grad_ptrs, nullptr, nullptr);
    } catch (...) { return CMN_ENOMEM; }
    p->have_grads = grad_ptrs != nullptr;
    p->have_opt = param_ptrs != nullptr;
    p->have_mean = mean_grad_ptrs != nullptr;
    p->have_state2 = false;          // a new binding starts without Adam moments and int8 scales
    p->have_scales = false;
    if (int rc2 = upload_image(p, dev_workspace, static_cast<hipStream_t>(stream))) return rc2;
    p->dev_ws = static_cast<char *>(dev_workspace);
    p->bound = true;
    return CMN_OK;
}

int cmn_plan_bind_adam(cmn_plan *plan, void *const *second_moment_ptrs, void *stream) {
    if (!plan || !second_moment_ptrs) return CMN_ENULL;
    if (!plan->bound || !plan->have_opt) return CMN_EUNBOUND;
    if (int rc = check_ptr_array(plan, second_moment_ptrs, 1, 4)) return rc;
    std::memcpy(plan->staging.data() + plan->ws.state2_ptrs, second_moment_ptrs, sizeof(void *) * size_t(plan->T));
    plan->have_state2 = true;
    plan->bound = false;
    try {
        fill_tile_table(plan, plan->staging.data(), bound_lists(plan));
    } catch (...) { return CMN_ENOMEM; }
    if (int rc = upload_image(plan, plan->dev_ws, static_cast<hipStream_t>(stream))) return rc;
    plan->bound = true;
    return CMN_OK;
}

int cmn_plan_bind_scales(cmn_plan *plan, const float *const *scale_ptrs, void *stream) {
    if (!plan || !scale_ptrs) return CMN_ENULL;
    if (plan->dtype != CMN_I8S) return CMN_EINVAL;
    if (!plan->bound) return CMN_EUNBOUND;
    for (int k = 0; k < plan->K; ++k) {
        if (!scale_ptrs[k]) return CMN_ENULL;
        if (reinterpret_cast<uintptr_t>(scale_ptrs[k]) % 4) return CMN_EALIGN;
    }
    std::memcpy(plan->staging.data() + plan->ws.scale_ptrs, scale_ptrs, sizeof(void *) * size_t(plan->K));
    plan->have_scales = true;
    plan->bound = false;
    if (int rc = upload_image(plan, plan->dev_ws, static_cast<hipStream_t>(stream))) return rc;
    plan->bound = true;
    return CMN_OK;
}

const char *cmn_strerror(int status) {
    switch (status) {
        case CMN_OK: return "ok";
        case CMN_EINVAL: return "invalid argument";
        case CMN_ENULL: return "required pointer is NULL";
        case CMN_ESIZE: return "size exceeds the supported maximum";
        case CMN_EALIGN: return "buffer is not sufficiently aligned";
        case CMN_EUNBOUND: return "plan is not bound to the tensors this call needs";
        case CMN_EHIP: return "HIP runtime error";
        case CMN_ENOMEM: return "out of host memory";
        default: return "unknown status";
    }
}

}  // extern "C"
