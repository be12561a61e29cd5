/*
 * cmn.h — C-ABI of libcmn: the per-iteration gradient aggregation + update of
 * synchronous data-parallel training on one MI355X (gfx950).
 *
 * What is computed (ChainerMN paper, Section 2.3, "Allreduce" and
 * "optimization" steps of an iteration; Section 3.3, the multi-node optimizer
 * that exchanges gradients and then runs the wrapped optimizer; Section 2.1,
 * the update rule):  K worker replicas each hold one gradient tensor per
 * parameter tensor.  The step forms the element-wise average over the K
 * replicas and updates the single shared copy of parameters with it.
 * All K replicas' gradients are resident on the one GPU; the K-way reduction is
 * the arithmetic every rank of an allreduce performs on its share.
 *
 * The order of the K-term float32 sum is fixed and part of the contract:
 * the tightly packed concatenation of all tensors (length N) is cut into
 * n_chunks equal chunks (each rounded up to align_bytes; only [N, L) is
 * padding), and element i of chunk c is summed as
 *     ((g[r0] + g[r1]) + g[r2]) + ... ,   r_j = (s + j) mod K,
 * with s = c mod K if ring_rotate (the order an ascending-rank ring
 * reduce-scatter produces) or s = 0 otherwise.
 *
 * Conventions for every function:
 *  - returns CMN_OK (0) or a negative cmn_status; never throws, never aborts;
 *  - pointers marked "host" are host memory read during the call only;
 *    pointers marked "device" are device memory owned by the caller, which must
 *    stay valid until the work queued on `stream` has finished;
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream);
 *    kernel entry points only enqueue work and do not synchronise;
 *  - the library never allocates or frees device memory;
 *  - a plan may be used by one host thread at a time;
 *  - gradients are read-only (except under CMN_MEAN_TO_ALL_REPLICAS); parameters,
 *    velocities and Adam moments are updated in place;
 *    parameters, velocities, mean gradients and all sums are float32;
 *  - no tensor may overlap another, except that mean_grad_ptrs[t] may equal
 *    replica 0's gradient tensor grad_ptrs[t] when grad_dtype is CMN_F32.
 */
#ifndef CMN_H_
#define CMN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cmn_plan cmn_plan; /* opaque; host memory owned by the library */

enum cmn_status {
    CMN_OK = 0,
    CMN_EINVAL = -1,   /* an argument is out of range                              */
    CMN_ENULL = -2,    /* a required pointer is NULL                                */
    CMN_ESIZE = -3,    /* a size exceeds what the library supports                  */
    CMN_EALIGN = -4,   /* a buffer that must be aligned is not                      */
    CMN_EUNBOUND = -5, /* a kernel entry point was called before cmn_plan_bind      */
    CMN_EHIP = -6,     /* the HIP runtime reported an error                         */
    CMN_ENOMEM = -7    /* host memory could not be obtained                         */
};

enum cmn_dtype {
    CMN_F32 = 0, /* gradients stored as IEEE binary32 */
    CMN_F16 = 1, /* gradients stored as IEEE binary16, decoded exactly and summed in binary32 */
    CMN_BF16 = 2, /* gradients stored as bfloat16 (upper half of a binary32), same treatment  */
    CMN_I8S = 3   /* gradients stored as int8 with one float32 scale per (replica, ring chunk):
                     value = (float)q * scale, the product rounded once, summed in binary32;
                     scales are bound with cmn_plan_bind_scales                               */
};

/* Where a fused step puts the averaged gradient. */
enum cmn_mean_dest {
    CMN_MEAN_NONE = 0,            /* nowhere: only p and the optimizer state are written      */
    CMN_MEAN_TO_MEAN_GRADS = 1,   /* into the bound mean_grad_ptrs (float32)                   */
    CMN_MEAN_TO_ALL_REPLICAS = 2  /* over every replica's own gradient tensors, i.e. the half of
                                     an allreduce that hands the result to every worker;
                                     rounded to nearest even when gradients are 16-bit        */
};

/* Which streams a kernel variant touches; index into cmn_tile.head. */
enum cmn_head_index {
    CMN_HEAD_STEP = 0,       /* K gradients, p, v                      (fused MomentumSGD)     */
    CMN_HEAD_STEP_MEAN = 1,  /* ... plus mean gradient                                          */
    CMN_HEAD_SGD = 2,        /* mean gradient, p, v                    (cmn_momentum_sgd)      */
    CMN_HEAD_ADAM = 3,       /* K gradients, p, m, v                   (fused Adam)            */
    CMN_HEAD_ADAM_MEAN = 4,  /* ... plus mean gradient                                          */
    CMN_HEAD_ADAM_OPT = 5    /* mean gradient, p, m, v                 (cmn_adam)              */
};

/* One unit of work of the tensor-space kernels: `len` consecutive elements of tensor
 * `tensor` starting at element `e0`, all inside one ring chunk whose sum starts at replica
 * `start_rank`.  head[i] is the number of leading elements handled one by one before the
 * first 16-byte aligned vector of every stream variant i touches, or -1 when those streams
 * have no common alignment (or are not bound) and the whole tile is processed element by
 * element.  Exposed for inspection only. */
typedef struct cmn_tile {
    int64_t e0;
    int32_t len;
    int32_t tensor;
    int32_t start_rank;
    int32_t chunk;          /* index of that ring chunk (selects the scale of int8 gradients) */
    int8_t head[8];
} cmn_tile;

/* The plan object, its chunk geometry and its tables are not in the paper: they are this build's
 * way of fixing the summation order and of finding K*T scattered tensors from a kernel.
 * Create a plan for `n_tensors` tensors of numel[t] >= 0 elements (host array, copied),
 * K >= 1 replicas, n_chunks >= 1 ring chunks, align_bytes a power of two that is a
 * multiple of 16 (256 in every published workload), grad_dtype a cmn_dtype, and
 * ring_rotate 0 or 1.  n_tensors may be 0 and tensors may be empty.  Pure host work.
 * Two environment variables are read here (launch shape only, results never change):
 * CMN_STEP_KERNEL=stream | two_phase forces the one-pass / the persistent two-phase kernels
 * wherever that kind exists, and CMN_TWO_PHASE_GRID=n caps the persistent grid at n workgroups.
 * Errors: CMN_ENULL (out, or numel with n_tensors > 0), CMN_EINVAL, CMN_ESIZE
 * (n_tensors or K above the supported maximum, or sizes that overflow), CMN_ENOMEM. */
int cmn_plan_create(cmn_plan **out, int n_tensors, const int64_t *numel /* host [T] */, int K,
                    int n_chunks, int align_bytes, int grad_dtype, int ring_rotate);

/* Free the plan's host memory.  NULL is accepted.  Device buffers are the caller's. */
int cmn_plan_destroy(cmn_plan *plan);

int64_t cmn_plan_total_elems(const cmn_plan *plan);  /* N = sum of numel; -1 if plan is NULL      */
int64_t cmn_plan_padded_elems(const cmn_plan *plan); /* L = n_chunks * chunk_elems                */
int64_t cmn_plan_chunk_elems(const cmn_plan *plan);  /* roundup(ceil(N / n_chunks), align_bytes)  */
int64_t cmn_plan_tile_count(const cmn_plan *plan);   /* number of cmn_tile work units             */
size_t cmn_plan_workspace_bytes(const cmn_plan *plan); /* device bytes cmn_plan_bind needs (>= 256) */
/* Which kernel kind the fused step launches for this plan with MomentumSGD (adam == 0) or Adam
 * (adam != 0) and the given cmn_mean_dest, over the whole list or over tensors
 * [tensor_begin, tensor_end): a tuning decision that never changes results; for benchmarks and
 * profiles.  1 = one pass, a workgroup per tile; 2 = persistent grid that reads first and
 * writes afterwards (small lists and layer groups use kind 1); 3 = kind 1 with parameters and
 * state requested ahead of the gradients (at most 4 float32 replicas); -1 if plan is NULL or
 * the range is not inside the list. */
int cmn_plan_step_kernel_kind(const cmn_plan *plan, int adam, int mean_dest);
int cmn_plan_range_kernel_kind(const cmn_plan *plan, int tensor_begin, int tensor_end, int adam, int mean_dest);
/* Number of kernel launches that fused step makes (kind 2 takes one launch per round of its
 * persistent grid; 0 for an empty range, -1 as above). */
int cmn_plan_range_launch_count(const cmn_plan *plan, int tensor_begin, int tensor_end, int adam, int mean_dest);

/* Pure host: compute the work-unit table that cmn_plan_bind would upload for these
 * pointer arrays (same meaning as in cmn_plan_bind; addresses are only inspected,
 * never dereferenced) into tiles[0 .. cmn_plan_tile_count).  For tests and tooling. */
int cmn_plan_describe_tiles(const cmn_plan *plan, const void *const *grad_ptrs, void *const *param_ptrs,
                            void *const *vel_ptrs, void *const *mean_grad_ptrs,
                            void *const *second_moment_ptrs /* as cmn_plan_bind_adam, or NULL */,
                            cmn_tile *tiles /* host */);

/* Bind device tensors to the plan and upload the plan's tables into `dev_workspace`
 * (device, 256-byte aligned, cmn_plan_workspace_bytes long; must outlive all later
 * calls on this plan).  grad_ptrs is a host array of K*T device pointers, replica-major
 * (grad_ptrs[k*T + t], element type grad_dtype, numel[t] elements, aligned to the
 * element size); param_ptrs / vel_ptrs / mean_grad_ptrs are host arrays of T device
 * float32 pointers (4-byte aligned).  Any of the four arrays may be NULL (param_ptrs and
 * vel_ptrs only together); an entry point that needs an array that was not bound returns
 * CMN_EUNBOUND: cmn_pack needs gradients, cmn_scale_unpack mean gradients,
 * cmn_momentum_sgd mean gradients + parameters + velocities, cmn_allreduce_step gradients
 * + parameters + velocities (+ mean gradients if asked to write them).  Pointers of empty
 * tensors are ignored.  The call waits for `stream` before it returns (set-up, not the hot
 * path: its tables travel from pageable host memory).  May be repeated to rebind; every bind
 * starts afresh, so Adam's second moments (cmn_plan_bind_adam) and int8 scales
 * (cmn_plan_bind_scales) of an earlier binding are dropped and must be bound again.
 * Errors: CMN_ENULL, CMN_EALIGN, CMN_EHIP. */
int cmn_plan_bind(cmn_plan *plan, void *dev_workspace, const void *const *grad_ptrs /* host [K*T] */,
                  void *const *param_ptrs /* host [T] */, void *const *vel_ptrs /* host [T] */,
                  void *const *mean_grad_ptrs /* host [T] or NULL */, void *stream);

/* S1 pack.  Not in the paper, which only says that gradients exist per parameter tensor
 * (Section 2.1) and are exchanged by Allreduce (Section 2.3); the contiguous buffer and its
 * chunking are this build's design.  For every replica k copy its T gradient tensors in list
 * order, with no gaps, to packed[k*L .. k*L + N) and write zeros to packed[k*L + N .. (k+1)*L).
 * packed: device, K*L elements of grad_dtype, 256-byte aligned.  Bit copy. */
int cmn_pack(const cmn_plan *plan, void *packed /* device [K][L] */, void *stream);

/* S2 ring-order reduction (the arithmetic share of the paper's Allreduce step, Section 2.3; the
 * ring order is this build's reading, see the top of this file).  reduced[i] = fixed-order
 * float32 sum over k of packed[k][i].  packed as written by cmn_pack; reduced: device, L float32,
 * 256-byte aligned, must not overlap packed.  Works on the two buffers alone: the plan need not
 * be bound (only a CMN_I8S plan must be, with scales: CMN_EUNBOUND otherwise). */
int cmn_ring_reduce(const cmn_plan *plan, const void *packed /* device [K][L] */,
                    float *reduced /* device [L] */, void *stream);

/* S3 + S4 scale and unpack: the sum becomes the average that Section 2.3 says every worker
 * obtains; how it is laid out is not in the paper (this build's design, like cmn_pack).
 * mean_grad[t][e] = reduced[off[t] + e] * (1.0f / (float)K) for every tensor; padding is
 * dropped.  Needs mean_grad_ptrs bound. */
int cmn_scale_unpack(const cmn_plan *plan, const float *reduced /* device [L] */, void *stream);

/* S5 MomentumSGD on every element, reading the bound mean gradients g:
 *     g' = g + wd * p   (skipped when wd == 0);   v = mu * v - lr * g';   p = p + v
 * each operation rounded to float32 once (no fused multiply-add).  lr is the learning
 * rate (written mu in the paper's Section 2.1), mu the momentum coefficient. */
int cmn_momentum_sgd(const cmn_plan *plan, float lr, float mu, float wd, void *stream);

/* S1..S5 fused into one pass over HBM with no intermediate buffer (one kernel launch for
 * lists up to about 26 M elements, a few back-to-back launches beyond): for every element
 * read the K replicas' gradients in the fixed order, sum, multiply by 1.0f/(float)K,
 * apply the MomentumSGD rule above to p and v in place, and put the averaged gradient
 * where mean_dest (a cmn_mean_dest; 0 and 1 keep the meaning of a boolean) says.
 * With CMN_MEAN_TO_ALL_REPLICAS the bound gradient tensors are overwritten.  Results are
 * identical, bit for bit, to cmn_pack -> cmn_ring_reduce -> cmn_scale_unpack ->
 * cmn_momentum_sgd. */
int cmn_allreduce_step(const cmn_plan *plan, float lr, float mu, float wd, int mean_dest, void *stream);

/* The same step restricted to tensors [tensor_begin, tensor_end) of the list: the unit a
 * training loop launches per layer group as soon as that group's gradients exist (the
 * building block for overlapping the exchange with the backward pass, which the paper's
 * conclusions name as future work).  Ring chunks and fold order are those of the whole list,
 * so stepping every tensor once, in any grouping and order, equals one cmn_allreduce_step.
 * Errors: CMN_EINVAL unless 0 <= tensor_begin <= tensor_end <= n_tensors. */
int cmn_allreduce_step_range(const cmn_plan *plan, int tensor_begin, int tensor_end, float lr, float mu,
                             float wd, int mean_dest, void *stream);

/* Bind the second-moment tensors of Adam (host array of T device float32 pointers).  The
 * first moment lives in the tensors bound as vel_ptrs.  Call after cmn_plan_bind (which must
 * have bound parameters); re-uploads the plan's tables and waits for `stream`. */
int cmn_plan_bind_adam(cmn_plan *plan, void *const *second_moment_ptrs /* host [T] */, void *stream);

/* Bind the scales of CMN_I8S gradients: host array of K device pointers, scale_ptrs[k] ->
 * n_chunks float32 values, element c scaling every element of replica k whose packed index
 * lies in ring chunk c.  The scale arrays are read by every later launch (they may be
 * rewritten between launches).  Call after cmn_plan_bind; re-uploads the tables and waits
 * for `stream`.  cmn_ring_reduce and the fused steps return CMN_EUNBOUND for a CMN_I8S plan
 * without scales, and CMN_EINVAL for CMN_MEAN_TO_ALL_REPLICAS (re-quantising the average is
 * not defined).  Errors: CMN_ENULL, CMN_EALIGN, CMN_EINVAL (plan is not CMN_I8S). */
int cmn_plan_bind_scales(cmn_plan *plan, const float *const *scale_ptrs /* host [K] */, void *stream);

/* Fused step with Adam in place of MomentumSGD (the optimizer the paper's Listing 1 wraps;
 * Section 3.3: the multi-node optimizer behaves like the optimizer it wraps).  Per element,
 * with g the averaged gradient and t >= 1 the iteration number:
 *     g' = g + wd * p                       (skipped when wd == 0)
 *     m  = m + (1 - beta1) * (g' - m)
 *     v  = v + (1 - beta2) * (g'*g' - v)
 *     p  = p - lr_t * m / (sqrt(v) + eps),  lr_t = alpha * sqrt(1 - beta2^t) / (1 - beta1^t)
 * each operation rounded to float32 once, sqrt and division correctly rounded; lr_t is formed
 * in double on the host and rounded once.  Errors as cmn_allreduce_step, CMN_EINVAL if t < 1,
 * CMN_EUNBOUND without cmn_plan_bind_adam. */
int cmn_allreduce_adam_step(const cmn_plan *plan, float alpha, float beta1, float beta2, float eps, float wd,
                            int t, int mean_dest, void *stream);
int cmn_allreduce_adam_step_range(const cmn_plan *plan, int tensor_begin, int tensor_end, float alpha,
                                  float beta1, float beta2, float eps, float wd, int t, int mean_dest,
                                  void *stream);

/* Adam on its own, reading the bound mean gradients (the staged counterpart, like
 * cmn_momentum_sgd). */
int cmn_adam(const cmn_plan *plan, float alpha, float beta1, float beta2, float eps, float wd, int t,
             void *stream);

/* For callers that cannot allocate device memory or bind a workspace (code under HIP graph
 * capture, serving loops, harnesses that forbid allocation): cmn_allreduce_step on a plan that
 * only has to be created, with the tensor lists passed in the call (host arrays as in
 * cmn_plan_bind; mean_grad_ptrs may be NULL unless mean_dest is CMN_MEAN_TO_MEAN_GRADS).  The
 * tables cmn_plan_bind would upload go into one CMN_NOALLOC_SCRATCH_BYTES array inside the
 * library's code object instead (every GPU the library runs on holds its copy until the process
 * ends), written by small kernels on `stream`; while successive calls on a device pass the same
 * plan and pointers only the step kernels are launched.  Results are cmn_allreduce_step's, bit
 * for bit.  The call allocates no device memory, copies nothing from host buffers and does not
 * wait for the stream.  The current device must be the stream's.  All calls on one GPU share
 * the one array: calls whose work may overlap there (different streams, or replays of a
 * captured call next to other calls) race; work queued on one stream is safe.
 * Errors: CMN_ESIZE if cmn_plan_workspace_bytes(plan) exceeds CMN_NOALLOC_SCRATCH_BYTES (161
 * tensors x 32 replicas need 1.7 MB, VGG-16 x 16 replicas 8.7 MB), CMN_EINVAL for a CMN_I8S
 * plan (its scales are bound through a workspace) or an unknown mean_dest, CMN_ENULL,
 * CMN_EALIGN, CMN_EUNBOUND, CMN_EHIP, CMN_ENOMEM (host). */
#define CMN_NOALLOC_SCRATCH_BYTES (16 * 1024 * 1024)
int cmn_allreduce_step_noalloc(cmn_plan *plan, const void *const *grad_ptrs /* host [K*T] */,
                               void *const *param_ptrs /* host [T] */, void *const *vel_ptrs /* host [T] */,
                               void *const *mean_grad_ptrs /* host [T] or NULL */, float lr, float mu, float wd,
                               int mean_dest, void *stream);

/* Static, never NULL. */
const char *cmn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* CMN_H_ */
