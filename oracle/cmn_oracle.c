/*
 * CPU oracle for the gradient aggregation + update step of synchronous
 * data-parallel training (ChainerMN paper, Section 2.3 "Synchronous vs.
 * Asynchronous": the Allreduce step and the optimization step; Section 2.1
 * for the optimizer rule).
 *
 * THIS IS TEST INFRASTRUCTURE, not the product.  It is plain, slow and meant
 * to be checked against the paper by eye.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may use it.  It shares no code, header,
 * table or helper with the HIP implementation.
 *
 * Arithmetic: IEEE-754 binary32, round-to-nearest-even, one rounding per
 * written operation (build with -ffp-contract=off, no fast-math), subnormals
 * kept.  The order of the K-term sum is part of the definition (see
 * orc_direct_fold).
 *
 * Pins (tests/test_oracle_pins.py): exact integer sums by brute force, the
 * float64 error bound of recursive summation, a hand-worked cancellation case
 * that fixes the fold order, ring simulation == direct fold and all ranks
 * identical, power-of-two scaling, closed-form momentum series, the paper's
 * plain rule theta - lr*g at mu = 0, torch.optim.SGD, and an exhaustive
 * binary16 decode against numpy.  No function here is "parity unpinned".
 *
 * dtype codes: 0 = float32 gradients, 1 = IEEE binary16 gradients, 2 = bfloat16
 * gradients (the upper 16 bits of a binary32), 3 = int8 gradients with one float32
 * scale per (replica, ring chunk): value = (float)q * scale, the product rounded once.
 * The narrow types are storage only; every sum is accumulated in float32.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_F32 0
#define ORC_F16 1
#define ORC_BF16 2
#define ORC_I8S 3

/* ---- binary16 -> binary32, bit level (exact, incl. subnormals, Inf, NaN) ---- */
float orc_half_bits_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t exp5 = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t man10 = (uint32_t)h & 0x3ffu;
    uint32_t bits;
    float f;
    if (exp5 == 0) {
        /* zero or subnormal: value = man10 * 2^-24, exactly representable */
        f = (float)man10 * 0x1p-24f;
        memcpy(&bits, &f, 4);
        bits |= sign << 31;
    } else if (exp5 == 31) {
        bits = (sign << 31) | 0x7f800000u | (man10 << 13); /* Inf / NaN */
    } else {
        bits = (sign << 31) | ((exp5 + 112u) << 23) | (man10 << 13); /* rebias 15 -> 127 */
    }
    memcpy(&f, &bits, 4);
    return f;
}

/* ---- bfloat16 <-> binary32: a bfloat16 is the sign, exponent and top 7 mantissa bits ---- */
float orc_bf16_bits_to_float(uint16_t b)
{
    uint32_t bits = (uint32_t)b << 16;   /* exact: the dropped mantissa bits are zero */
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

uint16_t orc_float_to_bf16_bits(float f)      /* round to nearest, ties to even */
{
    uint32_t x;
    memcpy(&x, &f, 4);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x0040u);   /* NaN stays NaN (quiet) */
    uint32_t kept = x >> 16, rem = x & 0xffffu;
    if (rem > 0x8000u || (rem == 0x8000u && (kept & 1u))) ++kept;   /* a carry into the exponent, or to Inf, is correct */
    return (uint16_t)kept;
}

void orc_float_to_bf16_array(int64_t n, const float *in, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_float_to_bf16_bits(in[i]);
}

static float load_grad(const void *base, int dtype, int64_t i, float scale)
{
    if (dtype == ORC_I8S) {
        float q = (float)((const int8_t *)base)[i];   /* exact */
        return q * scale;
    }
    if (dtype == ORC_F16)
        return orc_half_bits_to_float(((const uint16_t *)base)[i]);
    if (dtype == ORC_BF16)
        return orc_bf16_bits_to_float(((const uint16_t *)base)[i]);
    return ((const float *)base)[i];
}

static int elem_bytes(int dtype) { return dtype == ORC_F32 ? 4 : dtype == ORC_I8S ? 1 : 2; }

/* ---- geometry of the packed buffer ------------------------------------------
 * off[0] = 0, off[t+1] = off[t] + numel[t], N = off[T].
 * The packed buffer is cut into C equal chunks, each rounded up to align_bytes:
 *   chunk_elems = roundup(ceil(N / C), align_bytes / elem_bytes),  L = C * chunk_elems.
 * Tensors are packed tightly; only [N, L) is padding.
 * Returns 0, or -1 on invalid arguments. */
int orc_geometry(int T, const int64_t *numel, int C, int align_bytes, int dtype,
                 int64_t *off /* [T+1] */, int64_t *N, int64_t *chunk_elems, int64_t *L)
{
    int eb = elem_bytes(dtype);
    if (T < 0 || C < 1 || align_bytes < eb || align_bytes % eb != 0) return -1;
    off[0] = 0;
    for (int t = 0; t < T; ++t) {
        if (numel[t] < 0) return -1;
        off[t + 1] = off[t] + numel[t];
    }
    int64_t A = align_bytes / eb;
    int64_t per = (off[T] + C - 1) / C;          /* ceil(N / C) */
    int64_t ce = ((per + A - 1) / A) * A;        /* round up to the alignment */
    *N = off[T];
    *chunk_elems = ce;
    *L = ce * C;
    return 0;
}

/* ---- S1 pack: one replica's T tensors, in list order, tightly; zero the pad -- */
void orc_pack(int T, const int64_t *numel, const void *const *tensors, int dtype,
              int64_t L, void *packed)
{
    int eb = elem_bytes(dtype);
    char *dst = (char *)packed;
    int64_t o = 0;
    for (int t = 0; t < T; ++t) {
        memcpy(dst + o * eb, tensors[t], (size_t)(numel[t] * eb));
        o += numel[t];
    }
    memset(dst + o * eb, 0, (size_t)((L - o) * eb));   /* +0.0 in both formats */
}

/* ---- S2 (definition): direct left fold in ring order --------------------------
 * For chunk c and element i of that chunk:
 *     sum = ((g[r_0] + g[r_1]) + g[r_2]) + ... + g[r_{K-1}],   r_j = (s + j) mod K,
 * s = c mod K when ring_rotate != 0 (what an ascending-rank ring produces, see
 * orc_ring_allreduce), s = 0 otherwise (plain rank order 0, 1, ..., K-1).
 * Chunks are independent, so the OpenMP loop over chunks changes no bit. */
void orc_direct_fold(int K, int C, int64_t chunk_elems, const void *const *packed /* [K] */,
                     int dtype, int ring_rotate, const float *const *scales /* [K][C], int8 only, else NULL */,
                     float *sum /* [C*chunk_elems] */)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        int s = ring_rotate ? c % K : 0;
        for (int64_t i = c * chunk_elems; i < (c + 1) * chunk_elems; ++i) {
            float acc = load_grad(packed[s], dtype, i, scales ? scales[s][c] : 1.0f);
            for (int j = 1; j < K; ++j) {
                int r = (s + j) % K;
                acc = acc + load_grad(packed[r], dtype, i, scales ? scales[r][c] : 1.0f);
            }
            sum[i] = acc;
        }
    }
}

/* ---- S2 (message-passing simulation of the textbook ring allreduce) -----------
 * K ranks, K chunks, ascending-rank direction.  buf[r] is rank r's own float32
 * buffer of K*chunk_elems elements and is overwritten with the allreduce result.
 * Reduce-scatter, steps s = 0..K-2: every rank r sends its chunk (r - s) mod K to
 * rank (r + 1) mod K, which stores   received + own   into that chunk.  After
 * K-1 steps rank r owns the finished chunk (r + 1) mod K.
 * All-gather, steps s = 0..K-2: every rank r forwards chunk (r + 1 - s) mod K to
 * rank (r + 1) mod K, which copies it.
 * All sends of one step happen "at once": they are staged in msg before any
 * receive touches a buffer.  Returns 0, or -1 if memory cannot be obtained. */
int orc_ring_allreduce(int K, int64_t chunk_elems, float *const *buf /* [K] */)
{
    if (K <= 1) return 0;
    float *msg = (float *)malloc((size_t)K * (size_t)chunk_elems * sizeof(float) + 1);
    if (!msg) return -1;
    for (int phase = 0; phase < 2; ++phase) {
        for (int s = 0; s < K - 1; ++s) {
            for (int r = 0; r < K; ++r) {                       /* send */
                int c = (((r + phase - s) % K) + K) % K;
                memcpy(msg + (size_t)r * chunk_elems, buf[r] + (size_t)c * chunk_elems,
                       (size_t)chunk_elems * sizeof(float));
            }
            for (int r = 0; r < K; ++r) {                       /* receive at r+1 */
                int c = (((r + phase - s) % K) + K) % K;
                float *own = buf[(r + 1) % K] + (size_t)c * chunk_elems;
                const float *recv = msg + (size_t)r * chunk_elems;
                for (int64_t i = 0; i < chunk_elems; ++i)
                    own[i] = (phase == 0) ? recv[i] + own[i] : recv[i];
            }
        }
    }
    free(msg);
    return 0;
}

/* ---- S3 scale: gbar = sum * (1/K), the reciprocal formed once in float32 ------ */
void orc_scale(int64_t n, const float *sum, int K, float *gbar)
{
    float s = 1.0f / (float)K;
    for (int64_t i = 0; i < n; ++i) gbar[i] = sum[i] * s;
}

/* ---- S4 unpack: scatter gbar[0, N) back to T tensors; padding is dropped ------ */
void orc_unpack(int T, const int64_t *numel, const float *gbar, float *const *tensors)
{
    int64_t o = 0;
    for (int t = 0; t < T; ++t) {
        memcpy(tensors[t], gbar + o, (size_t)numel[t] * sizeof(float));
        o += numel[t];
    }
}

/* ---- S5 MomentumSGD (a "variation" of the paper's rule theta <- theta - lr*g,
 * Section 2.1; the paper writes the learning rate as mu, here mu is the
 * momentum coefficient and lr the learning rate):
 *     g' = g + wd * p      (only when wd != 0; L2 decay on the averaged gradient)
 *     v  = mu * v - lr * g'
 *     p  = p + v
 * each operation rounded to float32. */
void orc_momentum_sgd(int64_t n, const float *g, float *p, float *v, float lr, float mu, float wd)
{
    for (int64_t i = 0; i < n; ++i) {
        float gi = g[i];
        if (wd != 0.0f) {
            float d = wd * p[i];
            gi = gi + d;
        }
        float t1 = mu * v[i];
        float t2 = lr * gi;
        float vn = t1 - t2;
        v[i] = vn;
        p[i] = p[i] + vn;
    }
}

/* ---- binary32 -> binary16, round to nearest even, bit level ----------------------
 * Used where the averaged gradient is handed back to replicas that store binary16. */
uint16_t orc_float_to_half_bits(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t exp8 = (x >> 23) & 0xffu;
    uint32_t man23 = x & 0x7fffffu;
    if (exp8 == 255) return (uint16_t)(sign | 0x7c00u | (man23 ? 0x200u | (man23 >> 13) : 0u)); /* Inf, quiet NaN */
    int e = (int)exp8 - 127 + 15;               /* exponent in binary16's bias */
    if (e >= 31) return (uint16_t)(sign | 0x7c00u);                  /* too large: infinity */
    if (e <= 0) {                               /* result is subnormal or zero */
        if (e < -10) return sign;               /* below half of the smallest subnormal */
        uint32_t m = man23 | 0x800000u;         /* make the leading one explicit */
        int shift = 14 - e;                     /* 14 .. 24 */
        uint32_t q = m >> shift, rem = m & ((1u << shift) - 1u), half = 1u << (shift - 1);
        if (rem > half || (rem == half && (q & 1u))) ++q;            /* nearest, ties to even */
        return (uint16_t)(sign | q);            /* a carry lands on the smallest normal: correct */
    }
    uint32_t h = ((uint32_t)e << 10) | (man23 >> 13);
    uint32_t rem = man23 & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;          /* carry may reach infinity: correct */
    return (uint16_t)(sign | h);
}

void orc_float_to_half_array(int64_t n, const float *in, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_float_to_half_bits(in[i]);
}

/* ---- Adam (Kingma & Ba) in the arrangement with the bias corrections folded into
 * the step size; the paper's Listing 1 wraps this optimizer (Section 3.3):
 *     g' = g + wd * p                  (only when wd != 0)
 *     m  = m + (1 - beta1) * (g' - m)
 *     v  = v + (1 - beta2) * (g'*g' - v)
 *     p  = p - lr_t * m / (sqrt(v) + eps),   lr_t = alpha * sqrt(1 - beta2^t) / (1 - beta1^t)
 * Every operation is rounded to float32 once; sqrt and the division are correctly rounded.
 * lr_t is formed in double from the float32 hyper-parameters and rounded once. */
#include <math.h>
float orc_adam_lr(float alpha, float beta1, float beta2, int t)
{
    double b1 = 1.0 - pow((double)beta1, (double)t);
    double b2 = 1.0 - pow((double)beta2, (double)t);
    return (float)((double)alpha * sqrt(b2) / b1);
}

void orc_adam(int64_t n, const float *g, float *p, float *m, float *v, float lr_t, float beta1, float beta2,
              float eps, float wd)
{
    float c1 = 1.0f - beta1, c2 = 1.0f - beta2;
    for (int64_t i = 0; i < n; ++i) {
        float gi = g[i];
        if (wd != 0.0f) {
            float dec = wd * p[i];
            gi = gi + dec;
        }
        float t1 = gi - m[i];
        float t2 = c1 * t1;
        float mn = m[i] + t2;
        float t3 = gi * gi;
        float t4 = t3 - v[i];
        float t5 = c2 * t4;
        float vn = v[i] + t5;
        float s = sqrtf(vn);
        float den = s + eps;
        float q = mn / den;
        float u = lr_t * q;
        m[i] = mn;
        v[i] = vn;
        p[i] = p[i] - u;
    }
}

int orc_max_threads(void);
#ifdef _OPENMP
#include <omp.h>
int orc_max_threads(void) { return omp_get_max_threads(); }
void orc_set_threads(int n) { omp_set_num_threads(n); }
#else
int orc_max_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif
