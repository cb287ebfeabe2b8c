/*
 * CPU oracle for the per-GPU data path of MiCS partitioned data parallelism.
 * TEST INFRASTRUCTURE ONLY -- see mics_oracle.h.  Plain scalar loops written
 * from the paper's definitions (Sections 3.1-3.4); no blocking, no fusion, no
 * code shared with the HIP library.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * (-ffp-contract=off keeps every binary32 operation separately rounded).
 */
#include "mics_oracle.h"

#include <float.h>
#include <math.h>
#include <string.h>

#if FLT_EVAL_METHOD != 0
#error "binary32 expressions must be evaluated in binary32 (FLT_EVAL_METHOD 0)"
#endif
#ifdef __FAST_MATH__
#error "the oracle must not be built with fast-math"
#endif

static int g_threads = 1;

int orc_set_threads(int n)
{
    if (n >= 1) g_threads = n;
    return g_threads;
}

/* ---- bfloat16 ------------------------------------------------------------ */

float orc_bf16_widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

uint16_t orc_bf16_narrow(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t kept = u >> 16;        /* sign, exponent, top 7 fraction bits   */
    uint32_t dropped = u & 0xFFFFu; /* the 16 fraction bits that do not fit  */
    if ((u & 0x7F800000u) == 0x7F800000u) {
        /* Inf or NaN.  Inf has a zero fraction and passes through; a NaN must
         * stay a NaN even if its payload sat only in the dropped bits. */
        if ((u & 0x007FFFFFu) != 0) kept |= 0x0040u;
        return (uint16_t)kept;
    }
    /* Nearest of the two neighbouring bf16 values; on a tie the even one.
     * A carry out of the fraction moves into the exponent, which is the
     * right neighbour as well (up to and including +-Inf on overflow). */
    if (dropped > 0x8000u) kept += 1;
    else if (dropped == 0x8000u && (kept & 1u)) kept += 1;
    return (uint16_t)kept;
}

void orc_bf16_narrow_array(uint16_t* out, const float* in, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = orc_bf16_narrow(in[i]);
}

void orc_bf16_widen_array(float* out, const uint16_t* in, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = orc_bf16_widen(in[i]);
}

/* IEEE-754 binary16 -> binary32, exact (every binary16 value is a binary32 value). */
float orc_f16_widen(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t frac = h & 0x3FFu;
    uint32_t u;
    if (exp == 0x1Fu) {
        u = sign | 0x7F800000u | (frac << 13);               /* Inf or NaN */
    } else if (exp != 0) {
        u = sign | ((exp - 15 + 127) << 23) | (frac << 13);  /* normal */
    } else if (frac == 0) {
        u = sign;                                            /* zero */
    } else {
        /* subnormal: frac * 2^-24; normalise */
        int shift = 0;
        while (!(frac & 0x400u)) { frac <<= 1; ++shift; }
        frac &= 0x3FFu;
        u = sign | ((uint32_t)(127 - 15 + 1 - shift) << 23) | (frac << 13);
    }
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

void orc_f16_widen_array(float* out, const uint16_t* in, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = orc_f16_widen(in[i]);
}

/* binary32 -> IEEE-754 binary16, round to nearest, ties to even.  binary16 has 10 fraction
 * bits, exponents -14 .. 15 and subnormals that are multiples of 2^-24. */
uint16_t orc_f16_narrow(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t exp32 = (u >> 23) & 0xFFu;
    const uint32_t frac32 = u & 0x007FFFFFu;
    if (exp32 == 0xFFu)                                  /* Inf; NaN stays a (quiet) NaN */
        return (uint16_t)(sign | 0x7C00u | (frac32 ? 0x0200u | (frac32 >> 13) : 0u));
    const int e = (int)exp32 - 127;                      /* unbiased exponent of a normal input */
    if (exp32 == 0 || e < -25) return sign;              /* below half of the smallest subnormal */
    if (e > 15) return (uint16_t)(sign | 0x7C00u);       /* beyond the largest finite value */
    /* the 24-bit significand 1.frac32 as an integer, and how many of its low bits do not fit:
     * 13 for a normal result, more for a subnormal one (whose unit is 2^-24) */
    const uint32_t sig = frac32 | 0x00800000u;
    const int drop = e >= -14 ? 13 : 13 + (-14 - e);
    uint32_t kept = sig >> drop;
    const uint32_t rest = sig & ((1u << drop) - 1u);
    const uint32_t half = 1u << (drop - 1);
    if (rest > half || (rest == half && (kept & 1u))) kept += 1;
    /* normal: kept holds the hidden bit (bit 10), so adding the biased exponent minus one puts
     * both in place, and a carry out of the fraction moves into the exponent (up to Inf);
     * subnormal: kept is the fraction itself, and a carry makes the smallest normal */
    const uint32_t h = e >= -14 ? ((uint32_t)(e + 15 - 1) << 10) + kept : kept;
    return (uint16_t)(sign | h);
}

void orc_f16_narrow_array(uint16_t* out, const float* in, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = orc_f16_narrow(in[i]);
}

/* ---- hierarchical all-gather (Section 3.3) ------------------------------- */

static int geometry_ok(int p, int k, int elem_bytes)
{
    if (p < 1 || k < 1 || k > p) return 0;
    if (p % k != 0) return 0; /* the paper assumes p divisible by k */
    if (elem_bytes != 2 && elem_bytes != 4) return 0;
    return 1;
}

int orc_stage1_gather(void* T_l, const void* const* shards, size_t S,
                      int p, int k, int l, int elem_bytes)
{
    if (!geometry_ok(p, k, elem_bytes) || !T_l || !shards) return -1;
    if (l < 0 || l >= k) return -1;
    size_t eb = (size_t)elem_bytes;
    int nodes = p / k;
    /* The channel of local rank l holds one device per node; an all-gather
     * places member j's contribution at slot j.  Member j is group rank
     * j*k + l, whose contribution is its shard C_{j*k+l}. */
    for (int j = 0; j < nodes; ++j) {
        const unsigned char* src = (const unsigned char*)shards[j * k + l];
        if (!src) return -1;
        unsigned char* dst = (unsigned char*)T_l + (size_t)j * S * eb;
        for (size_t b = 0; b < S * eb; ++b) dst[b] = src[b];
    }
    return 0;
}

int orc_naive_intra_gather(void* W, const void* const* T, size_t S,
                           int p, int k, int elem_bytes)
{
    if (!geometry_ok(p, k, elem_bytes) || !W || !T) return -1;
    size_t per_rank = (size_t)(p / k) * S * (size_t)elem_bytes;
    /* Intra-node all-gather: local rank l's whole buffer lands at slot l. */
    for (int l = 0; l < k; ++l) {
        const unsigned char* src = (const unsigned char*)T[l];
        if (!src) return -1;
        unsigned char* dst = (unsigned char*)W + (size_t)l * per_rank;
        for (size_t b = 0; b < per_rank; ++b) dst[b] = src[b];
    }
    return 0;
}

int orc_concat_shards(void* F, const void* const* shards, size_t n_valid,
                      size_t S, int p, int elem_bytes)
{
    if (p < 1 || (elem_bytes != 2 && elem_bytes != 4) || !shards) return -1;
    if (n_valid > (size_t)p * S) return -1;
    if (n_valid && !F) return -1;
    size_t eb = (size_t)elem_bytes;
    unsigned char* out = (unsigned char*)F;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t x = 0; x < n_valid; ++x) {
        size_t g = x / S; /* owning group rank */
        size_t i = x % S; /* position inside its shard */
        const unsigned char* src = (const unsigned char*)shards[g];
        for (size_t b = 0; b < eb; ++b) out[x * eb + b] = src[i * eb + b];
    }
    return 0;
}

int orc_hier_gather_reorder(void* F, const void* const* T, size_t n_valid,
                            size_t S, int p, int k, int elem_bytes)
{
    if (!geometry_ok(p, k, elem_bytes) || !T) return -1;
    if (n_valid > (size_t)p * S) return -1;
    if (n_valid && !F) return -1;
    size_t eb = (size_t)elem_bytes;
    unsigned char* out = (unsigned char*)F;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t x = 0; x < n_valid; ++x) {
        size_t g = x / S;           /* chunk C_g owns flat element x        */
        size_t i = x % S;
        size_t j = g / (size_t)k;   /* node of rank g                        */
        size_t l = g % (size_t)k;   /* local rank of rank g                  */
        const unsigned char* src = (const unsigned char*)T[l];
        size_t at = j * S + i;      /* stage 1 put C_g at slot j of T_l      */
        for (size_t b = 0; b < eb; ++b) out[x * eb + b] = src[at * eb + b];
    }
    return 0;
}

/* ---- 2-hop gradient synchronisation (Section 3.4) ------------------------ */

int orc_reduce_scatter_accum(float* acc, const uint16_t* const* grads,
                             size_t elem_offset, size_t count, int p,
                             int accumulate)
{
    if (p < 1 || !grads) return -1;
    if (count && !acc) return -1;
    for (int q = 0; q < p; ++q) if (!grads[q]) return -1;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t i = 0; i < count; ++i) {
        size_t x = elem_offset + i;
        float partial = orc_bf16_widen(grads[0][x]);
        for (int q = 1; q < p; ++q) {
            float gq = orc_bf16_widen(grads[q][x]);
            partial = partial + gq;
        }
        float before = accumulate ? acc[i] : 0.0f;
        acc[i] = before + partial;
    }
    return 0;
}

static float widen_grad(const void* buf, size_t x, int dtype)
{
    if (dtype == ORC_DTYPE_F32) return ((const float*)buf)[x];
    if (dtype == ORC_DTYPE_F16) return orc_f16_widen(((const uint16_t*)buf)[x]);
    return orc_bf16_widen(((const uint16_t*)buf)[x]);
}

int orc_reduce_scatter_accum_typed(float* acc, const void* const* grads,
                                   size_t elem_offset, size_t count, int p,
                                   int accumulate, int dtype)
{
    if (p < 1 || !grads) return -1;
    if (dtype != ORC_DTYPE_BF16 && dtype != ORC_DTYPE_F16 && dtype != ORC_DTYPE_F32) return -1;
    if (count && !acc) return -1;
    for (int q = 0; q < p; ++q) if (!grads[q]) return -1;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t i = 0; i < count; ++i) {
        size_t x = elem_offset + i;
        float partial = widen_grad(grads[0], x, dtype);
        for (int q = 1; q < p; ++q) {
            float gq = widen_grad(grads[q], x, dtype);
            partial = partial + gq;
        }
        float before = accumulate ? acc[i] : 0.0f;
        acc[i] = before + partial;
    }
    return 0;
}

int orc_reduce_scatter_accum_f64(double* acc, const uint16_t* const* grads,
                                 size_t elem_offset, size_t count, int p,
                                 int accumulate)
{
    if (p < 1 || !grads) return -1;
    if (count && !acc) return -1;
    for (int q = 0; q < p; ++q) if (!grads[q]) return -1;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t i = 0; i < count; ++i) {
        size_t x = elem_offset + i;
        double partial = 0.0;
        for (int q = 0; q < p; ++q) partial += (double)orc_bf16_widen(grads[q][x]);
        acc[i] = (accumulate ? acc[i] : 0.0) + partial;
    }
    return 0;
}

int orc_replica_average(float* out, const float* const* copies, size_t count,
                        int r, float scale)
{
    if (r < 1 || !copies) return -1;
    if (count && !out) return -1;
    for (int c = 0; c < r; ++c) if (!copies[c]) return -1;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t i = 0; i < count; ++i) {
        float sum = copies[0][i];
        for (int c = 1; c < r; ++c) sum = sum + copies[c][i];
        out[i] = sum * scale;
    }
    return 0;
}

/* ---- mixed-precision Adam (Sections 2.1, 3.2) ---------------------------- */

static int adam_args_ok(const float* w, const float* m, const float* v,
                        const float* g, size_t count, int step)
{
    if (step < 1) return 0;
    if (count && (!w || !m || !v || !g)) return 0;
    return 1;
}

int orc_adam_shard(float* master, float* exp_avg, float* exp_avg_sq,
                   uint16_t* param_bf16, const float* grad, size_t count,
                   float lr, float beta1, float beta2, float eps,
                   float weight_decay, int step)
{
    if (!adam_args_ok(master, exp_avg, exp_avg_sq, grad, count, step)) return -1;
    const double b1 = beta1, b2 = beta2, a = lr, e = eps, wd = weight_decay;
    const double corr1 = 1.0 - pow(b1, (double)step);
    const double corr2 = 1.0 - pow(b2, (double)step);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t i = 0; i < count; ++i) {
        double g = grad[i], w = master[i], m = exp_avg[i], v = exp_avg_sq[i];
        double m_new = b1 * m + (1.0 - b1) * g;
        double v_new = b2 * v + (1.0 - b2) * g * g;
        double m_hat = m_new / corr1;
        double v_hat = v_new / corr2;
        double w_new = w - a * (m_hat / (sqrt(v_hat) + e) + wd * w);
        exp_avg[i] = (float)m_new;
        exp_avg_sq[i] = (float)v_new;
        master[i] = (float)w_new;
        if (param_bf16) param_bf16[i] = orc_bf16_narrow(master[i]);
    }
    return 0;
}

int orc_adam_shard_f32(float* master, float* exp_avg, float* exp_avg_sq,
                       uint16_t* param_bf16, const float* grad, size_t count,
                       float lr, float beta1, float beta2, float eps,
                       float weight_decay, int step)
{
    if (!adam_args_ok(master, exp_avg, exp_avg_sq, grad, count, step)) return -1;
    const float corr1 = (float)(1.0 - pow((double)beta1, (double)step));
    const float corr2 = (float)(1.0 - pow((double)beta2, (double)step));
    const float one_minus_b1 = 1.0f - beta1;
    const float one_minus_b2 = 1.0f - beta2;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (size_t i = 0; i < count; ++i) {
        /* one operation per line: each is rounded to binary32 on its own */
        float g = grad[i], w = master[i];
        float t1 = beta1 * exp_avg[i];
        float t2 = one_minus_b1 * g;
        float m_new = t1 + t2;
        float gg = g * g;
        float t3 = beta2 * exp_avg_sq[i];
        float t4 = one_minus_b2 * gg;
        float v_new = t3 + t4;
        float m_hat = m_new / corr1;
        float v_hat = v_new / corr2;
        float root = sqrtf(v_hat);
        float denom = root + eps;
        float ratio = m_hat / denom;
        float decay = weight_decay * w;
        float update = ratio + decay;
        float delta = lr * update;
        float w_new = w - delta;
        exp_avg[i] = m_new;
        exp_avg_sq[i] = v_new;
        master[i] = w_new;
        if (param_bf16) param_bf16[i] = orc_bf16_narrow(w_new);
    }
    return 0;
}
