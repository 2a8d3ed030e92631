/*
 * CPU oracle for the update phase of MLP-Offload (arXiv 2509.02480).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.
 *
 * What it computes (one optimizer step over a list of subgroups):
 *   - the mixed-precision scheme of Section 2 "Mixed Precision Training" and
 *     "Sharded Model and Optimizer States Into Subgroups": fp32 master
 *     parameters p, fp32 momentum m and variance v per subgroup, driven by
 *     half-precision gradients, with a half-precision working copy of p
 *     written back after the update;
 *   - the per-subgroup body of Algorithm 1 (upcast gradients on the fly,
 *     update, downcast parameters), Section 3.2 "Delayed In-place
 *     Mixed-Precision Gradient Conversion";
 *   - Adam is the optimizer the paper names (Section 3.2 "Cache-Friendly
 *     Ordering"); the paper prints no equations, so the arithmetic below is
 *     the textbook AdamW (decoupled weight decay, bias correction, eps added
 *     to the bias-corrected root), every operation rounded to fp32 once, in
 *     the order written, without fused multiply-add; the textbook Adam with
 *     the decay term added to the gradient is the other mode (l2_mode);
 *   - loss-scale removal, the non-finite check, the global L2 norm and the
 *     clip coefficient are not in the paper; they follow the usual
 *     mixed-precision convention (norm of the unscaled gradients, one flag
 *     skips the whole step).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * (no x87: x86-64 SSE arithmetic rounds every fp32 operation to fp32).
 *
 * Parity pins for every function here live in tests/test_oracle_*.py.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t bias_correction;
    int32_t l2_mode; /* 0: decoupled weight decay (AdamW); 1: Adam with the decay
                        term weight_decay * p added to the gradient */
} orc_hparams;

/* Scalars derived once per step (host side, fp64, each rounded once to fp32). */
typedef struct {
    float beta1, beta2, omb1, omb2, eps, step_size, sqbc2, decay;
    float l2; /* weight decay added to the gradient (l2_mode), else 0 */
} orc_consts;

/* ---- half-precision conversions (Section 2 "Mixed Precision Training") ---- */

/* bf16 is the upper half of an IEEE fp32 word: widening is exact. */
float orc_bf16_to_f32(uint16_t h) {
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even on the kept low bit.
 * Overflow rounds to infinity as IEEE does; every NaN becomes the canonical
 * quiet NaN with the input's sign. */
uint16_t orc_f32_to_bf16_rne(float f) {
    uint32_t w;
    memcpy(&w, &f, sizeof w);
    if ((w & 0x7FFFFFFFu) > 0x7F800000u) /* NaN */
        return (uint16_t)(((w >> 16) & 0x8000u) | 0x7FC0u);
    uint32_t lower = w & 0xFFFFu;
    uint32_t upper = w >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1u;
    return (uint16_t)upper;
}

/* Array forms of the two conversions (plain loops over the scalar routines). */
void orc_bf16_to_f32_array(const uint16_t* h, float* f, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) f[i] = orc_bf16_to_f32(h[i]);
}

void orc_f32_to_bf16_rne_array(const float* f, uint16_t* h, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) h[i] = orc_f32_to_bf16_rne(f[i]);
}

/* ---- the other half-precision format ---------------------------------------
 * The paper allows FP16 or BF16 for gradients and working parameters (Section 2
 * "Mixed Precision Training"; Algorithm 1 writes FP16).  Every routine below
 * exists in a form that takes the format: ORC_BF16 (0) or ORC_FP16 (1); the
 * forms without the argument are the bf16 ones. */
#define ORC_BF16 0
#define ORC_FP16 1

/* IEEE binary16 -> fp32: exact.  Built from the bit fields: sign, 5-bit
 * exponent (bias 15), 10-bit fraction; subnormals are fraction * 2^-24. */
float orc_f16_to_f32(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t frac = h & 0x3FFu;
    uint32_t w;
    if (e == 0x1Fu) {
        w = sign | 0x7F800000u | (frac << 13); /* inf or NaN, payload kept */
    } else if (e != 0) {
        w = sign | ((e + 112u) << 23) | (frac << 13); /* rebias 15 -> 127 */
    } else if (frac == 0) {
        w = sign;
    } else {
        /* subnormal: normalise the fraction */
        uint32_t shift = 0;
        while ((frac & 0x400u) == 0) {
            frac <<= 1;
            ++shift;
        }
        frac &= 0x3FFu;
        w = sign | ((113u - shift) << 23) | (frac << 13);
    }
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

/* fp32 -> IEEE binary16, round to nearest, ties to even; values of
 * magnitude >= 65520 round to infinity, results below 2^-14 are subnormal
 * (multiples of 2^-24), every NaN becomes the quiet NaN 0x7E00 with the
 * input's sign. */
uint16_t orc_f32_to_f16_rne(float f) {
    uint32_t w;
    memcpy(&w, &f, sizeof w);
    uint16_t sign = (uint16_t)((w >> 16) & 0x8000u);
    uint32_t mag = w & 0x7FFFFFFFu;
    if (mag > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);
    if (mag >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u); /* >= 65520 */
    int32_t e = (int32_t)(mag >> 23) - 127; /* unbiased exponent */
    uint32_t sig = (mag & 0x7FFFFFu) | 0x800000u; /* 24-bit significand */
    uint32_t drop; /* low bits of sig that do not fit */
    if (e >= -14) {
        drop = 13;
    } else if (e >= -25) {
        drop = (uint32_t)(13 + (-14 - e)); /* subnormal result: fewer kept bits */
    } else {
        return sign; /* below half of the smallest subnormal (fp32 zeros and subnormals included) */
    }
    uint32_t kept = sig >> drop;
    uint32_t rest = sig & ((1u << drop) - 1u);
    uint32_t half = 1u << (drop - 1);
    if (rest > half || (rest == half && (kept & 1u))) kept += 1u;
    /* kept now holds the result's significand in units of its last place;
     * adding the exponent field by arithmetic lets a carry run into it */
    uint32_t out;
    if (e >= -14)
        out = ((uint32_t)(e + 15) << 10) + (kept - 0x400u);
    else
        out = kept; /* subnormal (a carry to 0x400 is the smallest normal) */
    return (uint16_t)(sign | out);
}

float orc_half_to_f32(uint16_t h, int32_t half) {
    return half == ORC_FP16 ? orc_f16_to_f32(h) : orc_bf16_to_f32(h);
}

uint16_t orc_f32_to_half_rne(float f, int32_t half) {
    return half == ORC_FP16 ? orc_f32_to_f16_rne(f) : orc_f32_to_bf16_rne(f);
}

/* +-inf or NaN: the exponent field is all ones. */
static int orc_half_nonfinite(uint16_t h, int32_t half) {
    uint16_t mask = half == ORC_FP16 ? 0x7C00u : 0x7F80u;
    return (h & mask) == mask;
}

void orc_f16_to_f32_array(const uint16_t* h, float* f, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) f[i] = orc_f16_to_f32(h[i]);
}

void orc_f32_to_f16_rne_array(const float* f, uint16_t* h, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) h[i] = orc_f32_to_f16_rne(f[i]);
}

/* ---- gradient accumulation over micro-batches ----------------------------- */

/* The half-precision accumulation buffer of Section 3.2 "Delayed In-place
 * Mixed-Precision Gradient Conversion" (the buffer the update later upcasts
 * on the fly): the first micro-batch of a step overwrites it, every later
 * one is added element by element.  The paper does not print the
 * arithmetic; the reading taken is the one a half-precision buffer allows:
 * widen both (exact), one fp32 addition, round back to bf16 (nearest even).
 * A NaN sum is stored as the canonical quiet NaN 0x7FC0 whatever sign or
 * payload the addition produced, because IEEE 754 leaves those open. */
void orc_grad_accumulate_h(uint16_t* acc, const uint16_t* g, uint64_t n,
                           int32_t first, int32_t half) {
    uint16_t nan = half == ORC_FP16 ? 0x7E00u : 0x7FC0u;
    for (uint64_t i = 0; i < n; ++i) {
        if (first) {
            acc[i] = g[i];
            continue;
        }
        float sum = orc_half_to_f32(acc[i], half) + orc_half_to_f32(g[i], half);
        acc[i] = (sum != sum) ? nan : orc_f32_to_half_rne(sum, half);
    }
}

void orc_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n,
                         int32_t first) {
    orc_grad_accumulate_h(acc, g, n, first, ORC_BF16);
}

/* ---- gradient statistics over one subgroup ------------------------------ */

/* Adds to *sumsq the fp64 sum of squares of the unscaled gradients
 * u_i = f32(g_i) * inv_scale (one fp32 product), and ORs into *found_inf
 * whether any g_i is +-inf or NaN (bf16 exponent field all ones). */
void orc_grad_stats_h(const uint16_t* g, uint64_t n, float inv_scale,
                      int32_t half, double* sumsq, uint32_t* found_inf) {
    double s = *sumsq;
    uint32_t bad = *found_inf;
    for (uint64_t i = 0; i < n; ++i) {
        if (orc_half_nonfinite(g[i], half)) bad = 1u;
        float u = orc_half_to_f32(g[i], half) * inv_scale;
        s += (double)u * (double)u;
    }
    *sumsq = s;
    *found_inf = bad;
}

void orc_grad_stats(const uint16_t* g, uint64_t n, float inv_scale,
                    double* sumsq, uint32_t* found_inf) {
    orc_grad_stats_h(g, n, inv_scale, ORC_BF16, sumsq, found_inf);
}

/* norm = sqrt(sum of squares) rounded to fp32; clip coefficient
 * max_norm / (norm + 1e-6) when clipping is on and the norm exceeds
 * max_norm, else 1; gmul = inv_scale * clip_coef is the single factor the
 * update applies to the raw gradient. */
void orc_norm_finish(double sumsq, float inv_scale, float max_norm,
                     float* norm, float* clip_coef, float* gmul) {
    float nrm = (float)sqrt(sumsq);
    float coef = 1.0f;
    if (max_norm > 0.0f && nrm > max_norm) coef = max_norm / (nrm + 1e-6f);
    *norm = nrm;
    *clip_coef = coef;
    *gmul = inv_scale * coef;
}

/* ---- AdamW, fp32 state (the precision the paper fixes for p, m, v) ------- */

void orc_adamw_consts(const orc_hparams* hp, int64_t step, orc_consts* c) {
    double b1 = (double)hp->beta1, b2 = (double)hp->beta2;
    double bc1 = 1.0, bc2 = 1.0;
    if (hp->bias_correction) {
        bc1 = 1.0 - pow(b1, (double)step);
        bc2 = 1.0 - pow(b2, (double)step);
    }
    c->beta1 = hp->beta1;
    c->beta2 = hp->beta2;
    c->omb1 = (float)(1.0 - b1);
    c->omb2 = (float)(1.0 - b2);
    c->eps = hp->eps;
    c->step_size = (float)((double)hp->lr / bc1);
    c->sqbc2 = (float)sqrt(bc2);
    c->decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);
    c->l2 = 0.0f;
    if (hp->l2_mode) { /* the decay acts through the gradient only */
        c->decay = 1.0f;
        c->l2 = hp->weight_decay;
    }
}

/* One applied step (step is the 1-based count of applied steps) on one
 * subgroup, in place.  p16 receives the bf16 working copy of the new p. */
void orc_adamw_f32_h(float* p, float* m, float* v, const uint16_t* g,
                     uint16_t* p16, uint64_t n, const orc_hparams* hp,
                     int64_t step, float gmul, int32_t half) {
    orc_consts c;
    orc_adamw_consts(hp, step, &c);
    for (uint64_t i = 0; i < n; ++i) {
        float gi = orc_half_to_f32(g[i], half) * gmul;
        if (hp->l2_mode) {
            float t0 = c.l2 * p[i];
            gi = gi + t0;
        }
        float t1 = c.beta1 * m[i];
        float t2 = c.omb1 * gi;
        float mi = t1 + t2;
        float gg = gi * gi;
        float t3 = c.beta2 * v[i];
        float t4 = c.omb2 * gg;
        float vi = t3 + t4;
        float r = sqrtf(vi);
        float q = r / c.sqbc2;
        float d = q + c.eps;
        float ratio = mi / d;
        float upd = c.step_size * ratio;
        float pd = p[i] * c.decay;
        float pi = pd - upd;
        m[i] = mi;
        v[i] = vi;
        p[i] = pi;
        p16[i] = orc_f32_to_half_rne(pi, half);
    }
}

void orc_adamw_f32(float* p, float* m, float* v, const uint16_t* g,
                   uint16_t* p16, uint64_t n, const orc_hparams* hp,
                   int64_t step, float gmul) {
    orc_adamw_f32_h(p, m, v, g, p16, n, hp, step, gmul, ORC_BF16);
}

/* The same step with every quantity and operation in fp64, straight from the
 * textbook form (m-hat = m/(1-b1^t), v-hat = v/(1-b2^t)); used to pin the
 * fp32 routine on tiny inputs.  The fp32 hyper-parameters are widened. */
void orc_adamw_f64_h(double* p, double* m, double* v, const uint16_t* g,
                     uint64_t n, const orc_hparams* hp, int64_t step,
                     double gmul, int32_t half) {
    double b1 = hp->beta1, b2 = hp->beta2, lr = hp->lr, eps = hp->eps,
           wd = hp->weight_decay;
    double bc1 = 1.0, bc2 = 1.0;
    if (hp->bias_correction) {
        bc1 = 1.0 - pow(b1, (double)step);
        bc2 = 1.0 - pow(b2, (double)step);
    }
    for (uint64_t i = 0; i < n; ++i) {
        double gi = (double)orc_half_to_f32(g[i], half) * gmul;
        if (hp->l2_mode) gi += wd * p[i];
        m[i] = b1 * m[i] + (1.0 - b1) * gi;
        v[i] = b2 * v[i] + (1.0 - b2) * gi * gi;
        double mhat = m[i] / bc1;
        double vhat = v[i] / bc2;
        double keep = hp->l2_mode ? 1.0 : 1.0 - lr * wd;
        p[i] = p[i] * keep - lr * mhat / (sqrt(vhat) + eps);
    }
}

void orc_adamw_f64(double* p, double* m, double* v, const uint16_t* g,
                   uint64_t n, const orc_hparams* hp, int64_t step,
                   double gmul) {
    orc_adamw_f64_h(p, m, v, g, n, hp, step, gmul, ORC_BF16);
}

/* ---- one whole step over a list of subgroups ----------------------------- */

typedef struct {
    float* p;
    float* m;
    float* v;
    const uint16_t* g;
    uint16_t* p16;
    uint64_t n;
} orc_subgroup;

/* Runs statistics over all subgroups, then either skips everything (a
 * non-finite gradient anywhere) or applies the update to every subgroup.
 * step_applied is the number of steps applied so far; returns 1 when this
 * step was applied (the caller then counts it), 0 when skipped.  order, if
 * not NULL, is the sequence in which subgroups are visited (Algorithm 1's
 * processing order); results do not depend on it. */
int orc_step_h(const orc_subgroup* sg, int32_t n_sg, const int32_t* order,
               const orc_hparams* hp, int64_t steps_applied, float inv_scale,
               float max_norm, int32_t half, float* out_norm,
               uint32_t* out_found_inf, float* out_gmul) {
    double sumsq = 0.0;
    uint32_t bad = 0;
    for (int32_t k = 0; k < n_sg; ++k)
        orc_grad_stats_h(sg[k].g, sg[k].n, inv_scale, half, &sumsq, &bad);
    float norm, coef, gmul;
    orc_norm_finish(sumsq, inv_scale, max_norm, &norm, &coef, &gmul);
    /* Finite gradients can have a norm that fp32 cannot hold (two of the
     * largest bf16 value, or an unscale factor above 1): the clip factor
     * would then be 0 or infinity would enter the moments.  Such a step is
     * skipped like one with a non-finite gradient. */
    if (!(norm <= FLT_MAX)) bad = 1u;
    *out_norm = norm;
    *out_found_inf = bad;
    *out_gmul = gmul;
    if (bad) return 0;
    for (int32_t k = 0; k < n_sg; ++k) {
        const orc_subgroup* s = &sg[order ? order[k] : k];
        orc_adamw_f32_h(s->p, s->m, s->v, s->g, s->p16, s->n, hp,
                        steps_applied + 1, gmul, half);
    }
    return 1;
}

int orc_step(const orc_subgroup* sg, int32_t n_sg, const int32_t* order,
             const orc_hparams* hp, int64_t steps_applied, float inv_scale,
             float max_norm, float* out_norm, uint32_t* out_found_inf,
             float* out_gmul) {
    return orc_step_h(sg, n_sg, order, hp, steps_applied, inv_scale, max_norm,
                      ORC_BF16, out_norm, out_found_inf, out_gmul);
}

/* ---- the same routines driven over independent chunks by several threads --
 * Only used to time the oracle on all host cores.  Elements are independent
 * (Section 3.2 "Cache-Friendly Ordering"), so chunking changes nothing; the
 * per-chunk sums of squares are combined in index order so the result does
 * not depend on the thread count. */
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_CHUNK ((uint64_t)1 << 20)

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_adamw_f32_chunked(float* p, float* m, float* v, const uint16_t* g,
                           uint16_t* p16, uint64_t n, const orc_hparams* hp,
                           int64_t step, float gmul) {
    int64_t n_chunks = (int64_t)((n + ORC_CHUNK - 1) / ORC_CHUNK);
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n_chunks; ++c) {
        uint64_t lo = (uint64_t)c * ORC_CHUNK;
        uint64_t len = n - lo < ORC_CHUNK ? n - lo : ORC_CHUNK;
        orc_adamw_f32(p + lo, m + lo, v + lo, g + lo, p16 + lo, len, hp, step,
                      gmul);
    }
}

/* partial must hold ceil(n / 2^20) doubles. */
void orc_grad_stats_chunked(const uint16_t* g, uint64_t n, float inv_scale,
                            double* partial, double* sumsq,
                            uint32_t* found_inf) {
    int64_t n_chunks = (int64_t)((n + ORC_CHUNK - 1) / ORC_CHUNK);
    uint32_t bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t c = 0; c < n_chunks; ++c) {
        uint64_t lo = (uint64_t)c * ORC_CHUNK;
        uint64_t len = n - lo < ORC_CHUNK ? n - lo : ORC_CHUNK;
        double s = 0.0;
        uint32_t b = 0;
        orc_grad_stats(g + lo, len, inv_scale, &s, &b);
        partial[c] = s;
        bad |= b;
    }
    double s = *sumsq;
    for (int64_t c = 0; c < n_chunks; ++c) s += partial[c];
    *sumsq = s;
    *found_inf |= bad;
}
