/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Plain, slow, single-threaded CPU definition of what one optimizer step of a
 * data-parallel job computes on the *unsharded* flat state: sum the N
 * per-device gradient contributions in a fixed order, take the mean, and apply
 * mixed-precision Adam with decoupled weight decay to the FP32 master weights
 * and moments, then round the new weights to 16 bits (bf16 or binary16).  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg may call into this file.  It
 * shares no code, header, table or helper with the GPU library.
 *
 * What the paper fixes and what it leaves open:
 *   - The gradient used for the update is the global-batch mean; with equal
 *     local batches that is the sum of the per-device means divided by N
 *     (Theorem 3, Eq. 15; proof of Theorem 2 part 1; proof of Theorem 5
 *     step 2).
 *   - Adam keeps a first moment m and a second moment v per parameter, in
 *     FP32, next to FP32 master weights; parameters and gradients are 16-bit
 *     (Section 2.1 "Optimizer state"; Table 1; Remark 1).
 *   - The update is Theta_{t+1} = Theta_t - eta * optimizer(G_t, Omega_t)
 *     (proof of Theorem 3), applied by each device to its own shard
 *     (proof of Corollary 1 part 1).
 *   - All participants reduce in one data type and in one deterministic order
 *     (Theorem 4 and its violation list; Theorem 5 assumption 1; Remark 3).
 *   The paper prints no Adam formula.  The reading taken here is the textbook
 *   bias-corrected Adam with decoupled decay, eps added outside the root, the
 *   decay applied to the old weight, with every arithmetic step a single
 *   IEEE-754 binary32 operation in the order written below.  "parity
 *   unpinned" by any value printed in the paper for the Adam arithmetic; it is
 *   pinned instead by closed forms, invariants and a library optimizer on the
 *   CPU (see tests/test_oracle_pins.py).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math (see oracle/build.py).
 * With contraction off every `*`, `+`, `/` below is one correctly rounded
 * binary32 operation (x86-64 SSE has no excess precision); fmaf() and sqrtf()
 * are correctly rounded by definition.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- 16-bit <-> 32-bit conversions (Remark 1: 2-byte params and grads) ---- */

/* bf16 is the upper half of a binary32; widening is exact. */
static float widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

float oracle_widen_bf16(uint16_t h) { return widen_bf16(h); }

/* Round a binary32 to the nearest bf16, ties to the even mantissa.  Infinities
 * stay, finite values past the largest bf16 go to infinity, -0 keeps its sign,
 * any NaN becomes the quiet NaN 0x7FC0 with the input's sign. */
uint16_t oracle_bf16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)(((u >> 16) & 0x8000u) | 0x7fc0u);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7fffu + keep_lsb;
    return (uint16_t)(u >> 16);
}

/* The same cast over an array (used by the exhaustive cast checks). */
void oracle_bf16_rne_array(const float *x, uint16_t *out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i)
        out[i] = oracle_bf16_rne(x[i]);
}

/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits; the paper's FP16 of
 * Table 1) to binary32: exact for every pattern, subnormals included. */
static float widen_f16(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t ex = (h >> 10) & 0x1fu, frac = h & 0x3ffu;
    uint32_t u;
    float f;
    if (ex == 0) { /* zero or subnormal: frac * 2^-24 */
        f = ldexpf((float)frac, -24);
        memcpy(&u, &f, sizeof u);
        u |= sign;
    } else if (ex == 31) { /* infinity or NaN: payload moved to the top of the fraction */
        u = sign | 0x7f800000u | (frac << 13);
    } else { /* normal: rebias 15 -> 127 */
        u = sign | ((ex + 112u) << 23) | (frac << 13);
    }
    memcpy(&f, &u, sizeof f);
    return f;
}

float oracle_widen_f16(uint16_t h) { return widen_f16(h); }

/* Round a binary32 to the nearest binary16, ties to the even fraction.  Values
 * of magnitude >= 65520 (the largest binary16 plus half a unit in its last
 * place) go to infinity, magnitudes below 2^-14 land on the subnormal grid of
 * spacing 2^-24 (or on zero, or on 2^-14 itself), -0 keeps its sign, any NaN
 * becomes the quiet NaN 0x7E00 with the input's sign. */
uint16_t oracle_f16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u)
        return (uint16_t)(sign | 0x7e00u);
    if (a >= 0x477ff000u) /* 65520.0f and beyond, infinity included */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x38800000u) { /* below 2^-14: count units of 2^-24, nearest, ties to even */
        float mag;
        memcpy(&mag, &a, sizeof mag);
        float units = nearbyintf(mag * 16777216.0f); /* the product is exact */
        return (uint16_t)(sign | (uint16_t)units);
    }
    uint32_t keep_lsb = (a >> 13) & 1u;
    a += 0xfffu + keep_lsb;                         /* may carry into the exponent: intended */
    return (uint16_t)(sign | (uint16_t)((a >> 13) - (112u << 10)));
}

/* The same cast over an array (used by the exhaustive cast checks). */
void oracle_f16_rne_array(const float *x, uint16_t *out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i)
        out[i] = oracle_f16_rne(x[i]);
}

/* ---- scalars ---- */

typedef struct {
    float gs;   /* mean scale 1/N (or the caller's gradient scale)            */
    float cc;   /* clip coefficient, 1 when there is no clipping              */
    float b1;   /* beta1                                                      */
    float omb1; /* 1 - beta1                                                  */
    float b2;   /* beta2                                                      */
    float omb2; /* 1 - beta2                                                  */
    float ep;   /* eps                                                        */
    float step; /* lr / (1 - beta1^t)                                         */
    float isb2; /* 1 / sqrt(1 - beta2^t)                                      */
    float lw;   /* lr * weight_decay                                          */
} oracle_scalars;

/* Every scalar is formed in binary64 from the hyper-parameters and the 1-based
 * step count t and rounded once to binary32.  grad_scale <= 0 selects 1/N
 * (proof of Theorem 5, step 2); clip_coef <= 0 selects 1. */
void oracle_derive_scalars(double lr, double beta1, double beta2, double eps,
                           double weight_decay, uint64_t t, uint32_t n_devices,
                           double grad_scale, double clip_coef,
                           oracle_scalars *out)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    out->gs = (float)(grad_scale > 0.0 ? grad_scale : 1.0 / (double)n_devices);
    out->cc = (float)(clip_coef > 0.0 ? clip_coef : 1.0);
    out->b1 = (float)beta1;
    out->omb1 = (float)(1.0 - beta1);
    out->b2 = (float)beta2;
    out->omb2 = (float)(1.0 - beta2);
    out->ep = (float)eps;
    out->step = (float)(lr / bc1);
    out->isb2 = (float)(1.0 / sqrt(bc2));
    out->lw = (float)(lr * weight_decay);
}

/* ---- gradient contributions ---- */

/* Contribution r's element e, widened to binary32.  All contributions carry
 * one data type (Theorem 4: identical data types); dtype 0 = bf16, 1 = binary32,
 * 2 = binary16. */
static float contribution(const void *const *g, int dtype, uint32_t r, uint64_t e)
{
    if (dtype == 1)
        return ((const float *)g[r])[e];
    if (dtype == 2)
        return widen_f16(((const uint16_t *)g[r])[e]);
    return widen_bf16(((const uint16_t *)g[r])[e]);
}

/* The reduce-scatter result before the mean (Section 2.3 "Reduce-Scatter";
 * Theorem 2 part 2): acc[e] = ((g_0[e] + g_1[e]) + g_2[e]) + ... in binary32,
 * device index ascending. */
void oracle_reduce_sum(const void *const *g, uint32_t n_contrib, int dtype,
                       float *acc_out, uint64_t lo, uint64_t hi)
{
    for (uint64_t e = lo; e < hi; ++e) {
        float acc = contribution(g, dtype, 0, e);
        for (uint32_t r = 1; r < n_contrib; ++r)
            acc = acc + contribution(g, dtype, r, e);
        acc_out[e] = acc;
    }
}

/* Gradient accumulation over micro-batches (Limitations: several micro-batches
 * before one synchronisation).  Each call adds one micro-batch: its N
 * contributions are summed in the fixed order, then that sum is added to the
 * running binary32 total; the first micro-batch (overwrite != 0) stores its sum. */
void oracle_accumulate(const void *const *g, uint32_t n_contrib, int dtype,
                       float *accum, int overwrite, uint64_t lo, uint64_t hi)
{
    for (uint64_t e = lo; e < hi; ++e) {
        float acc = contribution(g, dtype, 0, e);
        for (uint32_t r = 1; r < n_contrib; ++r)
            acc = acc + contribution(g, dtype, r, e);
        accum[e] = overwrite ? acc : accum[e] + acc;
    }
}

/* Mean gradient g = acc * gs and the sum of its squares, the latter summed
 * sequentially in binary64 (each product of two widened binary32 values is
 * exact in binary64).  g_out may be NULL.  Returns the sum over [lo, hi). */
double oracle_mean_sumsq(const void *const *g, uint32_t n_contrib, int dtype,
                         float gs, float *g_out, uint64_t lo, uint64_t hi)
{
    double ss = 0.0;
    for (uint64_t e = lo; e < hi; ++e) {
        float acc = contribution(g, dtype, 0, e);
        for (uint32_t r = 1; r < n_contrib; ++r)
            acc = acc + contribution(g, dtype, r, e);
        float gm = acc * gs;
        if (g_out)
            g_out[e] = gm;
        ss += (double)gm * (double)gm;
    }
    return ss;
}

/* Global-norm clip coefficient in binary64: min(1, max_norm / (norm + 1e-6))
 * with norm the 2-norm of the mean gradient over all devices' shards. */
double oracle_clip_coef(double sumsq_local, double sumsq_others, double max_norm)
{
    double norm = sqrt(sumsq_local + sumsq_others);
    double c = max_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ---- the step, binary32 (the parity target) ---- */

/* One step on elements [lo, hi) of the full-length arrays.  theta, m, v are
 * updated in place; p receives the 16-bit image of the new theta: bf16, or
 * binary16 when p_f16 != 0. */
void oracle_step_f32(const void *const *g, uint32_t n_contrib, int dtype,
                     const oracle_scalars *s, float *theta, float *m, float *v,
                     uint16_t *p, int p_f16, uint64_t lo, uint64_t hi)
{
    for (uint64_t e = lo; e < hi; ++e) {
        float acc = contribution(g, dtype, 0, e);
        for (uint32_t r = 1; r < n_contrib; ++r)
            acc = acc + contribution(g, dtype, r, e);
        float gm = acc * s->gs;
        gm = gm * s->cc;
        float m1 = fmaf(s->b1, m[e], s->omb1 * gm);
        float v1 = fmaf(s->b2, v[e], (s->omb2 * gm) * gm);
        float den = fmaf(sqrtf(v1), s->isb2, s->ep);
        float u = m1 / den;
        float th = fmaf(-s->lw, theta[e], theta[e]);
        float t1 = fmaf(-s->step, u, th);
        m[e] = m1;
        v[e] = v1;
        theta[e] = t1;
        p[e] = p_f16 ? oracle_f16_rne(t1) : oracle_bf16_rne(t1);
    }
}

/* ---- the step, binary64 (a bound on the binary32 op order, not a target) ---- */

/* Same formulas with every scalar and operation in binary64 and the binary32
 * inputs widened; nothing is rounded to binary32.  Outputs go to separate
 * double arrays. */
void oracle_step_f64(const void *const *g, uint32_t n_contrib, int dtype,
                     double lr, double beta1, double beta2, double eps,
                     double weight_decay, uint64_t t, double grad_scale,
                     double clip_coef, const float *theta, const float *m,
                     const float *v, double *theta_out, double *m_out,
                     double *v_out, uint64_t lo, uint64_t hi)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    double gs = grad_scale > 0.0 ? grad_scale : 1.0 / (double)n_contrib;
    double cc = clip_coef > 0.0 ? clip_coef : 1.0;
    for (uint64_t e = lo; e < hi; ++e) {
        double acc = 0.0;
        for (uint32_t r = 0; r < n_contrib; ++r)
            acc += (double)contribution(g, dtype, r, e);
        double gm = acc * gs * cc;
        double m1 = beta1 * (double)m[e] + (1.0 - beta1) * gm;
        double v1 = beta2 * (double)v[e] + (1.0 - beta2) * gm * gm;
        double mhat = m1 / bc1;
        double vhat = v1 / bc2;
        double th = (double)theta[e];
        th = th - lr * weight_decay * th;
        th = th - lr * mhat / (sqrt(vhat) + eps);
        m_out[e] = m1;
        v_out[e] = v1;
        theta_out[e] = th;
    }
}

/* ---- verification protocol (Section 7.1: gradient integrity check, identical
 * checksums after a collective) ---- */

/* Sums for the relative gradient difference ||a - b|| / ||a||: out[0] = sum of
 * (a-b)^2, out[1] = sum of a^2, both sequential in binary64 (the difference of
 * two widened 16- or 32-bit values is exact in binary64). */
void oracle_diff_sumsq(const void *a, const void *b, int dtype, uint64_t lo,
                       uint64_t hi, double *out)
{
    const void *pa[1] = {a}, *pb[1] = {b};
    double sd = 0.0, sa = 0.0;
    for (uint64_t e = lo; e < hi; ++e) {
        double x = (double)contribution(pa, dtype, 0, e);
        double y = (double)contribution(pb, dtype, 0, e);
        double d = x - y;
        sd += d * d;
        sa += x * x;
    }
    out[0] = sd;
    out[1] = sa;
}

/* Position-sensitive 64-bit checksum of a buffer of 8-byte words: word i (index
 * counted from first_index) contributes the splitmix64 output function
 * (Steele, Lea, Flood 2014) of w_i + (i+1) * 0x9E3779B97F4A7C15; the contributions
 * are added modulo 2^64, so any summation order gives the same value and
 * checksums of consecutive pieces add up. */
uint64_t oracle_checksum(const uint64_t *w, uint64_t n_words, uint64_t first_index)
{
    uint64_t c = 0;
    for (uint64_t i = 0; i < n_words; ++i) {
        uint64_t z = w[i] + (first_index + i + 1) * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z = z ^ (z >> 31);
        c += z;
    }
    return c;
}
