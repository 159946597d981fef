/*
 * gs_oracle.c -- plain scalar CPU oracle for the per-layer optimizer step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.  It shares no code, header, table or constant
 * with the HIP library; it is written from the paper's description of the step and from
 * the textbook definition of AdamW the paper cites (Kingma & Ba for Adam; decoupled decay).
 *
 * What the step is, per the paper:
 *   - gradients of all micro-batches of a layer are accumulated in full precision
 *     (Sec. 2.1 "Gradient accumulation"; Sec. 1 footnote on the full-precision buffer);
 *   - gradient clipping needs the global L2 norm over all gradients (Sec. 2.1
 *     "Pipelined optimizer step");
 *   - each weight has three full-precision states: master parameter, momentum, variance
 *     (Sec. 2.2, last paragraph), updated element-wise (Sec. 2.1 "Vanilla LLM training");
 *   - the updated master parameter is converted to low precision to refresh the working
 *     parameter (Sec. 2.2, optimizer step (4) of Fig. 2(c));
 *   - the step is element-wise, so any chunk / partition of the range gives the same
 *     result (Sec. 2.2; Sec. 4.4 delay ratio alpha; Sec. 6.5 partition-independent results).
 *
 * The paper prints none of the arithmetic.  The readings taken here (all listed in the
 * design document): AdamW with decoupled decay applied multiplicatively to the old master
 * weight; eps added outside the square root after bias correction; bias corrections
 * 1-beta^t formed in double on the host and rounded to float once; micro-batch gradients
 * are SUMMED (no 1/k) in fp32, j ascending, starting from +0; clip coefficient
 * c = min(1, max_norm / (norm + 1e-6)), no clipping when max_norm <= 0; bf16 output by
 * round-to-nearest-even.
 *
 * Two variants of the element update:
 *   gs_oracle_accum_adamw      fp32 reference order, one rounding per operation, no FMA
 *                              contraction (build with -ffp-contract=off);
 *   gs_oracle_accum_adamw_f64  the same formulas evaluated in double from the same fp32
 *                              inputs, results left in double ("truth" that arbitrates).
 *
 * Build:  gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC gs_oracle.c -o libgs_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- bf16 <-> fp32 (storage format: upper 16 bits of an IEEE binary32) ---------------- */

float gs_oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round-to-nearest, ties-to-even.  NaN stays NaN (quiet bit forced so that a payload living
 * only in the discarded low half cannot turn into Inf).  Finite values above the largest
 * bf16 round to Inf, as RNE prescribes. */
uint16_t gs_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7fffu + keep_lsb;
    return (uint16_t)(u >> 16);
}

/* ---- a1: widen + k-way accumulate (Sec. 2.1 "Gradient accumulation") ------------------- */

static float accumulate_f32(const uint16_t *const *grads, int k, int64_t i)
{
    float a = 0.0f;
    for (int j = 0; j < k; ++j)
        a += gs_oracle_bf16_to_f32(grads[j][i]);
    return a;
}

/* a1 on its own: out[i] = fp32 sum of the k buffers at i, for i in [begin,end). */
void gs_oracle_accumulate(const uint16_t *const *grads, int k, int64_t begin, int64_t end, float *out)
{
    for (int64_t i = begin; i < end; ++i)
        out[i] = accumulate_f32(grads, k, i);
}

/* a1 as the paper runs it (Sec. 3.4, Sec. 4.3: one full-precision accumulation buffer per layer
 * on the GPU; each micro-batch's backward adds its gradient into it):
 *   acc[i] = (first ? +0 : acc[i]) + widen(grad[i])   for i in [begin,end).
 * Returns the squared L2 norm (double) of the updated acc over the range. */
double gs_oracle_accum_add(float *acc, const uint16_t *grad, int first, int64_t begin, int64_t end)
{
    double S = 0.0;
    for (int64_t i = begin; i < end; ++i) {
        float base = first ? 0.0f : acc[i];
        float a = base + gs_oracle_bf16_to_f32(grad[i]);
        acc[i] = a;
        double ad = (double)a;
        S += ad * ad;
    }
    return S;
}

/* a2 on a finished accumulation buffer: sum of acc[i]^2 over [begin,end), squares and sum in double. */
double gs_oracle_acc_sqnorm(const float *acc, int64_t begin, int64_t end)
{
    double S = 0.0;
    for (int64_t i = begin; i < end; ++i) {
        double x = (double)acc[i];
        S += x * x;
    }
    return S;
}

/* ---- a2: squared L2 norm of the accumulated gradient over [begin,end) ------------------ */
/* (Sec. 2.1: clipping needs the global L2 norm.)  Each square is exact in double. */
double gs_oracle_grad_sqnorm(const uint16_t *const *grads, int k, int64_t begin, int64_t end)
{
    double S = 0.0;
    for (int64_t i = begin; i < end; ++i) {
        float a = accumulate_f32(grads, k, i);
        S += (double)a * (double)a;
    }
    return S;
}

/* ---- a3: clip coefficient from the TOTAL squared norm ---------------------------------- */
float gs_oracle_clip_coef(double sqnorm_total, float max_norm)
{
    if (!(max_norm > 0.0f))
        return 1.0f;
    float norm = (float)sqrt(sqnorm_total);
    float c = max_norm / (norm + 1e-6f);
    /* Compare-select, so a NaN norm gives c = 1 (the NaN gradient element itself still
     * poisons its own state); an infinite norm gives c = 0. */
    return c < 1.0f ? c : 1.0f;
}

/* Hyper-parameters as the caller states them. */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float max_grad_norm;
    int32_t step;
} gs_oracle_hparams;

/* Per-step constants: formed in double, rounded to float once. */
typedef struct {
    float beta1, beta2, omb1, omb2, eps, step_size, rsbc2, decay;
} step_consts_f32;

static step_consts_f32 make_consts(const gs_oracle_hparams *hp)
{
    step_consts_f32 s;
    double b1 = (double)hp->beta1, b2 = (double)hp->beta2;
    double bc1 = 1.0 - pow(b1, (double)hp->step);
    double bc2 = 1.0 - pow(b2, (double)hp->step);
    s.beta1 = hp->beta1;
    s.beta2 = hp->beta2;
    s.omb1 = (float)(1.0 - b1);
    s.omb2 = (float)(1.0 - b2);
    s.eps = hp->eps;
    s.step_size = (float)((double)hp->lr / bc1);
    s.rsbc2 = (float)sqrt(bc2);
    s.decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);
    return s;
}

/* ---- a1 + a3..a6 over [begin,end), fp32 reference order -------------------------------- */
/* p, m, v updated in place; w (bf16) written.  c is the clip coefficient (1.0f = none). */
void gs_oracle_accum_adamw(float *p, float *m, float *v, uint16_t *w,
                           const uint16_t *const *grads, int k,
                           int64_t begin, int64_t end,
                           const gs_oracle_hparams *hp, float c)
{
    const step_consts_f32 s = make_consts(hp);
    for (int64_t i = begin; i < end; ++i) {
        float a = accumulate_f32(grads, k, i);
        float g = c * a;
        float t1 = s.beta1 * m[i];
        float t2 = s.omb1 * g;
        float mn = t1 + t2;
        float gg = g * g;
        float t3 = s.beta2 * v[i];
        float t4 = s.omb2 * gg;
        float vn = t3 + t4;
        float d = sqrtf(vn) / s.rsbc2;
        d = d + s.eps;
        float u = mn / d;
        float t5 = p[i] * s.decay;
        float t6 = s.step_size * u;
        float pn = t5 - t6;
        m[i] = mn;
        v[i] = vn;
        p[i] = pn;
        w[i] = gs_oracle_f32_to_bf16(pn);
    }
}

/* ---- the same step in double ("truth") -------------------------------------------------- */
/* Inputs are the fp32 states and bf16 gradients; outputs are the unrounded double results.
 * The clip coefficient is recomputed in double from sqnorm_total (pass a negative
 * sqnorm_total for "no clipping").  Nothing is rounded to float on the way. */
void gs_oracle_accum_adamw_f64(const float *p, const float *m, const float *v,
                               double *p_out, double *m_out, double *v_out,
                               const uint16_t *const *grads, int k,
                               int64_t begin, int64_t end,
                               const gs_oracle_hparams *hp, double sqnorm_total)
{
    double b1 = (double)hp->beta1, b2 = (double)hp->beta2;
    double lr = (double)hp->lr, wd = (double)hp->weight_decay, eps = (double)hp->eps;
    double bc1 = 1.0 - pow(b1, (double)hp->step);
    double bc2 = 1.0 - pow(b2, (double)hp->step);
    double c = 1.0;
    if (hp->max_grad_norm > 0.0f && sqnorm_total >= 0.0) {
        c = (double)hp->max_grad_norm / (sqrt(sqnorm_total) + 1e-6);
        if (c > 1.0) c = 1.0;
    }
    for (int64_t i = begin; i < end; ++i) {
        double a = 0.0;
        for (int j = 0; j < k; ++j)
            a += (double)gs_oracle_bf16_to_f32(grads[j][i]);
        double g = c * a;
        double mn = b1 * (double)m[i] + (1.0 - b1) * g;
        double vn = b2 * (double)v[i] + (1.0 - b2) * g * g;
        double mhat = mn / bc1;
        double vhat = vn / bc2;
        double pn = (double)p[i] * (1.0 - lr * wd) - lr * mhat / (sqrt(vhat) + eps);
        p_out[i] = pn;
        m_out[i] = mn;
        v_out[i] = vn;
    }
}
