/*
 * CheckFree recovery -- CPU oracle.  TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, obviously-correct statement of what the recovery hot path
 * computes, used only by the test-suite, by the smoke check and by the
 * benchmark's CPU-baseline leg.  It shares no code, header, table or helper
 * with the HIP library and must never be called from it.
 *
 * What is stated here (paper: section "CheckFree: Memoryless Recovery"):
 *
 *   omega_i  = || grad W^S_i ||^2        sum of squares of every gradient element
 *                                        of every tensor of stage i
 *                                        (definition of omega_{i-1}, omega_{i+1}
 *                                        in that section; Algorithm 1, the two
 *                                        "Receive" steps)
 *
 *   W^S_i    = (omega_{i-1} * W^S_{i-1} + omega_{i+1} * W^S_{i+1})
 *              / (omega_{i-1} + omega_{i+1})
 *                                        the display equation of that section.
 *                                        (Algorithm 1's third step prints
 *                                        omega_{i-1} on both terms; the display
 *                                        equation is taken as authoritative,
 *                                        because only it is consistent with the
 *                                        section's own special cases: a zero
 *                                        omega_{i+1} reduces it to a copy of
 *                                        the previous stage, equal omegas to
 *                                        the uniform average.)
 *
 *   copy     : CheckFree+ (section "CheckFree+: First and Last Stage
 *              Recovery") restores a first/last stage from its neighbour and
 *              the (de)embedding from a replica without any loss: a bytewise
 *              copy.
 *
 * Arithmetic: all floating point in IEEE binary64, evaluated literally in the
 * order the formulas are written (compile with -ffp-contract=off so that no
 * multiply-add is fused), one rounding to the storage type at the end.
 *
 * Where the paper is silent (omega sum zero, negative or not finite) the
 * reading taken is the unweighted variant the section itself mentions, the uniform average:
 * both weights are replaced by 1.  cfo_effective_omega states that rule.
 *
 * Pins: tests/test_oracle_*.py check every function against closed forms,
 * invariants and exact rational arithmetic.  The degenerate-omega rule is a
 * reading of ours, not the paper's: parity unpinned for that rule alone.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* omega: squared L2 norm, binary64 accumulation, index order          */
/* ------------------------------------------------------------------ */

/* Sum of squares of one fp32 tensor, elements taken in index order: one
 * tensor's share of omega = ||grad W^S||^2 (section "CheckFree: Memoryless
 * Recovery", definition of omega_{i-1}, omega_{i+1}). */
double cfo_sqnorm_f32(const float *g, uint64_t n)
{
    double acc = 0.0;
    for (uint64_t k = 0; k < n; ++k) {
        double v = (double)g[k];
        acc += v * v;
    }
    return acc;
}

static double bf16_to_f64(uint16_t h);

/* The same share of omega for a bfloat16 gradient tensor (bit patterns),
 * elements in index order. */
double cfo_sqnorm_bf16(const uint16_t *g, uint64_t n)
{
    double acc = 0.0;
    for (uint64_t k = 0; k < n; ++k) {
        double v = bf16_to_f64(g[k]);
        acc += v * v;
    }
    return acc;
}

/* omega of a stage: the squared norm of ALL its gradient elements, i.e. the
 * tensors' sums of squares added in list order (section "Problem Statement":
 * a stage's weights are the combination of its layers' weights; section
 * "CheckFree: Memoryless Recovery": omega is the squared gradient norm of
 * the stage). */
double cfo_stage_sqnorm_f32(const float *const *tensors, const uint64_t *numel,
                            uint32_t num_tensors)
{
    double omega = 0.0;
    for (uint32_t t = 0; t < num_tensors; ++t)
        omega += cfo_sqnorm_f32(tensors[t], numel[t]);
    return omega;
}

/* Same definition, the index range of each tensor cut into `threads`
 * contiguous pieces; the pieces' sums are added in piece order.  Only the
 * association of the binary64 additions differs from cfo_stage_sqnorm_f32. */
double cfo_stage_sqnorm_f32_mt(const float *const *tensors, const uint64_t *numel,
                               uint32_t num_tensors, int threads)
{
    if (threads < 1) threads = 1;
    if (threads > 1024) threads = 1024;
    double omega = 0.0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        double piece[1024];
        const float *g = tensors[t];
        uint64_t n = numel[t];
#pragma omp parallel for num_threads(threads) schedule(static, 1)
        for (int p = 0; p < threads; ++p) {
            uint64_t lo = n / (uint64_t)threads * (uint64_t)p;
            uint64_t hi = (p == threads - 1) ? n : n / (uint64_t)threads * (uint64_t)(p + 1);
            piece[p] = cfo_sqnorm_f32(g + lo, hi - lo);
        }
        for (int p = 0; p < threads; ++p) omega += piece[p];
    }
    return omega;
}

/* ------------------------------------------------------------------ */
/* weights                                                              */
/* ------------------------------------------------------------------ */

/* The weights the blend uses.  Returns 0 and passes the omegas through when
 * both are finite and non-negative and their binary64 sum is a positive normal
 * number; otherwise returns 1 and substitutes the uniform average (1, 1). */
int cfo_effective_omega(double omega_prev, double omega_next, double *eff_prev, double *eff_next)
{
    double d = omega_prev + omega_next;
    int ok = isfinite(omega_prev) && isfinite(omega_next) && omega_prev >= 0.0 &&
             omega_next >= 0.0 && isfinite(d) && d >= 2.2250738585072014e-308;
    if (ok) {
        *eff_prev = omega_prev;
        *eff_next = omega_next;
        return 0;
    }
    *eff_prev = 1.0;
    *eff_next = 1.0;
    return 1;
}

/* The display equation of section "CheckFree: Memoryless Recovery" is a ratio
 * of two expressions linear in (omega_{i-1}, omega_{i+1}): multiplying both
 * omegas by one positive number leaves W^S_i unchanged.  The blend uses that
 * freedom once, before any element is touched: both weights are multiplied by
 * the power of two that brings their binary64 sum into [1, 2).  A power of two
 * changes no significand, so wherever the unscaled formula stays inside the
 * binary64 range the scaled one gives the same bits; where it would not (omegas
 * near 1e300 or 1e-300 against weights of ordinary size) the scaled one still
 * gives the value of the equation. */
void cfo_common_scale(double *wp, double *wn)
{
    int e;
    (void)frexp(*wp + *wn, &e);       /* sum = m * 2^e, m in [0.5, 1) */
    *wp = ldexp(*wp, 1 - e);
    *wn = ldexp(*wn, 1 - e);
}

/* The display equation of section "CheckFree: Memoryless Recovery" for one
 * element, in binary64, written as printed: weighted sum of the two
 * neighbours' values over the sum of the weights. */
static double blend_value(double wp, double wn, double a, double b)
{
    double numerator = wp * a + wn * b;
    double denominator = wp + wn;
    return numerator / denominator;
}

/* ------------------------------------------------------------------ */
/* bfloat16 <-> binary64                                               */
/* ------------------------------------------------------------------ */

/* bfloat16 is the upper half of a binary32; widening is exact. */
static double bf16_to_f64(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* binary64 -> bfloat16, round to nearest, ties to even, in one rounding.
 * bfloat16: 1 sign, 8 exponent bits (bias 127), 7 fraction bits; subnormals
 * are kept (quantum 2^-133).  Relies on the default rounding mode. */
static uint16_t f64_to_bf16(double x)
{
    if (isnan(x)) return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double ax = fabs(x);
    if (ax == 0.0) return sign;
    if (isinf(ax)) return (uint16_t)(sign | 0x7F80u);
    int e;
    (void)frexp(ax, &e);          /* ax in [2^(e-1), 2^e) */
    int E = e - 1;                /* exponent of the leading bit */
    if (E < -126) E = -126;       /* subnormal range: fixed quantum */
    double scaled = ldexp(ax, 7 - E);     /* exact; [128,256) if normal */
    double r = nearbyint(scaled);         /* ties to even */
    if (r >= 256.0) { r = 128.0; E += 1; }
    if (E > 127) return (uint16_t)(sign | 0x7F80u);
    if (r < 128.0) return (uint16_t)(sign | (uint16_t)r);            /* subnormal or zero */
    return (uint16_t)(sign | (uint16_t)((E + 127) << 7) | ((uint16_t)r - 128u));
}

/* Exposed so the tests can pin the conversions on their own. */
double cfo_bf16_to_f64(uint16_t h) { return bf16_to_f64(h); }
uint16_t cfo_f64_to_bf16(double x) { return f64_to_bf16(x); }

/* ------------------------------------------------------------------ */
/* blend: one tensor                                                    */
/* ------------------------------------------------------------------ */

/* W^S_i for one fp32 tensor pair: the display equation element by element,
 * rounded once to binary32 (Algorithm 1, third step, with the display
 * equation's weights). */
void cfo_blend_f32(double omega_prev, double omega_next, const float *prev, const float *next,
                   float *out, uint64_t n, int threads)
{
    double wp, wn;
    cfo_effective_omega(omega_prev, omega_next, &wp, &wn);
    cfo_common_scale(&wp, &wn);
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (uint64_t k = 0; k < n; ++k)
        out[k] = (float)blend_value(wp, wn, (double)prev[k], (double)next[k]);
}

/* The same for a bfloat16 tensor pair, rounded once to bfloat16. */
void cfo_blend_bf16(double omega_prev, double omega_next, const uint16_t *prev,
                    const uint16_t *next, uint16_t *out, uint64_t n, int threads)
{
    double wp, wn;
    cfo_effective_omega(omega_prev, omega_next, &wp, &wn);
    cfo_common_scale(&wp, &wn);
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (uint64_t k = 0; k < n; ++k)
        out[k] = f64_to_bf16(blend_value(wp, wn, bf16_to_f64(prev[k]), bf16_to_f64(next[k])));
}

/* The unrounded binary64 value of the blend (no final narrowing), for the
 * linearity and exact-arithmetic pins. */
void cfo_blend_f64(double omega_prev, double omega_next, const double *prev, const double *next,
                   double *out, uint64_t n)
{
    double wp, wn;
    cfo_effective_omega(omega_prev, omega_next, &wp, &wn);
    cfo_common_scale(&wp, &wn);
    for (uint64_t k = 0; k < n; ++k) out[k] = blend_value(wp, wn, prev[k], next[k]);
}

/* ------------------------------------------------------------------ */
/* copy                                                                 */
/* ------------------------------------------------------------------ */

/* CheckFree+ (section "CheckFree+: First and Last Stage Recovery"): an end
 * stage from its neighbour, embedding and de-embedding from their replicas,
 * without loss: the bytes of src, unchanged. */
void cfo_copy_bytes(void *dst, const void *src, uint64_t nbytes, int threads)
{
    if (threads <= 1) {
        memcpy(dst, src, nbytes);
        return;
    }
#pragma omp parallel for num_threads(threads) schedule(static, 1)
    for (int p = 0; p < threads; ++p) {
        uint64_t lo = nbytes / (uint64_t)threads * (uint64_t)p;
        uint64_t hi = (p == threads - 1) ? nbytes : nbytes / (uint64_t)threads * (uint64_t)(p + 1);
        memcpy((char *)dst + lo, (const char *)src + lo, hi - lo);
    }
}

/* One slice of a replica refresh (section "CheckFree+: First and Last Stage
 * Recovery", last paragraph: the neighbouring stages hold copies of the
 * embedding and de-embedding layers; a copy stays current only if it is made
 * again every iteration, and it may be made piece by piece): `count` elements
 * of `elem_bytes` bytes each, from element `first` on, carried from src to dst;
 * every other byte of dst stays as it was. */
void cfo_copy_range(void *dst, const void *src, uint64_t first, uint64_t count, uint32_t elem_bytes)
{
    const char *s = (const char *)src + first * elem_bytes;
    char *d = (char *)dst + first * elem_bytes;
    for (uint64_t k = 0; k < count * elem_bytes; ++k) d[k] = s[k];
}

/* ------------------------------------------------------------------ */
/* omega as a by-product of the optimizer step                          */
/* ------------------------------------------------------------------ */

/* The paper trains with Adam, no weight decay, betas (0.9, 0.999) (appendix
 * "Optimizers"), and every stage keeps omega = ||grad W^S||^2 of its last
 * gradient (section "CheckFree: Memoryless Recovery").  The optimizer step is
 * the one pass of an iteration that reads every gradient element anyway, so
 * omega can leave it as a by-product.  This is that step for one fp32 tensor,
 * written as Adam is defined (Kingma & Ba, "Adam: A Method for Stochastic
 * Optimization", Algorithm 1), t counted from 1:
 *
 *     m_t = beta1 m_{t-1} + (1 - beta1) g
 *     v_t = beta2 v_{t-1} + (1 - beta2) g^2
 *     mhat = m_t / (1 - beta1^t),  vhat = v_t / (1 - beta2^t)
 *     w_t = w_{t-1} - lr * mhat / (sqrt(vhat) + eps)
 *
 * Readings where paper and definition leave room: the moments and the weights
 * are stored in binary32; all arithmetic is binary64; m_t and v_t are rounded
 * once to binary32 when stored and the weight update uses those stored values
 * (what a later step, or anyone else, would read back); w_t is rounded once.
 * eps is added to the square root, outside it.  Returns this tensor's share
 * of omega, the sum of g^2 in index order. */
double cfo_adam_step_f32(float *w, float *m, float *v, const float *g, uint64_t n, double lr,
                         double beta1, double beta2, double eps, uint64_t t)
{
    double correction1 = 1.0 - pow(beta1, (double)t);
    double correction2 = 1.0 - pow(beta2, (double)t);
    double omega = 0.0;
    for (uint64_t k = 0; k < n; ++k) {
        double grad = (double)g[k];
        omega += grad * grad;
        m[k] = (float)(beta1 * (double)m[k] + (1.0 - beta1) * grad);
        v[k] = (float)(beta2 * (double)v[k] + (1.0 - beta2) * (grad * grad));
        double mhat = (double)m[k] / correction1;
        double vhat = (double)v[k] / correction2;
        w[k] = (float)((double)w[k] - lr * mhat / (sqrt(vhat) + eps));
    }
    return omega;
}

int cfo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
