/*
 * abs_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, CPU-only statement of what the ABS-SGD data-parallel hot path
 * computes.  It exists only so that tests, the smoke check and the benchmark's
 * CPU-baseline leg can compare the GPU library against it.  It shares no code,
 * header, table or helper with the HIP library and must never be called from
 * the product path.
 *
 * What it follows (ABS-SGD paper, Section "Algorithm", Algorithm 1):
 *   - Step 2, initialisation:  G_t^i = 0,  M_t^i = 0.
 *   - Step 2, inner loop:      G_t^i += (sum of the per-sample gradients of one
 *                              reference batch);  M_t^i += M_r.
 *   - Step 1:                  Gbar_{t-1} = (sum_i G_{t-1}^i) / (sum_i M_{t-1}^i)
 *                              (the weighted gradient averaging mechanism).
 *   - Update:                  x_{t+1} = x_t - gamma * Gbar_{t-1}   (delay of one
 *                              iteration; heterogeneous-aware delayed synchronous
 *                              parallel mechanism).
 * The paper uses plain SGD (Section "Conclusions and Future Work").  The task this
 * oracle serves asks for momentum SGD with weight decay on top of it; the
 * conventional coupled form is used,
 *       d = Gbar + wd*x ;  v = mu*v + d ;  x = x - gamma*v ,
 * which is exactly the paper's rule when mu = 0 and wd = 0.
 *
 * A reference batch arrives as its MEAN gradient g (what a backward pass over
 * M_r samples of a mean-reduced loss yields), so the sum of its per-sample
 * gradients is M_r * g.
 *
 * Delayed gradient compensation (Section "Algorithm", third mechanism; the
 * compensation line of Algorithm 1):
 *       Gtilde_t = Gbar_{t-1} + lambda * Gbar_{t-1} (.) Gbar_{t-1} (.) (x_t - x_{t-1})
 * element-wise, applied in place of Gbar in the update.  The paper states it for
 * plain SGD; with momentum and weight decay the compensated gradient takes
 * Gbar's place (compensate first, then weight decay, then momentum).  The
 * functions with the suffix _dc keep x_{t-1} in a buffer of their own, as the
 * paper's remark on memory overhead implies.  The functions with the suffix
 * _dcm state the same correction without that buffer: every applied update is
 * x_t = x_{t-1} - gamma_{t-1} * v_t, so x_t - x_{t-1} = -gamma_{t-1} * v_t with
 * v_t the momentum as it stands before this update (gamma_{t-1} = 0 when the
 * previous iteration applied nothing).  Equal to the _dc form in exact
 * arithmetic; the CPU tests pin one against the other.
 *
 * Adam variant (the paper's Section "Conclusions and Future Work" names Adam as
 * the next update rule to put behind the delayed synchronous mechanism; the
 * paper does not spell it out).  Here it is the standard Adam recursion driven
 * by the delayed weighted average, with coupled weight decay:
 *       g = Gbar + wd*x;  m = b1*m + (1-b1)*g;  v = b2*v + (1-b2)*g*g;
 *       x = x - gamma * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps),
 * t = 1, 2, ... counting the updates actually applied.
 *
 * LARS variant (the other rule named in "Conclusions and Future Work"; not spelt
 * out by the paper).  The published layer-wise rule, per tensor ("layer") l, driven
 * by the delayed weighted average g_l = Gbar restricted to the layer:
 *       rate_l = eta * ||x_l|| / (||g_l|| + wd * ||x_l||)   (1 when either norm is 0)
 *       v_l = mu * v_l + gamma * rate_l * (g_l + wd * x_l);   x_l = x_l - v_l
 * with Euclidean norms over the layer.
 *
 * Precision: everything in IEEE double.  Inputs (fp32 or bf16 gradients, fp32
 * hyper-parameters) are widened exactly before use.
 *
 * A second family, oracle32_*, restates the same steps in fp32 with one fixed
 * operation order so that an fp32 implementation following that order can be
 * compared bit for bit.  It is pinned against the double family in the CPU
 * tests; it is not the judge of accuracy, the double family is.
 *
 * The loops over the n parameters are independent per element; the only
 * parallelism is "#pragma omp parallel for" over that index.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- helpers ----------------------------------------------------------- */

/* bfloat16 is the upper half of an IEEE binary32: widening is a 16-bit shift. */
static inline float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- double family: the definition ------------------------------------ */

/* Algorithm 1, Step 2, initialisation: G_t^i = 0. (M_t^i = 0 is the caller's
 * integer.) */
void oracle_zero(double *G, int64_t n_params)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_params; ++i) G[i] = 0.0;
}

/* Algorithm 1, Step 2, inner loop, one reference batch of M_r samples whose
 * mean gradient is g (fp32): G += M_r * g.  The caller adds M_r to M_t^i. */
void oracle_accumulate_f32(double *G, const float *g, int64_t n_params, int64_t M_r)
{
    const double m = (double)M_r;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_params; ++i) G[i] += m * (double)g[i];
}

/* Same, gradient stored as bfloat16 bit patterns. */
void oracle_accumulate_bf16(double *G, const uint16_t *g, int64_t n_params, int64_t M_r)
{
    const double m = (double)M_r;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_params; ++i)
        G[i] += m * (double)bf16_bits_to_float(g[i]);
}

/* Algorithm 1, Step 1 + parameter update, with the delayed accumulators
 * G[0..N-1] and batch sizes M[0..N-1] of the previous iteration.
 * Returns 1 and touches nothing when sum(M) == 0 (G_{-1} = 0 with no batch
 * size defined: the first iteration applies nothing); else returns 0.
 * Workers with M[i] == 0 hold G[i] == 0 by the initialisation above, so the
 * plain sum over all N workers is the definition. */
int oracle_sync_update(double *x, double *v, const double *const *G, const int64_t *M,
                       int N, int64_t n_params, double gamma, double mu, double wd)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const double Mt = (double)M_total;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        double s = 0.0;
        for (int i = 0; i < N; ++i) s += G[i][j];
        const double Gbar = s / Mt;
        const double d = Gbar + wd * x[j];
        v[j] = mu * v[j] + d;
        x[j] = x[j] - gamma * v[j];
    }
    return 0;
}

/* Same with the delayed gradient compensation.  x_prev holds x_{t-1} on entry
 * (equal to x when no update has been applied yet, so the correction vanishes
 * at the first applied step) and x_t on return -- also when sum(M) == 0, in
 * which case x_{t+1} = x_t and the function returns 1. */
int oracle_sync_update_dc(double *x, double *x_prev, double *v, const double *const *G,
                          const int64_t *M, int N, int64_t n_params, double gamma, double mu,
                          double wd, double lambda)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) {
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n_params; ++j) x_prev[j] = x[j];
        return 1;
    }
    const double Mt = (double)M_total;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        double s = 0.0;
        for (int i = 0; i < N; ++i) s += G[i][j];
        const double Gbar = s / Mt;
        const double Gtilde = Gbar + lambda * Gbar * Gbar * (x[j] - x_prev[j]);
        const double d = Gtilde + wd * x[j];
        v[j] = mu * v[j] + d;
        x_prev[j] = x[j];
        x[j] = x[j] - gamma * v[j];
    }
    return 0;
}

/* Compensation with x_t - x_{t-1} taken from the momentum: gamma_prev is the
 * step size of the previous applied update, 0 when the previous iteration
 * applied none (then x_t = x_{t-1}).  Returns 1 and touches nothing when
 * sum(M) == 0. */
int oracle_sync_update_dcm(double *x, double *v, const double *const *G, const int64_t *M, int N,
                           int64_t n_params, double gamma, double mu, double wd, double lambda,
                           double gamma_prev)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const double Mt = (double)M_total;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        double s = 0.0;
        for (int i = 0; i < N; ++i) s += G[i][j];
        const double Gbar = s / Mt;
        const double diff = -(gamma_prev * v[j]);
        const double Gtilde = Gbar + lambda * Gbar * Gbar * diff;
        const double d = Gtilde + wd * x[j];
        v[j] = mu * v[j] + d;
        x[j] = x[j] - gamma * v[j];
    }
    return 0;
}

/* Adam driven by the delayed weighted average.  step >= 1 is the index of this
 * update among the applied ones.  Returns 1 and touches nothing when
 * sum(M) == 0. */
int oracle_sync_update_adam(double *x, double *m, double *v, const double *const *G,
                            const int64_t *M, int N, int64_t n_params, double gamma, double beta1,
                            double beta2, double eps, double wd, int64_t step)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const double Mt = (double)M_total;
    const double bc1 = 1.0 - pow(beta1, (double)step);
    const double bc2 = 1.0 - pow(beta2, (double)step);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        double s = 0.0;
        for (int i = 0; i < N; ++i) s += G[i][j];
        const double g = s / Mt + wd * x[j];
        m[j] = beta1 * m[j] + (1.0 - beta1) * g;
        v[j] = beta2 * v[j] + (1.0 - beta2) * g * g;
        const double mhat = m[j] / bc1;
        const double vhat = v[j] / bc2;
        x[j] = x[j] - gamma * mhat / (sqrt(vhat) + eps);
    }
    return 0;
}

/* LARS over n_tensors consecutive layers of the flat vector; sizes[l] elements each
 * (they sum to n_params).  Returns 1 and touches nothing when sum(M) == 0. */
int oracle_sync_update_lars(double *x, double *v, const double *const *G, const int64_t *M, int N,
                            int n_tensors, const int64_t *sizes, double gamma, double mu, double wd,
                            double eta)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const double Mt = (double)M_total;
    int64_t base = 0;
    for (int l = 0; l < n_tensors; ++l) {
        const int64_t n = sizes[l];
        double xx = 0.0, gg = 0.0;
        for (int64_t j = base; j < base + n; ++j) {
            double s = 0.0;
            for (int i = 0; i < N; ++i) s += G[i][j];
            const double g = s / Mt;
            xx += x[j] * x[j];
            gg += g * g;
        }
        const double xn = sqrt(xx), gn = sqrt(gg);
        const double rate = (xn > 0.0 && gn > 0.0) ? eta * xn / (gn + wd * xn) : 1.0;
        for (int64_t j = base; j < base + n; ++j) {
            double s = 0.0;
            for (int i = 0; i < N; ++i) s += G[i][j];
            const double g = s / Mt;
            v[j] = mu * v[j] + gamma * rate * (g + wd * x[j]);
            x[j] = x[j] - v[j];
        }
        base += n;
    }
    return 0;
}

/* ---- fp32 family with a fixed operation order -------------------------- */

/* first != 0: this is the first reference batch since the accumulator was
 * reset, so G = 0 and the result is the rounded product.  Otherwise one fused
 * multiply-add. */
void oracle32_accumulate_f32(float *G, const float *g, int64_t n_params, int64_t M_r,
                             int first)
{
    const float m = (float)M_r;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_params; ++i)
        G[i] = first ? m * g[i] : fmaf(m, g[i], G[i]);
}

void oracle32_accumulate_bf16(float *G, const uint16_t *g, int64_t n_params, int64_t M_r,
                              int first)
{
    const float m = (float)M_r;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_params; ++i) {
        const float gi = bf16_bits_to_float(g[i]);
        G[i] = first ? m * gi : fmaf(m, gi, G[i]);
    }
}

/* Order: s = G[i0]; s += G[i] for the remaining workers with M[i] > 0 in
 * ascending i; Gbar = s / (float)sum(M) (correctly rounded divide);
 * d = fma(wd, x, Gbar); v = fma(mu, v, d); x = fma(-gamma, v, x). */
int oracle32_sync_update(float *x, float *v, const float *const *G, const int64_t *M, int N,
                         int64_t n_params, float gamma, float mu, float wd)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const float Mt = (float)M_total;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        float s = 0.0f;
        int seen = 0;
        for (int i = 0; i < N; ++i) {
            if (M[i] <= 0) continue;
            s = seen ? s + G[i][j] : G[i][j];
            seen = 1;
        }
        const float Gbar = s / Mt;
        const float d = fmaf(wd, x[j], Gbar);
        const float vn = fmaf(mu, v[j], d);
        v[j] = vn;
        x[j] = fmaf(-gamma, vn, x[j]);
    }
    return 0;
}

/* With compensation.  Order: Gbar as above; q = Gbar * Gbar; c = lambda * q;
 * diff = x - x_prev; Gtilde = fma(c, diff, Gbar); d = fma(wd, x, Gtilde);
 * v = fma(mu, v, d); x_prev = x; x = fma(-gamma, v, x). */
int oracle32_sync_update_dc(float *x, float *x_prev, float *v, const float *const *G,
                            const int64_t *M, int N, int64_t n_params, float gamma, float mu,
                            float wd, float lambda)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) {
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n_params; ++j) x_prev[j] = x[j];
        return 1;
    }
    const float Mt = (float)M_total;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        float s = 0.0f;
        int seen = 0;
        for (int i = 0; i < N; ++i) {
            if (M[i] <= 0) continue;
            s = seen ? s + G[i][j] : G[i][j];
            seen = 1;
        }
        const float Gbar = s / Mt;
        const float q = Gbar * Gbar;
        const float c = lambda * q;
        const float diff = x[j] - x_prev[j];
        const float Gtilde = fmaf(c, diff, Gbar);
        const float d = fmaf(wd, x[j], Gtilde);
        const float vn = fmaf(mu, v[j], d);
        v[j] = vn;
        x_prev[j] = x[j];
        x[j] = fmaf(-gamma, vn, x[j]);
    }
    return 0;
}

/* Compensation from the momentum.  Order: Gbar as above; q = Gbar * Gbar;
 * c = lambda * q; diff = (-gamma_prev) * v; Gtilde = fma(c, diff, Gbar);
 * d = fma(wd, x, Gtilde); v = fma(mu, v, d); x = fma(-gamma, v, x). */
int oracle32_sync_update_dcm(float *x, float *v, const float *const *G, const int64_t *M, int N,
                             int64_t n_params, float gamma, float mu, float wd, float lambda,
                             float gamma_prev)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const float Mt = (float)M_total;
    const float ngp = -gamma_prev;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        float s = 0.0f;
        int seen = 0;
        for (int i = 0; i < N; ++i) {
            if (M[i] <= 0) continue;
            s = seen ? s + G[i][j] : G[i][j];
            seen = 1;
        }
        const float Gbar = s / Mt;
        const float q = Gbar * Gbar;
        const float c = lambda * q;
        const float diff = ngp * v[j];
        const float Gtilde = fmaf(c, diff, Gbar);
        const float d = fmaf(wd, x[j], Gtilde);
        const float vn = fmaf(mu, v[j], d);
        v[j] = vn;
        x[j] = fmaf(-gamma, vn, x[j]);
    }
    return 0;
}

/* Adam.  Order: Gbar as above; g = fma(wd, x, Gbar); m = fma(beta1, m, (1-beta1)*g)
 * with (1-beta1) rounded to fp32 first; v = fma(beta2, v, (1-beta2)*(g*g));
 * mh = m / bc1; vh = v / bc2 with bc = (float)(1 - beta^step) evaluated in double
 * from the fp32 betas; den = sqrtf(vh) + eps; x = fma(-gamma, mh / den, x). */
int oracle32_sync_update_adam(float *x, float *m, float *v, const float *const *G,
                              const int64_t *M, int N, int64_t n_params, float gamma, float beta1,
                              float beta2, float eps, float wd, int64_t step)
{
    int64_t M_total = 0;
    for (int i = 0; i < N; ++i) M_total += M[i];
    if (M_total == 0) return 1;
    const float Mt = (float)M_total;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    const float bc1 = (float)(1.0 - pow((double)beta1, (double)step));
    const float bc2 = (float)(1.0 - pow((double)beta2, (double)step));
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_params; ++j) {
        float s = 0.0f;
        int seen = 0;
        for (int i = 0; i < N; ++i) {
            if (M[i] <= 0) continue;
            s = seen ? s + G[i][j] : G[i][j];
            seen = 1;
        }
        const float Gbar = s / Mt;
        const float g = fmaf(wd, x[j], Gbar);
        const float t1 = omb1 * g;
        const float mn = fmaf(beta1, m[j], t1);
        const float g2 = g * g;
        const float t2 = omb2 * g2;
        const float vn = fmaf(beta2, v[j], t2);
        m[j] = mn;
        v[j] = vn;
        const float mh = mn / bc1;
        const float vh = vn / bc2;
        const float den = sqrtf(vh) + eps;
        const float q = mh / den;
        x[j] = fmaf(-gamma, q, x[j]);
    }
    return 0;
}
