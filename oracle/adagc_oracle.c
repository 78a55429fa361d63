/*
 * CPU oracle for one AdaGC optimizer step (arxiv 2502.11034).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It is never part of the product path, it
 * shares no code with the HIP sources, and it is written for readability, not
 * speed: one thread, scalar loops, every floating-point scalar in double.
 *
 * What follows the paper:
 *   - l2 norm of one gradient tensor ............ Sec. 4.1 "Preliminaries" (notation); Eq. 3 (Sec. 4.2)
 *   - AdaGC coefficient h_{t,i} and EMA gamma .... Eq. 3, Alg. 1 (AdaGC branch)
 *   - warm-up: GlobalGC + running minimum ........ Eq. 2, Alg. 1 (warm-up branch)
 *   - GlobalGC on every step (the baseline) ...... Eq. 2
 *   - "Global AdaGC" (one adaptive threshold for the whole model; ablation
 *     "Adaptivity Efficacy and Locality Granularity" of the "Ablation Study", Sec. 5.6): Eq. 3 and the
 *     warm-up branch applied to the global norm with a single gamma
 *   - ZClip (a baseline of the paper's comparison): Table 2 prints the
 *     coefficient min{1, tau_t/||g_t||}, tau_t = mu_t + xi(z_t) sigma_t and
 *     z_t = (||g_t|| - mu_t)/sigma_t over the GLOBAL norm; the appendix
 *     "Clipping Hyper-Parameters" gives alpha = 0.97 and z_thres = 2.0.  The
 *     adjustment function xi and the update of mu, sigma are not printed: see
 *     oracle_zclip_rule for the reading taken ("parity unpinned by the paper").
 *   - AGC and Clippy (update-clipping baselines of the paper's comparison):
 *     Table 2 prints min{1, lambda_rel ||theta||/||Delta||} (l2) and
 *     min{1, (lambda_rel ||theta||_inf + lambda_abs)/(eta ||Delta||_inf)};
 *     see oracle_agc_coef / oracle_clippy_coef for the readings taken
 *   - AdamW moments, bias correction, update ..... Alg. 1 (last four statements)
 * What the paper does not print and is taken from its citation:
 *   - Lion update rule (Chen et al., "Symbolic discovery of optimization
 *     algorithms"): c = b1 m + (1-b1) g; theta -= lr (sign(c) + wd theta);
 *     m = b2 m + (1-b2) g.          "parity unpinned by the paper" for the rule
 *     itself; its arithmetic is pinned by hand-worked cases in the tests.
 *
 * Readings taken where the paper is silent (each also listed in the design
 * notes of the repository):
 *   - the EMA takes the CLIPPED norm (sentence after Eq. 3, Alg. 1), evaluated
 *     analytically: lambda_rel*gamma when clipped, the raw norm otherwise;
 *   - the clip is active only for norm > lambda_rel*gamma (strict);
 *   - the step counter passed in is 1-based and is the t of the bias
 *     correction; warm-up covers steps 1..T_start ("the first T_start steps"),
 *     and on step 1 gamma is set to the (globally clipped) norm of that step;
 *   - gamma, theta, m, v are stored as 32-bit floats; each is rounded exactly
 *     once per step, from the double result;
 *   - a bf16 copy of theta is the round-to-nearest-even of the stored float;
 *   - a bf16 gradient is widened exactly before use.
 *
 * The all-cores build.  The same file compiled with -fopenmp gives a second
 * library that spreads the per-element loops over the host's cores, for
 * checking lists of billions of parameters in minutes.  Every element of
 * theta, m, v and the bf16 copy is computed by the same statements, so those
 * come out bit-identical to the one-thread build.  A sum of squares is cut
 * into one contiguous block of indices per thread, each block summed in index
 * order and the block sums added in block order: a different rounding order of
 * the same sum (relative difference ~1e-16), nothing else.  The one-thread
 * build stays the definition; a test holds the two against each other.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#define ORACLE_PARALLEL_FOR _Pragma("omp parallel for schedule(static)")
#else
#define ORACLE_PARALLEL_FOR
#endif

/* Threads the per-element loops run on: 1 in the one-thread build. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- bf16 <-> float, from the format definition (1-8-7 bits, the top half
 *      of an IEEE binary32) -------------------------------------------------- */

float oracle_bf16_to_float(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round to nearest, ties to even, by comparing the discarded 16 bits with one
 * half unit in the last kept place.  NaN stays NaN (quiet bit forced). */
uint16_t oracle_float_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t kept = u >> 16;
    uint32_t dropped = u & 0xFFFFu;
    if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u)))
        kept += 1u; /* carry into the exponent is the correct rounding, up to inf */
    return (uint16_t)kept;
}

/* ---- l2 norm of one tensor (notation of Sec. 4.1; used by Eq. 3, Sec. 4.2) -- */

/* grad_dtype: 0 = float32, 1 = bf16.  Sum of squares of elements [begin, end) in index order. */
static double sum_squares_range(const void *g, int64_t begin, int64_t end, int grad_dtype)
{
    double s = 0.0;
    if (grad_dtype == 0) {
        const float *gf = (const float *)g;
        for (int64_t j = begin; j < end; ++j) {
            double x = (double)gf[j];
            s += x * x;
        }
    } else {
        const uint16_t *gb = (const uint16_t *)g;
        for (int64_t j = begin; j < end; ++j) {
            double x = (double)oracle_bf16_to_float(gb[j]);
            s += x * x;
        }
    }
    return s;
}

double oracle_sum_squares(const void *g, int64_t numel, int grad_dtype)
{
#ifdef _OPENMP
    /* one contiguous block per thread; block sums added in block order */
    enum { MAX_BLOCKS = 1024 };
    double block_sum[MAX_BLOCKS];
    int blocks = omp_get_max_threads();
    if (blocks > MAX_BLOCKS) blocks = MAX_BLOCKS;
    if ((int64_t)blocks > numel) blocks = numel > 0 ? (int)numel : 1;
    int64_t per_block = numel / blocks, extra = numel % blocks; /* the first `extra` blocks hold one more */
    #pragma omp parallel for schedule(static, 1) num_threads(blocks)
    for (int b = 0; b < blocks; ++b) {
        int64_t begin = b * per_block + (b < extra ? b : extra);
        int64_t end = begin + per_block + (b < extra ? 1 : 0);
        block_sum[b] = sum_squares_range(g, begin, end, grad_dtype);
    }
    double s = 0.0;
    for (int b = 0; b < blocks; ++b)
        s += block_sum[b];
    return s;
#else
    return sum_squares_range(g, 0, numel, grad_dtype);
#endif
}

double oracle_l2_norm(const void *g, int64_t numel, int grad_dtype)
{
    return sqrt(oracle_sum_squares(g, numel, grad_dtype));
}

/* ---- per-tensor quantities the paper plots next to the gradient norm (Fig. 2 and the
 *      optimizer-state figures of the appendix): l2 norms of the first moment, of the
 *      second moment, and of the parameter update theta_t - theta_{t-1}, all from the
 *      stored float32 values ------------------------------------------------------------ */

double oracle_l2_norm_of_difference(const float *a, const float *b, int64_t numel)
{
    double s = 0.0;
    for (int64_t j = 0; j < numel; ++j) {
        double d = (double)a[j] - (double)b[j];
        s += d * d;
    }
    return sqrt(s);
}

void oracle_state_norms(const float *theta_before, const float *theta_after, const float *m,
                        const float *v /* may be NULL */, int64_t numel, double *m_norm,
                        double *v_norm, double *update_norm)
{
    *m_norm = oracle_l2_norm(m, numel, 0);
    *v_norm = v ? oracle_l2_norm(v, numel, 0) : 0.0;
    *update_norm = oracle_l2_norm_of_difference(theta_after, theta_before, numel);
}

/* ---- Eq. 3, Alg. 1 AdaGC branch: one tensor's scalars --------------------- */

/* norm = ||g_{t,i}||, gamma_prev = gamma_{t-1,i}.
 * Outputs h_{t,i}, gamma_{t,i}, and whether the clip was active. */
void oracle_adagc_rule(double norm, double gamma_prev, double lambda_rel, double beta,
                       double *h, double *gamma_new, int *clipped)
{
    double threshold = lambda_rel * gamma_prev;
    int active = (norm > threshold);       /* strict; false for NaN operands */
    double coef = active ? threshold / norm : 1.0;
    double clipped_norm = active ? threshold : norm; /* = ||h g|| */
    *h = coef;
    *gamma_new = beta * gamma_prev + (1.0 - beta) * clipped_norm;
    *clipped = active;
}

/* ---- Eq. 2, Alg. 1 warm-up branch ----------------------------------------- */

/* h_t = min{lambda_abs / ||g_t||, 1}. */
double oracle_globalgc_coef(double global_norm, double lambda_abs)
{
    int active = (global_norm > lambda_abs);
    return active ? lambda_abs / global_norm : 1.0;
}

/* gamma_{t,i} = min{gamma_{t-1,i}, ||ghat_{t,i}||}; on the very first step
 * gamma is the clipped norm of that step. */
double oracle_warmup_gamma(double gamma_prev, double clipped_norm, int first_step)
{
    if (first_step)
        return clipped_norm;
    return clipped_norm < gamma_prev ? clipped_norm : gamma_prev;
}

/* ---- ZClip (Table 2 "Comparison of major gradient/update clipping methods") ---
 *
 * Printed: h = min{1, tau/||g||}, tau = mu + xi(z) sigma, z = (||g|| - mu)/sigma, with mu and
 * sigma the EMA mean and standard deviation of the global gradient norm; alpha = 0.97 and
 * z_thres = 2.0 (appendix "Clipping Hyper-Parameters").
 * Not printed, reading taken here:
 *   - the clip is active only for z > z_thres (strict);
 *   - xi(z) = z_thres^2 / z, the reciprocal adjustment: the further out the norm lies, the lower
 *     the threshold; at z = z_thres it gives tau = ||g||, so h is continuous there;
 *   - the statistics take the CLIPPED norm nhat (tau when active, ||g|| otherwise), as AdaGC's
 *     own EMA does: mu' = alpha mu + (1-alpha) nhat, var' = alpha var + (1-alpha)(nhat - mu')^2,
 *     sigma = sqrt(var); mu and var are kept as two 32-bit floats.
 * sigma = 0 needs no special case: z is +inf, -inf or NaN, and IEEE arithmetic gives tau = mu
 * for a norm above mu and no clip otherwise. */
void oracle_zclip_rule(double norm, double mu_prev, double var_prev, double alpha, double z_thres,
                       double *h, double *mu_new, double *var_new, int *clipped)
{
    double sigma = sqrt(var_prev);
    double z = (norm - mu_prev) / sigma;
    int active = (z > z_thres);            /* false for NaN */
    double xi = z_thres * z_thres / z;
    double tau = mu_prev + xi * sigma;
    double coef = active ? tau / norm : 1.0;
    double clipped_norm = active ? tau : norm;
    double mu = alpha * mu_prev + (1.0 - alpha) * clipped_norm;
    double dev = clipped_norm - mu;
    *h = coef;
    *mu_new = mu;
    *var_new = alpha * var_prev + (1.0 - alpha) * dev * dev;
    *clipped = active;
}

/* Statistics of the steps before the z-score rule applies (the first t_start steps, on which the
 * gradient only passes through GlobalGC): the first step sets mu to its clipped norm with zero
 * variance, later ones update both as above. */
void oracle_zclip_gather(double clipped_norm, double mu_prev, double var_prev, double alpha,
                         int first_step, double *mu_new, double *var_new)
{
    if (first_step) {
        *mu_new = clipped_norm;
        *var_new = 0.0;
        return;
    }
    double mu = alpha * mu_prev + (1.0 - alpha) * clipped_norm;
    double dev = clipped_norm - mu;
    *mu_new = mu;
    *var_new = alpha * var_prev + (1.0 - alpha) * dev * dev;
}

/* ---- Alg. 1, last four statements: AdamW on the clipped gradient ----------- */

typedef struct {
    double lr, beta1, beta2, eps, weight_decay;
} oracle_opt_hyper;

static double grad_at(const void *g, int64_t j, int grad_dtype)
{
    if (grad_dtype == 0)
        return (double)((const float *)g)[j];
    return (double)oracle_bf16_to_float(((const uint16_t *)g)[j]);
}

/* update_coef scales the optimizer's direction Delta = mhat/(sqrt(vhat)+eps) (update clipping, AGC and
 * Clippy rows of Table 2); 1.0, an exact factor, everywhere else. */
static void adamw_update_scaled(float *theta, float *m, float *v, const void *g, int grad_dtype,
                                int64_t numel, double h, double update_coef, const oracle_opt_hyper *hp,
                                int64_t t, uint16_t *theta_bf16 /* may be NULL */)
{
    double bias1 = 1.0 - pow(hp->beta1, (double)t);
    double bias2 = 1.0 - pow(hp->beta2, (double)t);
    ORACLE_PARALLEL_FOR
    for (int64_t j = 0; j < numel; ++j) {
        double ghat = h * grad_at(g, j, grad_dtype);
        double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * ghat;
        double vj = hp->beta2 * (double)v[j] + (1.0 - hp->beta2) * ghat * ghat;
        double mhat = mj / bias1;
        double vhat = vj / bias2;
        double th = (double)theta[j];
        th = th - hp->lr * hp->weight_decay * th - update_coef * (hp->lr * mhat / (sqrt(vhat) + hp->eps));
        m[j] = (float)mj;
        v[j] = (float)vj;
        theta[j] = (float)th;
        if (theta_bf16)
            theta_bf16[j] = oracle_float_to_bf16_rne(theta[j]);
    }
}

void oracle_adamw_update(float *theta, float *m, float *v, const void *g, int grad_dtype,
                         int64_t numel, double h, const oracle_opt_hyper *hp, int64_t t,
                         uint16_t *theta_bf16 /* may be NULL */)
{
    adamw_update_scaled(theta, m, v, g, grad_dtype, numel, h, 1.0, hp, t, theta_bf16);
}

/* The same step with the gradient unclipped and the direction scaled by update_coef. */
void oracle_adamw_update_clipped(float *theta, float *m, float *v, const void *g, int grad_dtype,
                                 int64_t numel, double update_coef, const oracle_opt_hyper *hp, int64_t t,
                                 uint16_t *theta_bf16 /* may be NULL */)
{
    adamw_update_scaled(theta, m, v, g, grad_dtype, numel, 1.0, update_coef, hp, t, theta_bf16);
}

/* ---- Lion on the clipped gradient (rule imported from its own paper) ------- */

static void lion_update_scaled(float *theta, float *m, const void *g, int grad_dtype, int64_t numel,
                               double h, double update_coef, const oracle_opt_hyper *hp, uint16_t *theta_bf16)
{
    ORACLE_PARALLEL_FOR
    for (int64_t j = 0; j < numel; ++j) {
        double ghat = h * grad_at(g, j, grad_dtype);
        double mprev = (double)m[j];
        double c = hp->beta1 * mprev + (1.0 - hp->beta1) * ghat;
        double sgn = (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);
        double th = (double)theta[j];
        th = th - hp->lr * (update_coef * sgn + hp->weight_decay * th);
        double mj = hp->beta2 * mprev + (1.0 - hp->beta2) * ghat;
        theta[j] = (float)th;
        m[j] = (float)mj;
        if (theta_bf16)
            theta_bf16[j] = oracle_float_to_bf16_rne(theta[j]);
    }
}

void oracle_lion_update(float *theta, float *m, const void *g, int grad_dtype, int64_t numel,
                        double h, const oracle_opt_hyper *hp, uint16_t *theta_bf16)
{
    lion_update_scaled(theta, m, g, grad_dtype, numel, h, 1.0, hp, theta_bf16);
}

void oracle_lion_update_clipped(float *theta, float *m, const void *g, int grad_dtype, int64_t numel,
                                double update_coef, const oracle_opt_hyper *hp, uint16_t *theta_bf16)
{
    lion_update_scaled(theta, m, g, grad_dtype, numel, 1.0, update_coef, hp, theta_bf16);
}

/* ---- AGC and Clippy (Table 2): clipping of the optimizer's update -------------------------------
 *
 * Printed: AGC    min{1, lambda_rel ||theta_t|| / ||Delta_t||}                      (l2 norms, per unit)
 *          Clippy min{1, min((lambda_rel ||theta_t||_inf + lambda_abs)/(eta_t ||Delta_t||_inf))}  (per tensor)
 * with Delta_t "the optimizer update"; hyper-parameters in the appendix "Clipping Hyper-Parameters"
 * (AGC lambda_rel 1e-3; Clippy lambda_abs 0.5, lambda_rel 1e-2).  Both leave the gradient alone
 * (Table 2, column "Gradient") and scale the update.
 * Readings taken:
 *   - Delta_t is the optimizer's direction before the learning rate (Clippy's row multiplies it by
 *     eta_t itself): mhat/(sqrt(vhat)+eps) for AdamW, sign(c) for Lion, from this step's moments;
 *     decoupled weight decay is not part of it and is applied unscaled;
 *   - theta_t is the parameter tensor before this step's update;
 *   - a "unit" is one tensor of the list (a caller who wants rows as units lists the rows);
 *   - with norms of the whole tensor the inner min of Clippy's row has one argument;
 *   - the clip is active only when the ratio is below 1 (strict), so 0/0 and x/0 leave the update
 *     alone; a tensor of zeros has ratio 0 under AGC and its update is scaled to nothing: the
 *     printed rule has no floor on ||theta|| and none is invented. */
double oracle_agc_coef(double theta_norm, double delta_norm, double lambda_rel, int *clipped)
{
    double ratio = lambda_rel * theta_norm / delta_norm;
    int active = (ratio < 1.0);            /* false for NaN */
    *clipped = active;
    return active ? ratio : 1.0;
}

double oracle_clippy_coef(double theta_inf, double delta_inf, double lambda_rel, double lambda_abs,
                          double lr, int *clipped)
{
    double ratio = (lambda_rel * theta_inf + lambda_abs) / (lr * delta_inf);
    int active = (ratio < 1.0);
    *clipped = active;
    return active ? ratio : 1.0;
}

/* l2 and l-infinity norms of theta (before the step) and of the direction Delta this step's
 * unclipped gradient produces; m, v are read, not written.  v is unused for Lion. */
void oracle_direction_norms(const float *theta, const float *m, const float *v, const void *g,
                            int grad_dtype, int64_t numel, const oracle_opt_hyper *hp, int optimizer,
                            int64_t t, double *theta_l2, double *delta_l2, double *theta_inf,
                            double *delta_inf)
{
    double bias1 = 1.0 - pow(hp->beta1, (double)t);
    double bias2 = 1.0 - pow(hp->beta2, (double)t);
    double s_theta = 0.0, s_delta = 0.0, max_theta = 0.0, max_delta = 0.0;
    for (int64_t j = 0; j < numel; ++j) {
        double gj = grad_at(g, j, grad_dtype);
        double delta;
        if (optimizer == 0) {
            double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * gj;
            double vj = hp->beta2 * (double)v[j] + (1.0 - hp->beta2) * gj * gj;
            delta = (mj / bias1) / (sqrt(vj / bias2) + hp->eps);
        } else {
            double c = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * gj;
            delta = (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);
        }
        double th = (double)theta[j];
        s_theta += th * th;
        s_delta += delta * delta;
        if (fabs(th) > max_theta) max_theta = fabs(th);
        if (fabs(delta) > max_delta) max_delta = fabs(delta);
    }
    *theta_l2 = sqrt(s_theta);
    *delta_l2 = sqrt(s_delta);
    *theta_inf = max_theta;
    *delta_inf = max_delta;
}

/* ---- Alg. 1, one pass of the repeat-loop body over a list of tensors ------- */

typedef struct {
    double lr, beta1, beta2, eps, weight_decay; /* eta_t, beta_1, beta_2, epsilon, lambda_w */
    double lambda_rel, ema_beta;                /* lambda_rel, beta                        */
    double lambda_abs;                          /* GlobalGC threshold of the warm-up        */
    int64_t t_start;                            /* number of warm-up steps                  */
    int32_t optimizer;                          /* 0 = AdamW, 1 = Lion                      */
    int32_t grad_dtype;                         /* 0 = float32, 1 = bf16                    */
    int32_t clip_mode;                          /* 0 = AdaGC (Alg. 1), 1 = GlobalGC on every step (Eq. 2),
                                                   2 = Global AdaGC (single gamma, kept in gamma[0]),
                                                   3 = ZClip (mu in gamma[0], variance in gamma[1];
                                                       ema_beta is its alpha),
                                                   4 = AGC, 5 = Clippy: the update is clipped, the
                                                       gradient is not; no state; lambda_rel (and, for
                                                       Clippy, lambda_abs) are Table 2's */
    int32_t reserved;
    double z_thres;                             /* ZClip's z-score threshold */
} oracle_step_hyper;

/* Arrays of per-tensor pointers; state is updated in place.  v may be NULL for
 * Lion, theta_bf16 may be NULL.  step is the 1-based t.  out_* receive the
 * per-tensor pre-clip norm, coefficient, and clip flag (each may be NULL).
 * Returns 0, or -1 on a bad argument. */
int oracle_adagc_step(int64_t n_tensors, const int64_t *numel, float *const *theta,
                      const void *const *grad, float *const *m, float *const *v,
                      uint16_t *const *theta_bf16, float *gamma, const oracle_step_hyper *hp,
                      int64_t step, double *out_norm, double *out_coef, uint8_t *out_clipped)
{
    if (n_tensors <= 0 || step < 1 || !numel || !theta || !grad || !m || !gamma || !hp)
        return -1;
    if (hp->optimizer == 0 && !v)
        return -1;

    oracle_opt_hyper oh = { hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay };
    int warmup = (step - 1) < hp->t_start; /* steps 1..T_start */

    const int mode = hp->clip_mode;
    if (mode < 0 || mode > 5)
        return -1;

    if (mode == 4 || mode == 5) {
        /* update clipping: out_norm reports the norm of the direction the rule acts on */
        for (int64_t i = 0; i < n_tensors; ++i) {
            double th2, d2, thinf, dinf, c;
            int clipped;
            oracle_direction_norms(theta[i], m[i], v ? v[i] : NULL, grad[i], hp->grad_dtype, numel[i], &oh,
                                   hp->optimizer, step, &th2, &d2, &thinf, &dinf);
            if (mode == 4)
                c = oracle_agc_coef(th2, d2, hp->lambda_rel, &clipped);
            else
                c = oracle_clippy_coef(thinf, dinf, hp->lambda_rel, hp->lambda_abs, hp->lr, &clipped);
            if (out_norm) out_norm[i] = (mode == 4) ? d2 : dinf;
            if (out_coef) out_coef[i] = c;
            if (out_clipped) out_clipped[i] = (uint8_t)clipped;
            uint16_t *copy = theta_bf16 ? theta_bf16[i] : NULL;
            if (hp->optimizer == 0)
                oracle_adamw_update_clipped(theta[i], m[i], v[i], grad[i], hp->grad_dtype, numel[i], c, &oh,
                                            step, copy);
            else
                oracle_lion_update_clipped(theta[i], m[i], grad[i], hp->grad_dtype, numel[i], c, &oh, copy);
        }
        return 0;
    }

    /* ||g_t|| over the whole model: tensors in list order, elements in index order */
    double h_global = 1.0;
    int clipped_global = 0;
    if (warmup || mode != 0) {
        double s = 0.0;
        for (int64_t i = 0; i < n_tensors; ++i)
            s += oracle_sum_squares(grad[i], numel[i], hp->grad_dtype);
        double global_norm = sqrt(s);
        if (mode == 2 && !warmup) {
            /* Eq. 3 with the model as the single "tensor" */
            double gamma_new;
            oracle_adagc_rule(global_norm, (double)gamma[0], hp->lambda_rel, hp->ema_beta, &h_global,
                              &gamma_new, &clipped_global);
            gamma[0] = (float)gamma_new;
        } else if (mode == 3 && !warmup) {
            double mu_new, var_new;
            oracle_zclip_rule(global_norm, (double)gamma[0], (double)gamma[1], hp->ema_beta, hp->z_thres,
                              &h_global, &mu_new, &var_new, &clipped_global);
            gamma[0] = (float)mu_new;
            gamma[1] = (float)var_new;
        } else {
            h_global = oracle_globalgc_coef(global_norm, hp->lambda_abs);
            clipped_global = (h_global < 1.0);
            if (mode == 2)
                gamma[0] = (float)oracle_warmup_gamma((double)gamma[0], h_global * global_norm, step == 1);
            if (mode == 3) {
                double mu_new, var_new;
                oracle_zclip_gather(h_global * global_norm, (double)gamma[0], (double)gamma[1],
                                    hp->ema_beta, step == 1, &mu_new, &var_new);
                gamma[0] = (float)mu_new;
                gamma[1] = (float)var_new;
            }
        }
    }

    for (int64_t i = 0; i < n_tensors; ++i) {
        double norm = oracle_l2_norm(grad[i], numel[i], hp->grad_dtype);
        double h;
        int clipped;
        if (mode != 0) {
            /* one coefficient for every tensor; no per-tensor state */
            h = h_global;
            clipped = clipped_global;
        } else {
            double gamma_prev = (double)gamma[i];
            double gamma_new;
            if (warmup) {
                h = h_global;
                clipped = clipped_global;
                gamma_new = oracle_warmup_gamma(gamma_prev, h * norm, step == 1);
            } else {
                oracle_adagc_rule(norm, gamma_prev, hp->lambda_rel, hp->ema_beta, &h, &gamma_new,
                                  &clipped);
            }
            gamma[i] = (float)gamma_new;
        }
        if (out_norm) out_norm[i] = norm;
        if (out_coef) out_coef[i] = h;
        if (out_clipped) out_clipped[i] = (uint8_t)clipped;

        uint16_t *copy = theta_bf16 ? theta_bf16[i] : NULL;
        if (hp->optimizer == 0)
            oracle_adamw_update(theta[i], m[i], v[i], grad[i], hp->grad_dtype, numel[i], h, &oh,
                                step, copy);
        else
            oracle_lion_update(theta[i], m[i], grad[i], hp->grad_dtype, numel[i], h, &oh, copy);
    }
    return 0;
}
