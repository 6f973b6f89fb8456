/*
 * gxpo_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, obviously-correct fp64 CPU statement of what one GXPO
 * training step computes in parameter space (Algorithm 1 of the paper).  It
 * exists only so that tests, the smoke check and the bench's CPU-baseline leg
 * have something independent to compare the GPU engine against.  It shares
 * no code, header, table or helper with the HIP library, and the HIP library
 * never calls it.
 *
 * Every function works on double arrays.  Callers up-cast the fp32 / bf16
 * buffers the GPU consumed (an exact conversion) before handing them in.
 *
 * There is no blocking, fusion, vectorisation or reordering here: each
 * function is the paper's formula, one coordinate after another.
 *
 * Readings taken where the paper is silent are marked READING and are listed
 * again in the design notes of the repository.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/* ------------------------------------------------------------------------
 * OptimStep (Section 2 "Method", first paragraph; Algorithm 1 lines that call
 * OptimStep).  The paper names two instances:
 *
 *   optimizer == 0 : plain gradient descent, theta <- theta - eta * g
 *                    (Section 2.1, the step that produces Eq. (2); Appendix
 *                    A.3 first display).
 *   optimizer == 1 : AdamW, the optimizer the experiments run on (Section 2,
 *                    citing Loshchilov & Hutter).  The paper does
 *                    not write AdamW out; this is the published decoupled
 *                    weight-decay form:
 *                        s     <- s + 1
 *                        theta <- theta * (1 - lr * wd)
 *                        m     <- beta1 m + (1 - beta1) g
 *                        v     <- beta2 v + (1 - beta2) g^2
 *                        theta <- theta - lr * (m / (1 - beta1^s))
 *                                            / (sqrt(v / (1 - beta2^s)) + eps)
 *
 * `*step_count` is the optimizer's own step counter s.  READING (Section 2.3,
 * paragraph after Eq. (9), which says that with a stateful optimizer the two
 * fast steps advance its state, the parameters are then moved by hand, and
 * the third step uses g_slow): every OptimStep call advances s, m and v, and
 * nothing is rolled back when the parameters are repositioned.
 *
 * theta_in and theta_out may be the same array.  m and v are ignored (may be
 * NULL) for plain GD.
 * ---------------------------------------------------------------------- */
void gxpo_oracle_optim_step(int optimizer, double lr, double beta1, double beta2,
                            double eps, double weight_decay,
                            int64_t n, int64_t *step_count,
                            const double *theta_in, const double *g,
                            double *m, double *v, double *theta_out)
{
    *step_count += 1;
    if (optimizer == 0) {
        for (int64_t i = 0; i < n; ++i)
            theta_out[i] = theta_in[i] - lr * g[i];
        return;
    }
    const double s = (double)(*step_count);
    const double bias1 = 1.0 - pow(beta1, s);
    const double bias2 = 1.0 - pow(beta2, s);
    for (int64_t i = 0; i < n; ++i) {
        double th = theta_in[i] * (1.0 - lr * weight_decay);
        m[i] = beta1 * m[i] + (1.0 - beta1) * g[i];
        v[i] = beta2 * v[i] + (1.0 - beta2) * g[i] * g[i];
        double m_hat = m[i] / bias1;
        double v_hat = v[i] / bias2;
        theta_out[i] = th - lr * m_hat / (sqrt(v_hat) + eps);
    }
}

/* ------------------------------------------------------------------------
 * Geometric sum S_n(x) = sum_{j=0}^{n-1} x^j  (Appendix A.4, Proposition on
 * total displacement, definition of S_K).  Written as the sum itself, so the
 * x = 1 case (S = n) needs no special branch and nothing cancels near x = 1.
 * ---------------------------------------------------------------------- */
double gxpo_oracle_geometric_sum(double x, int n)
{
    double sum = 0.0, power = 1.0;
    for (int j = 0; j < n; ++j) {
        sum += power;
        power *= x;
    }
    return sum;
}

/* ------------------------------------------------------------------------
 * Extrapolation factor of one coordinate (Algorithm 1: active set, retention
 * ratio, geometric sum, extrapolation factor; Eqs. (4) and (7)).
 *
 *   active  <=> |g0| > delta            (strict, Section 2.2 last paragraph)
 *   r       =  g1 / g0                  (Eq. (4))
 *   scale   =  S_K(r) / S_2(r)          (Eq. (7)),  1 when not active
 *
 * READINGS:
 *  - delta is compared after rounding it to fp32, because the GPU engine
 *    compares fp32 gradients against an fp32 threshold and set membership
 *    must not depend on which side evaluates it.
 *  - r_max (finite) clamps r into [-r_max, r_max] before the sums; r_max is
 *    rounded to fp32 for the same reason.  r_max = +inf is the rule exactly
 *    as printed.  (The error lemma of Appendix A.5 assumes |r_i| <= R; the
 *    printed algorithm has no clamp.)
 *  - S_2(r) = 1 + r vanishes at r = -1.  The paper's policy for coordinates
 *    whose ratio is unusable is to keep the observed two-probe displacement
 *    (Remark "Ratio safeguards in practice"), so r == -1 gives scale = 1.
 * ---------------------------------------------------------------------- */
/* The retention ratio as the rule uses it: returns 0 when the coordinate is off
 * the active set (then *r_out is untouched), 1 otherwise with *r_out = g1/g0
 * after the optional clamp. */
static int retention_ratio(double g0, double g1, double delta, double r_max, double *r_out)
{
    const double delta32 = (double)(float)delta;
    if (!(fabs(g0) > delta32))
        return 0;
    double r = g1 / g0;
    if (isfinite(r_max)) {
        const double R = (double)(float)r_max;
        if (r > R) r = R;
        if (r < -R) r = -R;
    }
    *r_out = r;
    return 1;
}

double gxpo_oracle_scale(double g0, double g1, int K, double delta, double r_max)
{
    double r;
    if (!retention_ratio(g0, g1, delta, r_max, &r))
        return 1.0;
    if (r == -1.0)
        return 1.0;
    return gxpo_oracle_geometric_sum(r, K) / gxpo_oracle_geometric_sum(r, 2);
}

/* ------------------------------------------------------------------------
 * Extrapolate and reposition (Algorithm 1 "Extrapolate" and "Reposition";
 * Eqs. (8) and (9)):
 *
 *   theta_K     = theta_0 + (theta_2 - theta_0) * scale
 *   theta_tilde = theta_0 + alpha * (theta_K - theta_0)
 *
 * theta_2 - theta_0 is the displacement the optimizer actually produced over
 * the two fast steps (Section 2.3, paragraph after the K-step displacement
 * display), weight decay and moment effects included.
 *
 * scale_out, theta_K_out may be NULL.
 * ---------------------------------------------------------------------- */
void gxpo_oracle_extrapolate(int64_t n, const double *theta_0, const double *theta_2,
                             const double *g0, const double *g1,
                             int K, double alpha, double delta, double r_max,
                             double *scale_out, double *theta_K_out,
                             double *theta_tilde_out)
{
    for (int64_t i = 0; i < n; ++i) {
        double scale = gxpo_oracle_scale(g0[i], g1[i], K, delta, r_max);
        double theta_K = theta_0[i] + (theta_2[i] - theta_0[i]) * scale;
        double theta_tilde = theta_0[i] + alpha * (theta_K - theta_0[i]);
        if (scale_out) scale_out[i] = scale;
        if (theta_K_out) theta_K_out[i] = theta_K;
        theta_tilde_out[i] = theta_tilde;
    }
}

/* ------------------------------------------------------------------------
 * Sum of squares of a gradient buffer; the caller takes the square root of
 * the total over all tensors to get ||g_slow||_2 of Eq. (10).  Accumulated in
 * long double so the value is the mathematical sum to well below fp64
 * resolution at any length used here.
 * ---------------------------------------------------------------------- */
double gxpo_oracle_sum_squares(int64_t n, const double *g)
{
    long double acc = 0.0L;
    for (int64_t i = 0; i < n; ++i)
        acc += (long double)g[i] * (long double)g[i];
    return (double)acc;
}

/* ------------------------------------------------------------------------
 * Global-norm gradient clipping (Section 3.1 lists "gradient clipping at 1.0"
 * among the training settings and says nothing more).  READING: the widely
 * used rule -- every gradient handed to an OptimStep is multiplied by
 *     c = min(1, max_norm / (||g||_2 + 1e-6)),
 * the norm taken over all tensors of that gradient.  max_norm <= 0 disables it.
 * ---------------------------------------------------------------------- */
double gxpo_oracle_clip_coefficient(double total_norm, double max_norm)
{
    if (!(max_norm > 0.0))
        return 1.0;
    double c = max_norm / (total_norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ------------------------------------------------------------------------
 * Mechanism diagnostics of one active step: the quantities of the paper's
 * appendix table "Active-phase GXPO diagnostics" (gradient norms,
 * cos(g0, g_slow), retention ratio mean and deviation over the active set,
 * ||Delta_K|| / ||Delta_2||, mean scale, inactive fraction), for one tensor.
 * Plain two-pass definitions, accumulated in long double.
 *
 * READINGS (the table gives names, not formulas): the retention statistics and
 * the mean scale run over the active set {|g0| > delta} and use r after the
 * optional clamp; the deviation is the population deviation;
 * Delta_2 = theta^{t,2} - theta^t, Delta_K = theta^{t,K} - theta^t.
 *
 * out[0] sum g0^2      out[1] sum g1^2       out[2] sum g_slow^2
 * out[3] sum g0*g_slow out[4] active count   out[5] sum_active r
 * out[6] sum_active (r - mean_r)^2           out[7] sum_active scale
 * out[8] sum Delta_2^2 out[9] sum Delta_K^2
 * mean_r (the mean over the active set of ALL tensors) is passed in for the
 * second pass; call once with NAN to get out[4], out[5], then again.
 * ---------------------------------------------------------------------- */
void gxpo_oracle_diagnostic_sums(int64_t n, const double *theta_0, const double *theta_2,
                                 const double *g0, const double *g1, const double *g_slow,
                                 int K, double delta, double r_max, double mean_r, double *out)
{
    long double a[10] = {0};
    for (int64_t i = 0; i < n; ++i) {
        a[0] += (long double)g0[i] * g0[i];
        a[1] += (long double)g1[i] * g1[i];
        a[2] += (long double)g_slow[i] * g_slow[i];
        a[3] += (long double)g0[i] * g_slow[i];
        double r;
        double scale = gxpo_oracle_scale(g0[i], g1[i], K, delta, r_max);
        if (retention_ratio(g0[i], g1[i], delta, r_max, &r)) {
            a[4] += 1.0L;
            a[5] += r;
            if (!isnan(mean_r))
                a[6] += ((long double)r - mean_r) * ((long double)r - mean_r);
            a[7] += scale;
        }
        const double d2 = theta_2[i] - theta_0[i];
        const double dK = d2 * scale;
        a[8] += (long double)d2 * d2;
        a[9] += (long double)dK * dK;
    }
    for (int j = 0; j < 10; ++j)
        out[j] = (double)a[j];
}

/* ------------------------------------------------------------------------
 * Round an fp32 value to bf16 (round to nearest, ties to even) and return
 * the 16 stored bits.  This is the published bfloat16 format: the top 16
 * bits of the IEEE-754 binary32 pattern.  Used to check the bf16 model copy
 * the engine writes next to its fp32 master weights (Section 3.1: runs use
 * bf16 precision).  NaN stays NaN (quiet bit forced).
 * ---------------------------------------------------------------------- */
uint16_t gxpo_oracle_bf16_bits(float x)
{
    union { float f; uint32_t u; } b;
    b.f = x;
    if ((b.u & 0x7fffffffu) > 0x7f800000u)          /* NaN */
        return (uint16_t)((b.u >> 16) | 0x0040u);
    uint32_t kept_lsb = (b.u >> 16) & 1u;
    uint32_t rounded = b.u + 0x7fffu + kept_lsb;
    return (uint16_t)(rounded >> 16);
}

void gxpo_oracle_bf16_round_array(int64_t n, const float *x, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = gxpo_oracle_bf16_bits(x[i]);
}
