/* Every entry point of the C oracle on exact-size heap arrays (sizes 0..69, so any access one element
 * past an end is caught), built with -fsanitize=address,undefined.  CPU only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <math.h>
void gxpo_oracle_optim_step(int, double, double, double, double, double, int64_t, int64_t *, const double *, const double *, double *, double *, double *);
void gxpo_oracle_extrapolate(int64_t, const double *, const double *, const double *, const double *, int, double, double, double, double *, double *, double *);
double gxpo_oracle_sum_squares(int64_t, const double *);
double gxpo_oracle_geometric_sum(double, int);
double gxpo_oracle_scale(double, double, int, double, double);
double gxpo_oracle_clip_coefficient(double, double);
void gxpo_oracle_diagnostic_sums(int64_t, const double *, const double *, const double *, const double *, const double *, int, double, double, double, double *);
void gxpo_oracle_bf16_round_array(int64_t, const float *, uint16_t *);
static double *arr(int64_t n, unsigned seed) { double *a = malloc(n * sizeof *a); srand(seed); for (int64_t i = 0; i < n; ++i) a[i] = rand() / (double)RAND_MAX - 0.5; return a; }
int main(void) {
    for (int64_t n = 0; n < 70; ++n) {
        double *th = arr(n, 1), *g0 = arr(n, 2), *g1 = arr(n, 3), *gs = arr(n, 4), *m = calloc(n ? n : 1, 8), *v = calloc(n ? n : 1, 8), *out = arr(n, 5), *th2 = arr(n, 6);
        double *sc = arr(n, 7), *tk = arr(n, 8);
        int64_t cnt = 0;
        gxpo_oracle_optim_step(1, 1e-3, .9, .999, 1e-8, .01, n, &cnt, th, g0, m, v, out);
        gxpo_oracle_optim_step(0, 1e-3, .9, .999, 1e-8, .01, n, &cnt, th, g0, NULL, NULL, out);
        for (int K = 2; K < 7; ++K) {
            gxpo_oracle_extrapolate(n, th, th2, g0, g1, K, 0.5, 1e-3, INFINITY, sc, tk, out);
            gxpo_oracle_extrapolate(n, th, th2, g0, g1, K, 0.5, 1e-3, 2.0, NULL, NULL, out);
        }
        double d[10];
        gxpo_oracle_diagnostic_sums(n, th, th2, g0, g1, gs, 5, 1e-3, INFINITY, NAN, d);
        gxpo_oracle_diagnostic_sums(n, th, th2, g0, g1, gs, 5, 1e-3, INFINITY, 0.9, d);
        (void)gxpo_oracle_sum_squares(n, gs);
        float *f = malloc((n ? n : 1) * 4); uint16_t *b = malloc((n ? n : 1) * 2);
        for (int64_t i = 0; i < n; ++i) f[i] = (float)g0[i];
        gxpo_oracle_bf16_round_array(n, f, b);
        free(th); free(g0); free(g1); free(gs); free(m); free(v); free(out); free(th2); free(sc); free(tk); free(f); free(b);
    }
    for (int K = 2; K < 12; ++K) {
        static const double r[] = {-2.0, -1.0, -0.5, 0.0, 0.5, 1.0, 3.0};
        for (unsigned i = 0; i < sizeof r / sizeof r[0]; ++i) {
            (void)gxpo_oracle_geometric_sum(r[i], K);
            (void)gxpo_oracle_scale(1.0, r[i], K, 1e-3, INFINITY);
            (void)gxpo_oracle_scale(1e-4, r[i], K, 1e-3, 2.0);
            (void)gxpo_oracle_scale(0.0, r[i], K, 0.0, INFINITY);
        }
    }
    (void)gxpo_oracle_clip_coefficient(0.0, 1.0);
    (void)gxpo_oracle_clip_coefficient(INFINITY, 1.0);
    (void)gxpo_oracle_clip_coefficient(NAN, 1.0);
    puts("oracle clean under ASan + UBSan");
    return 0;
}
