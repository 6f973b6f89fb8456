/*
 * A plain C program (built with gcc, no Python, no torch) that drives the GXPO engine through its
 * C ABI on the GPU: one ragged two-tensor problem on the paper's diagonal quadratic surrogate with
 * plain gradient descent, where every result has a closed form (Section 2.4 corollary and
 * Appendix A.6: on a diagonal quadratic the extrapolated point is the K-th gradient-descent
 * iterate, so one active step with alpha = 1 equals K + 1 gradient-descent steps).
 *
 * Exit status 0 and a last line "abi driver ok" on success.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "gxpo.h"

#define N_TENSORS 2
static const uint64_t numel[N_TENSORS] = {1000, 4099};

#define HIP_OK(call)                                                                 \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            return 2;                                                                \
        }                                                                            \
    } while (0)
#define GXPO_OK_OR_DIE(call)                                                         \
    do {                                                                             \
        int rc_ = (call);                                                            \
        if (rc_ != GXPO_OK) {                                                        \
            fprintf(stderr, "%s -> %d: %s\n", #call, rc_, gxpo_last_error(ctx));     \
            return 3;                                                                \
        }                                                                            \
    } while (0)

/* the surrogate: L = 1/2 sum h_i (theta_i - star_i)^2, values chosen to be exact in fp32 */
static float h_of(uint64_t i) { return 0.125f + 0.0625f * (float)(i % 13); }          /* 0.125 .. 0.875 */
static float star_of(uint64_t i) { return 0.5f * (float)((int)(i % 7) - 3); }
static float start_of(uint64_t i) { return 0.25f * (float)((int)(i % 11) - 5); }

/* AdamW on the same surrogate, two active steps and one fallback step, once updating theta, m, v in place and once with
 * the second buffer set (theta_probe, m_alt, v_alt) the passes alternate with: the parameters and both moments must
 * come out bit for bit the same, in the set gxpo_state.current_set names.  Returns 0, or an exit status. */
static int adamw_run(int alternating, float *out[3]) {
    const uint64_t n = 4099;
    const size_t bytes = n * sizeof(float);
    gxpo_tensor x;
    memset(&x, 0, sizeof x);
    x.numel = n;
    float **bufs[] = {&x.theta, &x.theta_probe, &x.m, &x.v, &x.m_alt, &x.v_alt};
    for (int b = 0; b < (alternating ? 6 : 4); ++b) {
        HIP_OK(hipMalloc((void **)bufs[b], bytes));
        HIP_OK(hipMemset(*bufs[b], 0, bytes));
    }
    float *d_g[3], *h = (float *)malloc(bytes), *g = (float *)malloc(bytes);
    for (int r = 0; r < 3; ++r) HIP_OK(hipMalloc((void **)&d_g[r], bytes));
    for (uint64_t i = 0; i < n; ++i) h[i] = start_of(i);
    HIP_OK(hipMemcpy(x.theta, h, bytes, hipMemcpyHostToDevice));
    gxpo_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.struct_size = sizeof cfg, cfg.optimizer = GXPO_OPT_ADAMW, cfg.grad_dtype = GXPO_GRAD_F32, cfg.K = 5, cfg.fuse_step2 = 1;
    cfg.window = 4, cfg.lr = 1e-2, cfg.beta1 = 0.9, cfg.beta2 = 0.999, cfg.adam_eps = 1e-8, cfg.weight_decay = 0.01;
    cfg.alpha = 0.5, cfg.delta = 1e-3, cfg.r_max = 4.0, cfg.tau = 1e30, cfg.gate_eps = 1e-8;
    gxpo_ctx *ctx = NULL;
    GXPO_OK_OR_DIE(gxpo_init(&ctx, &cfg, &x, 1));
    gxpo_state st;
#define CURRENT(set) ((set) ? x.theta_probe : x.theta)
#define GRAD_AT(buffer, role)                                                                      \
    do {                                                                                           \
        HIP_OK(hipMemcpy(h, (buffer), bytes, hipMemcpyDeviceToHost));                              \
        for (uint64_t i = 0; i < n; ++i) g[i] = h_of(i) * (h[i] - star_of(i));                     \
        HIP_OK(hipMemcpy(d_g[role], g, bytes, hipMemcpyHostToDevice));                             \
    } while (0)
    for (int step = 0; step < 3; ++step) {
        const void *l0[1] = {d_g[0]}, *l1[1] = {d_g[1]}, *l2[1] = {d_g[2]};
        GXPO_OK_OR_DIE(gxpo_get_state(ctx, &st));
        const unsigned c = st.current_set;
        if (!alternating && c != 0) return 8;
        GRAD_AT(CURRENT(c), 0);
        if (step == 2) {                                   /* the gate is forced shut: one fallback step */
            st.s_star = st.t;
            GXPO_OK_OR_DIE(gxpo_set_state(ctx, &st));
            GXPO_OK_OR_DIE(gxpo_fallback_step(ctx, l0, NULL));
            break;
        }
        GXPO_OK_OR_DIE(gxpo_fast_steps(ctx, 0, l0, NULL));
        GRAD_AT(alternating ? CURRENT(1 - c) : x.theta_probe, 1);          /* theta^{t,1} */
        GXPO_OK_OR_DIE(gxpo_fast_steps(ctx, 1, l1, NULL));
        GXPO_OK_OR_DIE(gxpo_extrapolate(ctx, l0, l1, NULL));
        GXPO_OK_OR_DIE(gxpo_get_state(ctx, &st));
        if (st.current_set != (alternating ? 1 - c : 0)) return 8;
        GRAD_AT(CURRENT(st.current_set), 2);                               /* theta~ */
        GXPO_OK_OR_DIE(gxpo_slow_step(ctx, l2, NULL));
        gxpo_gate_info info;
        GXPO_OK_OR_DIE(gxpo_gate(ctx, &info, NULL));
    }
    GXPO_OK_OR_DIE(gxpo_get_state(ctx, &st));
    if (st.current_set != (alternating ? 1u : 0u) || st.optim_steps != 7) return 8;
    float *final[3] = {st.current_set ? x.theta_probe : x.theta, st.current_set ? x.m_alt : x.m, st.current_set ? x.v_alt : x.v};
    for (int k = 0; k < 3; ++k) {
        out[k] = (float *)malloc(bytes);
        HIP_OK(hipMemcpy(out[k], final[k], bytes, hipMemcpyDeviceToHost));
    }
    gxpo_destroy(ctx);
    for (int b = 0; b < (alternating ? 6 : 4); ++b) HIP_OK(hipFree(*bufs[b]));
    for (int r = 0; r < 3; ++r) HIP_OK(hipFree(d_g[r]));
    free(h), free(g);
    return 0;
}

int main(void) {
    const double eta = 0.25;
    const unsigned K = 4;
    int n_dev = 0;
    HIP_OK(hipGetDeviceCount(&n_dev));
    if (n_dev < 1) { fprintf(stderr, "no GPU visible\n"); return 2; }
    HIP_OK(hipSetDevice(0));

    gxpo_tensor tensors[N_TENSORS];
    float *d_g[3][N_TENSORS];
    float *h_theta[N_TENSORS], *h_g[N_TENSORS];
    memset(tensors, 0, sizeof tensors);
    for (int t = 0; t < N_TENSORS; ++t) {
        const size_t bytes = numel[t] * sizeof(float);
        tensors[t].numel = numel[t];
        HIP_OK(hipMalloc((void **)&tensors[t].theta, bytes));
        HIP_OK(hipMalloc((void **)&tensors[t].theta_probe, bytes));
        for (int r = 0; r < 3; ++r) HIP_OK(hipMalloc((void **)&d_g[r][t], bytes));
        h_theta[t] = (float *)malloc(bytes);
        h_g[t] = (float *)malloc(bytes);
        for (uint64_t i = 0; i < numel[t]; ++i) h_theta[t][i] = start_of(i + 17 * t);
        HIP_OK(hipMemcpy(tensors[t].theta, h_theta[t], bytes, hipMemcpyHostToDevice));
    }

    gxpo_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.struct_size = sizeof cfg;
    cfg.optimizer = GXPO_OPT_GD;
    cfg.grad_dtype = GXPO_GRAD_F32;
    cfg.K = K;
    cfg.fuse_step2 = 1;
    cfg.window = 4;
    cfg.gate_min_count = 2;
    cfg.lr = eta;
    cfg.alpha = 1.0;
    cfg.delta = 0.0;
    cfg.r_max = INFINITY;
    cfg.tau = 3.0;
    cfg.gate_eps = 1e-8;

    gxpo_ctx *ctx = NULL;
    GXPO_OK_OR_DIE(gxpo_init(&ctx, &cfg, tensors, N_TENSORS));

    /* a call out of Algorithm-1 order is refused and changes nothing */
    const void *lists[3][N_TENSORS];
    for (int r = 0; r < 3; ++r)
        for (int t = 0; t < N_TENSORS; ++t) lists[r][t] = d_g[r][t];
    if (gxpo_slow_step(ctx, lists[2], NULL) != GXPO_ERR_BAD_STATE) { fprintf(stderr, "out-of-order call was not refused\n"); return 4; }

    /* the trainer: gradient of the surrogate at a device buffer, evaluated on the host */
#define GRADIENT_AT(which_buffer, role)                                                            \
    for (int t = 0; t < N_TENSORS; ++t) {                                                          \
        const size_t bytes = numel[t] * sizeof(float);                                             \
        HIP_OK(hipMemcpy(h_theta[t], tensors[t].which_buffer, bytes, hipMemcpyDeviceToHost));      \
        for (uint64_t i = 0; i < numel[t]; ++i)                                                    \
            h_g[t][i] = h_of(i + 5 * t) * (h_theta[t][i] - star_of(i + 3 * t));                    \
        HIP_OK(hipMemcpy(d_g[role][t], h_g[t], bytes, hipMemcpyHostToDevice));                     \
    }

    const int n_steps = 3;
    double last_norm = INFINITY;
    for (int step = 0; step < n_steps; ++step) {
        GRADIENT_AT(theta, 0);
        GXPO_OK_OR_DIE(gxpo_fast_steps(ctx, 0, lists[0], NULL));
        GRADIENT_AT(theta_probe, 1);
        GXPO_OK_OR_DIE(gxpo_fast_steps(ctx, 1, lists[1], NULL));
        GXPO_OK_OR_DIE(gxpo_extrapolate(ctx, lists[0], lists[1], NULL));
        GRADIENT_AT(theta, 2);
        GXPO_OK_OR_DIE(gxpo_slow_step(ctx, lists[2], NULL));
        gxpo_gate_info info;
        GXPO_OK_OR_DIE(gxpo_gate(ctx, &info, NULL));
        /* the norm the gate saw is the norm of the gradient handed in */
        double ss = 0.0;
        for (int t = 0; t < N_TENSORS; ++t)
            for (uint64_t i = 0; i < numel[t]; ++i) ss += (double)h_g[t][i] * (double)h_g[t][i];
        if (fabs(info.norm - sqrt(ss)) > 1e-12 * sqrt(ss)) { fprintf(stderr, "step %d: norm %.17g, expected %.17g\n", step, info.norm, sqrt(ss)); return 5; }
        if (info.tripped || !(info.norm < last_norm)) { fprintf(stderr, "step %d: gate tripped or norm did not shrink\n", step); return 5; }
        last_norm = info.norm;
    }

    /* closed form: n_steps * (K + 1) gradient-descent steps */
    double worst = 0.0;
    for (int t = 0; t < N_TENSORS; ++t) {
        HIP_OK(hipMemcpy(h_theta[t], tensors[t].theta, numel[t] * sizeof(float), hipMemcpyDeviceToHost));
        for (uint64_t i = 0; i < numel[t]; ++i) {
            const double h = h_of(i + 5 * t), star = star_of(i + 3 * t), start = start_of(i + 17 * t);
            const double want = star + pow(1.0 - eta * h, (double)(n_steps * (K + 1))) * (start - star);
            const double err = fabs((double)h_theta[t][i] - want);
            const double allowed = 1e-5 * fabs(want) + 1e-5;
            if (err > allowed) { fprintf(stderr, "tensor %d element %llu: %.9g, closed form %.9g\n", t, (unsigned long long)i, h_theta[t][i], want); return 6; }
            if (err > worst) worst = err;
        }
    }
    gxpo_state st;
    GXPO_OK_OR_DIE(gxpo_get_state(ctx, &st));
    if (st.t != n_steps || st.optim_steps != 3 * n_steps || st.backward_passes != 3 * n_steps || st.s_star != -1) { fprintf(stderr, "state counters are off\n"); return 7; }
    printf("closed form matched on %llu + %llu parameters, largest deviation %.3g\n", (unsigned long long)numel[0], (unsigned long long)numel[1], worst);

    gxpo_destroy(ctx);
    for (int t = 0; t < N_TENSORS; ++t) {
        HIP_OK(hipFree(tensors[t].theta));
        HIP_OK(hipFree(tensors[t].theta_probe));
        for (int r = 0; r < 3; ++r) HIP_OK(hipFree(d_g[r][t]));
        free(h_theta[t]);
        free(h_g[t]);
    }
    /* the second buffer set changes where the results are, not what they are */
    float *in_place[3], *alternating[3];
    int rc = adamw_run(0, in_place);
    if (rc == 0) rc = adamw_run(1, alternating);
    if (rc != 0) { fprintf(stderr, "AdamW run failed (%d)\n", rc); return rc; }
    for (int k = 0; k < 3; ++k)
        if (memcmp(in_place[k], alternating[k], 4099 * sizeof(float)) != 0) { fprintf(stderr, "alternating state: buffer %d differs from the in-place run\n", k); return 9; }
    printf("alternating state: theta, m, v bit-identical to the in-place run after 2 active steps and 1 fallback step\n");
    for (int k = 0; k < 3; ++k) free(in_place[k]), free(alternating[k]);
    puts("abi driver ok");
    return 0;
}
