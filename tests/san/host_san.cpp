// The host-only logic of the C ABI (config validation, block plan, gate rule, the argument checks of
// gxpo_init and of the call entry points that run before the GPU is needed) built with
// -fsanitize=address,undefined.  CPU only: the kernel launchers are replaced by stubs that must never
// be reached, and without a GPU the HIP runtime answers every query with an error the library turns
// into a status code.
#include "gxpo.h"
#include "gxpo_internal.h"

#include <cassert>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

namespace gxpo {
static hipError_t never() {
    fprintf(stderr, "a kernel launcher was reached in a host-only test\n");
    abort();
}
hipError_t launch_step(const Layout &, int, int, const GradArg &, const StepParams &, int, int, int, int, double *, const GradArg &, const float *,
                       int, hipStream_t) { return never(); }
hipError_t launch_sumsq(const Layout &, int, const GradArg &, double *, int, hipStream_t) { return never(); }
hipError_t launch_clip_coefficient(const double *, uint32_t, int, double, float *, int, hipStream_t) { return never(); }
hipError_t launch_extrapolate(const Layout &, int, const GradArg &, const GradArg &, const ExtrapParams &, int, double *, const float *,
                              hipStream_t) { return never(); }
hipError_t launch_reposition(const Layout &, float, int, hipStream_t) { return never(); }
hipError_t launch_fused_steps_extrapolate(const Layout &, int, int, const GradArg &, const GradArg &, const StepParams &, const StepParams &,
                                          const ExtrapParams &, int, int, int, double *, const float *, hipStream_t) { return never(); }
hipError_t launch_finalize(const double *, uint32_t, const SegRec *, uint32_t, const uint32_t *, uint32_t, double *, double *, int, int,
                           hipStream_t) { return never(); }
hipError_t launch_stream_copy(void *, const void *, uint64_t, hipStream_t) { return never(); }
hipError_t launch_slow_step_noalloc(const Layout &, int, int, const GradArg &, const StepParams &, int, double *, hipStream_t) { return never(); }
}  // namespace gxpo

static gxpo_config cfg0() {
    gxpo_config c;
    memset(&c, 0, sizeof c);
    c.struct_size = sizeof c, c.optimizer = GXPO_OPT_ADAMW, c.K = 8, c.fuse_step2 = 1, c.window = 10;
    c.lr = 1e-6, c.beta1 = .9, c.beta2 = .999, c.adam_eps = 1e-8, c.weight_decay = .01, c.alpha = .5, c.delta = 1e-3;
    c.r_max = INFINITY, c.tau = 3, c.gate_eps = 1e-8;
    return c;
}

int main() {
    char msg[8];
    gxpo_config c = cfg0();
    assert(gxpo_validate_config(&c, msg, sizeof msg) == GXPO_OK);
    c.K = 1;
    assert(gxpo_validate_config(&c, msg, sizeof msg) == GXPO_ERR_INVALID_ARG);      // message truncated into 8 bytes
    assert(gxpo_validate_config(nullptr, nullptr, 0) == GXPO_ERR_INVALID_ARG);
    c = cfg0();
    // block plan on random ragged lists
    std::mt19937_64 rng(1);
    for (int rep = 0; rep < 200; ++rep) {
        const uint32_t n = 1 + rng() % 300;
        std::vector<uint64_t> numel(n);
        for (auto &x : numel) x = 1 + rng() % 100000;
        std::vector<uint32_t> start(n + 1);
        uint32_t epb = 0;
        assert(gxpo_plan_blocks(numel.data(), n, start.data(), &epb) == GXPO_OK && epb == 256);
    }
    uint64_t zero = 0, huge = 1ull << 50;
    uint32_t st2[2];
    assert(gxpo_plan_blocks(&zero, 1, st2, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_plan_blocks(&huge, 1, st2, nullptr) == GXPO_ERR_INVALID_ARG);
    // gate: windows 2..256, long runs, NaN
    for (uint32_t w : {2u, 3u, 10u, 255u, 256u}) {
        c.window = w, c.gate_min_count = 0;
        gxpo_state s;
        memset(&s, 0, sizeof s);
        s.struct_size = sizeof s, s.s_star = -1;
        std::normal_distribution<double> nd(10, .1);
        for (int t = 0; t < 1000; ++t) {
            gxpo_gate_info gi;
            assert(gxpo_host_gate_step(&c, &s, t == 700 ? NAN : nd(rng), &gi) == GXPO_OK);
        }
        assert(s.window_len == w && s.t == 1000 && s.s_star >= 0);
        s.window_len = 257;
        assert(gxpo_host_gate_step(&c, &s, 1.0, nullptr) == GXPO_ERR_INVALID_ARG);
    }
    // layout hint
    uint64_t ph = 1, per = 1;
    assert(gxpo_layout_hint(GXPO_BUF_M, &ph, &per) == GXPO_OK && ph == 32768 && per == 65536);
    assert(gxpo_layout_hint(99, &ph, &per) == GXPO_ERR_INVALID_ARG);
    // init argument checks (stop before the GPU is needed, or fail cleanly without one)
    c = cfg0();
    gxpo_ctx *ctx = (gxpo_ctx *)0x1;
    assert(gxpo_init(&ctx, &c, nullptr, 0) == GXPO_ERR_INVALID_ARG && ctx == nullptr);
    gxpo_tensor t;
    memset(&t, 0, sizeof t);
    t.numel = 100;
    t.theta = (float *)0x10000, t.theta_probe = (float *)0x20000, t.m = (float *)0x30000, t.v = (float *)0x40000;
    int rc = gxpo_init(&ctx, &c, &t, 1);      // pointers are not device memory / there is no device
    assert(rc != GXPO_OK && ctx == nullptr && strlen(gxpo_last_error(nullptr)) > 0);
    printf("init on fake pointers: rc=%d (%s)\n", rc, gxpo_last_error(nullptr));
    t.m = (float *)0x10010;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_INVALID_ARG);                  // m overlaps theta
    t.m = (float *)0x30004;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_ALIGNMENT);
    // second buffers for the moments (alternating state): a pair, never half of one; only with the fused AdamW schedule
    t.m = (float *)0x30000, t.m_alt = (float *)0x50000;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_INVALID_ARG && strstr(gxpo_last_error(nullptr), "m_alt"));
    t.v_alt = (float *)0x60000;
    c.fuse_step2 = 0;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_UNSUPPORTED);
    c.fuse_step2 = 1, c.explicit_steps = 3;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_UNSUPPORTED);
    c.explicit_steps = 0;
    t.v_alt = (float *)0x40010;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_INVALID_ARG);                  // v_alt overlaps v
    t.v_alt = (float *)0x60000, t.theta_probe = nullptr;
    assert(gxpo_init(&ctx, &c, &t, 1) == GXPO_ERR_INVALID_ARG);                  // no second parameter buffer
    t.theta_probe = (float *)0x20000, t.m_alt = t.v_alt = nullptr;
    // entry points on a NULL context / NULL arguments
    assert(gxpo_fast_steps(nullptr, 0, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_extrapolate(nullptr, nullptr, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_slow_step(nullptr, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_gate(nullptr, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_fallback_step(nullptr, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_get_state(nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_current_params(nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_set_state(nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_update_config(nullptr, &c) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_set_tensor_options(nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_tensor_norms(nullptr, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_get_diagnostics(nullptr, nullptr, nullptr) == GXPO_ERR_INVALID_ARG);
    // the entry point without a context: argument checks that need no GPU
    t.m = (float *)0x30000;
    double *out = (double *)0x50000;
    assert(gxpo_slow_step_noalloc(&c, nullptr, 1, (void *)0x60000, out, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_slow_step_noalloc(&c, &t, 0, (void *)0x60000, out, nullptr) == GXPO_ERR_INVALID_ARG);
    t.numel = GXPO_NOALLOC_MAX_NUMEL + 1;
    assert(gxpo_slow_step_noalloc(&c, &t, 1, (void *)0x60000, out, nullptr) == GXPO_ERR_INVALID_ARG);
    t.numel = 100;
    assert(gxpo_slow_step_noalloc(&c, &t, 1, (void *)0x60004, out, nullptr) == GXPO_ERR_ALIGNMENT);
    rc = gxpo_slow_step_noalloc(&c, &t, 1, (void *)0x60000, out, nullptr);      // not device memory
    assert(rc != GXPO_OK);
    c.clip_norm = 1.0;
    assert(gxpo_slow_step_noalloc(&c, &t, 1, (void *)0x60000, out, nullptr) == GXPO_ERR_UNSUPPORTED);
    assert(gxpo_stream_copy(nullptr, nullptr, 16, nullptr) == GXPO_ERR_INVALID_ARG);
    assert(gxpo_stream_copy((void *)0x10000, (void *)0x20000, 17, nullptr) == GXPO_ERR_ALIGNMENT);
    gxpo_destroy(nullptr);
    puts("host logic clean under ASan + UBSan");
    return 0;
}
