// Host side of the GXPO update engine: the C ABI of include/gxpo.h, argument
// validation, the Algorithm-1 call-order state machine, the block plan for
// ragged tensor lists, gradient-pointer tables, and the rolling z-score gate.
#include "gxpo.h"
#include "gxpo_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <new>
#include <string>
#include <vector>

using namespace gxpo;

namespace {

thread_local std::string g_init_error = "";

std::string format(const char *fmt, va_list ap) {
    char buf[512];
    vsnprintf(buf, sizeof buf, fmt, ap);
    return std::string(buf);
}

constexpr int kGradRoles = 3;        // g0, g1, g_slow
constexpr int kStageSlots = 8;       // pinned staging slots for pointer-table uploads
enum { kRoleG0 = 0, kRoleG1 = 1, kRoleSlow = 2 };

struct Interval { uintptr_t lo, hi; uint32_t t; const char *what; };

}  // namespace

struct gxpo_ctx {
    gxpo_config cfg{};
    uint32_t n = 0;
    int device = -1;
    std::vector<gxpo_tensor> tensors;
    std::vector<gxpo_tensor_options> options;   // parameter groups, all {1, 1} unless set
    std::vector<uint32_t> blk_start;
    std::vector<Interval> owned;             // every engine buffer, sorted by address, pairwise disjoint

    // device tables
    TensorRec *d_tab = nullptr;
    uint32_t *d_blk_start = nullptr;
    uint32_t *d_coarse = nullptr;
    const void **d_grads = nullptr;          // [kGradRoles][n]
    // reduction workspace
    double *d_partial = nullptr;             // one per block
    SegRec *d_seg = nullptr;
    uint32_t *d_tensor_seg_start = nullptr;
    double *d_seg_sum = nullptr;
    double *d_result = nullptr;              // [n_acc][1 + n]
    float *d_clip = nullptr;                 // clipping factors of g0, g1, g_slow (nullptr: clipping off)
    double *h_result = nullptr;              // pinned, [1 + n]
    uint32_t n_blocks = 0, n_segs = 0;
    bool have_norms = false;
    bool have_diag = false, cos_valid = false;
    int64_t diag_t = -1;
    uint32_t n_acc = 1;                      // accumulators the workspace holds (1, or kNumAcc with diagnostics)
    bool alternating = false;                // every tensor brought m_alt, v_alt: passes read one set and write the other

    // gradient pointer staging
    const void **h_stage = nullptr;          // pinned, [kStageSlots][n]
    hipEvent_t stage_event[kStageSlots]{};
    bool stage_used[kStageSlots]{};
    int next_slot = 0;
    std::vector<const void *> shadow[kGradRoles];
    std::vector<const void *> pending_g0;    // fuse_step2: the gradients the probe pass used
    std::vector<const void *> pending_g1;    // fuse_step2: recorded by gxpo_fast_steps(1)
    uint32_t fast_done = 0;                  // fast steps taken in the current training step
    int64_t pending_step1 = 0;               // optimizer step numbers of the two fast steps the
    int64_t pending_step2 = 0;               //   fused pass applies

    gxpo_state st{};
    mutable std::string err;

    TensorRec record(uint32_t t) const {
        const gxpo_tensor &x = tensors[t];
        const gxpo_tensor_options &o = options[t];
        return TensorRec{x.theta, x.theta_probe, x.m, x.v, x.model_copy, x.m_alt, x.v_alt, x.numel, (float)o.lr_scale,
                         (float)(o.lr_scale * o.weight_decay_scale)};
    }
    Layout layout() const { return Layout{d_tab, d_blk_start, d_coarse, n, n_blocks, record(0)}; }
    // the set that holds the state, and the set a state-advancing pass writes
    int cur_set() const { return st.current_set ? kSetAlt : kSetMain; }
    int next_set() const { return alternating ? (st.current_set ? kSetMain : kSetAlt) : kSetMain; }
    void advance_set() { if (alternating) st.current_set ^= 1u; }
};

namespace {

int fail(const gxpo_ctx *ctx, int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    std::string msg = format(fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = msg;
    else g_init_error = msg;
    return code;
}

int fail_hip(const gxpo_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, GXPO_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define GXPO_HIP(ctx, call)                                    \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return fail_hip(ctx, e_, #call); \
    } while (0)

int check_config(const gxpo_config *c, std::string &msg) {
    auto bad = [&](const char *m) { msg = m; return (int)GXPO_ERR_INVALID_ARG; };
    if (!c) return bad("config is NULL");
    if (c->struct_size != sizeof(gxpo_config)) return bad("config.struct_size does not match this library");
    if (c->optimizer != GXPO_OPT_GD && c->optimizer != GXPO_OPT_ADAMW) { msg = "unknown optimizer"; return GXPO_ERR_UNSUPPORTED; }
    if (c->grad_dtype != GXPO_GRAD_F32 && c->grad_dtype != GXPO_GRAD_BF16) { msg = "unknown grad_dtype"; return GXPO_ERR_UNSUPPORTED; }
    if (c->K < 2) return bad("K must be >= 2");
    if (c->K > 4096) return bad("K must be <= 4096");
    if (c->fuse_step2 > 1) return bad("fuse_step2 must be 0 or 1");
    if (c->copy_mask & ~7u) return bad("copy_mask has unknown bits");
    if (c->window < 2 || c->window > GXPO_MAX_WINDOW) return bad("window must be in [2, GXPO_MAX_WINDOW]");
    if (c->gate_min_count == 1 || c->gate_min_count > c->window) return bad("gate_min_count must be 0 or in [2, window]");
    if (c->gate_ddof > 1) return bad("gate_ddof must be 0 or 1");
    if (c->diagnostics > 1) return bad("diagnostics must be 0 or 1");
    if (c->explicit_steps == 1 || c->explicit_steps > 4096) return bad("explicit_steps must be 0 or in [2, 4096]");
    if (c->explicit_steps && c->diagnostics) return bad("diagnostics need the extrapolation (explicit_steps == 0)");
    if (!(c->lr > 0.0) || !std::isfinite(c->lr)) return bad("lr must be finite and > 0");
    if (c->optimizer == GXPO_OPT_ADAMW) {
        if (!(c->beta1 >= 0.0 && c->beta1 < 1.0)) return bad("beta1 must be in [0, 1)");
        if (!(c->beta2 >= 0.0 && c->beta2 < 1.0)) return bad("beta2 must be in [0, 1)");
        if (!(c->adam_eps >= 0.0) || !std::isfinite(c->adam_eps)) return bad("adam_eps must be finite and >= 0");
        if (!(c->weight_decay >= 0.0) || !std::isfinite(c->weight_decay)) return bad("weight_decay must be finite and >= 0");
    }
    if (!(c->alpha >= 0.0 && c->alpha <= 1.0)) return bad("alpha must be in [0, 1]");
    if (!(c->delta >= 0.0)) return bad("delta must be >= 0 (+inf allowed)");
    if (!(c->r_max > 0.0)) return bad("r_max must be > 0 (+inf = no clamp)");
    if (!(c->clip_norm >= 0.0) || !std::isfinite(c->clip_norm)) return bad("clip_norm must be finite and >= 0 (0 = off)");
    if (std::isnan(c->tau)) return bad("tau is NaN");
    if (!(c->gate_eps > 0.0) || !std::isfinite(c->gate_eps)) return bad("gate_eps must be finite and > 0");
    return GXPO_OK;
}

int plan_blocks(const uint64_t *numel, uint32_t n, std::vector<uint32_t> &start, std::string &msg) {
    const uint64_t epb = kWaveElems;
    start.assign((size_t)n + 1, 0);
    uint64_t total = 0;
    for (uint32_t t = 0; t < n; ++t) {
        if (numel[t] == 0) { msg = "a tensor has numel == 0"; return GXPO_ERR_INVALID_ARG; }
        start[t] = (uint32_t)total;
        total += (numel[t] + epb - 1) / epb;
        if (total > 0x7fffffffull) { msg = "too many elements for one launch grid"; return GXPO_ERR_INVALID_ARG; }
    }
    start[n] = (uint32_t)total;
    return GXPO_OK;
}

// Is every byte of [p, p + bytes) device memory of the current GPU?  Usually the range lies in one
// allocation; a buffer assembled from physical chunks mapped back to back into one reserved
// address range (HIP's virtual-memory API) is a run of adjacent allocations, which is walked.
int check_device_range(const gxpo_ctx *ctx, const void *p, uint64_t bytes, const char *what, uint32_t t) {
    const char *q = (const char *)p, *const end = q + bytes;
    for (int hops = 0; q < end; ++hops) {
        hipDeviceptr_t base = nullptr;
        size_t size = 0;
        hipError_t e = hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)q);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            if (hops == 0)
                return fail(ctx, GXPO_ERR_INVALID_ARG, "tensor %u: %s is not a device allocation (%s)", t, what, hipGetErrorString(e));
            return fail(ctx, GXPO_ERR_INVALID_ARG, "tensor %u: %s + numel runs past the end of its device allocation", t, what);
        }
        const char *b = (const char *)base;
        if (q < b || q >= b + size || size == 0)
            return fail(ctx, GXPO_ERR_INVALID_ARG, "tensor %u: %s + numel runs past the end of its device allocation", t, what);
        q = b + size;                              // first byte after this allocation
        if (hops > (1 << 20)) return fail(ctx, GXPO_ERR_INVALID_ARG, "tensor %u: %s spans too many allocations", t, what);
    }
    return GXPO_OK;
}

template <typename T> int dev_alloc(gxpo_ctx *ctx, T **p, size_t count) {
    hipError_t e = hipMalloc((void **)p, std::max<size_t>(count, 1) * sizeof(T));
    if (e != hipSuccess) { *p = nullptr; return fail(nullptr, GXPO_ERR_NOMEM, "hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e)); }
    (void)ctx;
    return GXPO_OK;
}

bool is_fallback_phase(const gxpo_state &s) { return s.s_star >= 0 && s.t >= s.s_star; }

StepParams make_step_params(const gxpo_config &c, int64_t s) {
    StepParams p{};
    p.lr = (float)c.lr;
    if (c.optimizer == GXPO_OPT_ADAMW) {
        p.beta1 = (float)c.beta1;
        p.one_minus_beta1 = (float)(1.0 - c.beta1);
        p.beta2 = (float)c.beta2;
        p.one_minus_beta2 = (float)(1.0 - c.beta2);
        p.lr_wd = (float)(c.lr * c.weight_decay);
        p.step_size = (float)(c.lr / (1.0 - std::pow(c.beta1, (double)s)));
        p.rsqrt_bias2 = (float)(1.0 / std::sqrt(1.0 - std::pow(c.beta2, (double)s)));
        p.eps = (float)c.adam_eps;
    }
    return p;
}

ExtrapParams make_extrap_params(const gxpo_config &c) {
    ExtrapParams e{};
    e.alpha = (float)c.alpha;
    e.delta = (float)c.delta;
    e.r_max = (float)c.r_max;
    e.odd = c.K & 1u;
    e.half = e.odd ? (c.K - 1) / 2 : c.K / 2;
    return e;
}

int check_call(gxpo_ctx *ctx, const void *const *grads, const char *name) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!grads) return fail(ctx, GXPO_ERR_INVALID_ARG, "%s: gradient list is NULL", name);
    int dev = -1;
    GXPO_HIP(ctx, hipGetDevice(&dev));
    if (dev != ctx->device)
        return fail(ctx, GXPO_ERR_INVALID_ARG, "%s: current device %d is not the context's device %d", name, dev, ctx->device);
    return GXPO_OK;
}

// The engine buffer that [p, p + bytes) touches, or nullptr.
const Interval *overlapping_buffer(const gxpo_ctx *ctx, const void *p, uint64_t bytes) {
    const uintptr_t lo = (uintptr_t)p, hi = lo + bytes;
    // first owned interval that ends after lo; the intervals are disjoint, so their ends are sorted too
    auto it = std::upper_bound(ctx->owned.begin(), ctx->owned.end(), lo, [](uintptr_t x, const Interval &iv) { return x < iv.hi; });
    return (it != ctx->owned.end() && it->lo < hi) ? &*it : nullptr;
}

// Make the device pointer table of `role` hold `grads`; returns the device table.
int stage_grads(gxpo_ctx *ctx, int role, const void *const *grads, hipStream_t stream, GradArg *d_out) {
    const uint32_t n = ctx->n;
    const uint32_t gbytes = ctx->cfg.grad_dtype == GXPO_GRAD_F32 ? 4u : 2u;
    const uintptr_t align = ctx->cfg.grad_dtype == GXPO_GRAD_F32 ? 16u : 8u;
    std::vector<const void *> &sh = ctx->shadow[role];
    bool changed = false;
    for (uint32_t t = 0; t < n; ++t) {
        const void *g = grads[t];
        // NULL first: the shadow table starts out all NULL, so a NULL entry would otherwise pass as "unchanged"
        if (!g) return fail(ctx, GXPO_ERR_INVALID_ARG, "gradient pointer of tensor %u is NULL", t);
        if (g == sh[t]) continue;
        if ((uintptr_t)g % align) return fail(ctx, GXPO_ERR_ALIGNMENT, "gradient pointer of tensor %u is not %u-byte aligned", t, (unsigned)align);
        int rc = check_device_range(ctx, g, ctx->tensors[t].numel * gbytes, "gradient", t);
        if (rc != GXPO_OK) return rc;
        if (const Interval *hit = overlapping_buffer(ctx, g, ctx->tensors[t].numel * gbytes))
            return fail(ctx, GXPO_ERR_INVALID_ARG, "gradient of tensor %u overlaps %s of tensor %u", t, hit->what, hit->t);
        changed = true;
    }
    const void **d_tab = ctx->d_grads + (size_t)role * n;
    if (changed) {
        const int slot = ctx->next_slot;
        ctx->next_slot = (slot + 1) % kStageSlots;
        if (ctx->stage_used[slot]) GXPO_HIP(ctx, hipEventSynchronize(ctx->stage_event[slot]));
        const void **h = ctx->h_stage + (size_t)slot * n;
        std::memcpy(h, grads, sizeof(void *) * n);
        GXPO_HIP(ctx, hipMemcpyAsync(d_tab, h, sizeof(void *) * n, hipMemcpyHostToDevice, stream));
        GXPO_HIP(ctx, hipEventRecord(ctx->stage_event[slot], stream));
        ctx->stage_used[slot] = true;
        sh.assign(grads, grads + n);
    }
    *d_out = GradArg{d_tab, grads[0]};
    return GXPO_OK;
}

// Gradient clipping: norm of the staged gradient list -> its clipping factor on the device.
int clip_prepass(gxpo_ctx *ctx, const GradArg &g, int acc, int clip_index, hipStream_t s) {
    if (!ctx->d_clip) return GXPO_OK;
    GXPO_HIP(ctx, launch_sumsq(ctx->layout(), (int)ctx->cfg.grad_dtype, g, ctx->d_partial, acc, s));
    GXPO_HIP(ctx, launch_finalize(ctx->d_partial, ctx->n_blocks, ctx->d_seg, ctx->n_segs, ctx->d_tensor_seg_start, ctx->n,
                                  ctx->d_seg_sum, ctx->d_result, acc, 1, s));
    GXPO_HIP(ctx, launch_clip_coefficient(ctx->d_result, ctx->n, acc, ctx->cfg.clip_norm, ctx->d_clip, clip_index, s));
    return GXPO_OK;
}

void release(gxpo_ctx *ctx) {
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    (void)hipFree(ctx->d_tab);
    (void)hipFree(ctx->d_blk_start);
    (void)hipFree(ctx->d_coarse);
    (void)hipFree((void *)ctx->d_grads);
    (void)hipFree(ctx->d_partial);
    (void)hipFree(ctx->d_seg);
    (void)hipFree(ctx->d_tensor_seg_start);
    (void)hipFree(ctx->d_seg_sum);
    (void)hipFree(ctx->d_result);
    (void)hipFree(ctx->d_clip);
    if (ctx->h_result) (void)hipHostFree(ctx->h_result);
    if (ctx->h_stage) (void)hipHostFree((void *)ctx->h_stage);
    for (int i = 0; i < kStageSlots; ++i)
        if (ctx->stage_event[i]) (void)hipEventDestroy(ctx->stage_event[i]);
    delete ctx;
}

}  // namespace

// ---------------------------------------------------------------------------------------
extern "C" {

int gxpo_validate_config(const gxpo_config *cfg, char *msg, size_t cap) {
    std::string m;
    int rc = check_config(cfg, m);
    if (msg && cap) {
        std::snprintf(msg, cap, "%s", m.c_str());
    }
    return rc;
}

int gxpo_plan_blocks(const uint64_t *numel, uint32_t n_tensors, uint32_t *block_start, uint32_t *elems_per_block) {
    if (!numel || !block_start || n_tensors == 0) return GXPO_ERR_INVALID_ARG;
    std::vector<uint32_t> start;
    std::string msg;
    int rc = plan_blocks(numel, n_tensors, start, msg);
    if (rc != GXPO_OK) return rc;
    std::copy(start.begin(), start.end(), block_start);
    if (elems_per_block) *elems_per_block = kWaveElems;
    return GXPO_OK;
}

int gxpo_layout_hint(int buffer_kind, uint64_t *phase_bytes, uint64_t *period_bytes) {
    if (!phase_bytes || !period_bytes || buffer_kind < GXPO_BUF_THETA || buffer_kind > GXPO_BUF_GRAD) return GXPO_ERR_INVALID_ARG;
    // the moments sit half a period away from everything else, which splits the traffic of every
    // pass about evenly between the two halves of the period
    *period_bytes = 64u * 1024u;
    *phase_bytes = (buffer_kind == GXPO_BUF_M || buffer_kind == GXPO_BUF_V) ? 32u * 1024u : 0u;
    return GXPO_OK;
}

int gxpo_host_gate_step(const gxpo_config *cfg, gxpo_state *st, double norm, gxpo_gate_info *out) {
    if (!cfg || !st) return GXPO_ERR_INVALID_ARG;
    if (st->window_len > GXPO_MAX_WINDOW || cfg->window < 2 || cfg->window > GXPO_MAX_WINDOW) return GXPO_ERR_INVALID_ARG;
    const uint32_t min_count = cfg->gate_min_count ? cfg->gate_min_count : cfg->window;
    const uint32_t len = st->window_len;
    gxpo_gate_info info{};
    info.norm = norm;
    info.mu = info.sigma = info.z = std::numeric_limits<double>::quiet_NaN();
    info.t = st->t;
    bool tripped = false;
    if (len >= min_count && len > cfg->gate_ddof) {
        // mean and deviation of the buffer as it stands, i.e. before this norm goes in
        double sum = 0.0;
        for (uint32_t i = 0; i < len; ++i) sum += st->window[i];
        const double mu = sum / len;
        double ss = 0.0;
        for (uint32_t i = 0; i < len; ++i) ss += (st->window[i] - mu) * (st->window[i] - mu);
        const double sigma = std::sqrt(ss / (len - cfg->gate_ddof));
        info.evaluated = 1;
        info.mu = mu;
        info.sigma = sigma;
        info.z = (norm - mu) / (sigma + cfg->gate_eps);
        tripped = info.z >= cfg->tau;
    }
    if (!std::isfinite(norm)) tripped = true;
    if (tripped && st->s_star < 0) st->s_star = st->t + 1;
    // push, dropping the oldest beyond w
    if (len == cfg->window) {
        std::memmove(&st->window[0], &st->window[1], sizeof(double) * (len - 1));
        st->window[len - 1] = norm;
    } else {
        st->window[len] = norm;
        st->window_len = len + 1;
    }
    info.tripped = (st->s_star >= 0) ? 1 : 0;
    info.s_star = st->s_star;
    st->t += 1;
    if (out) *out = info;
    return GXPO_OK;
}

const char *gxpo_last_error(const gxpo_ctx *ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

int gxpo_init(gxpo_ctx **out, const gxpo_config *cfg, const gxpo_tensor *tensors, uint32_t n_tensors) {
    if (!out) return fail(nullptr, GXPO_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::string msg;
    int rc = check_config(cfg, msg);
    if (rc != GXPO_OK) return fail(nullptr, rc, "%s", msg.c_str());
    if (!tensors || n_tensors == 0) return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor list is empty");

    const bool adam = cfg->optimizer == GXPO_OPT_ADAMW;
    std::vector<uint64_t> numel(n_tensors);
    for (uint32_t t = 0; t < n_tensors; ++t) {
        const gxpo_tensor &x = tensors[t];
        numel[t] = x.numel;
        if (x.numel == 0) return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor %u: numel is 0", t);
        if (!x.theta) return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor %u: theta is NULL", t);
        if (adam && (!x.m || !x.v)) return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor %u: AdamW needs m and v", t);
        if (!adam && (x.m || x.v)) return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor %u: m and v must be NULL for plain GD", t);
        if ((x.m_alt == nullptr) != (x.v_alt == nullptr) || (x.m_alt != nullptr) != (tensors[0].m_alt != nullptr))
            return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor %u: m_alt and v_alt come together, for every tensor or for none", t);
        if (x.m_alt && !x.theta_probe)
            return fail(nullptr, GXPO_ERR_INVALID_ARG, "tensor %u: alternating state (m_alt, v_alt) needs theta_probe as the second parameter buffer", t);
        if (x.m_alt && (!adam || !cfg->fuse_step2 || cfg->explicit_steps))
            return fail(nullptr, GXPO_ERR_UNSUPPORTED, "alternating state (m_alt, v_alt) needs AdamW, fuse_step2 = 1 and explicit_steps = 0");
        const void *f32[] = {x.theta, x.theta_probe, x.m, x.v, x.m_alt, x.v_alt};
        for (const void *p : f32)
            if (p && (uintptr_t)p % 16) return fail(nullptr, GXPO_ERR_ALIGNMENT, "tensor %u: an fp32 buffer is not 16-byte aligned", t);
        if (x.model_copy && (uintptr_t)x.model_copy % 8)
            return fail(nullptr, GXPO_ERR_ALIGNMENT, "tensor %u: model_copy is not 8-byte aligned", t);
    }
    std::vector<uint32_t> blk_start;
    rc = plan_blocks(numel.data(), n_tensors, blk_start, msg);
    if (rc != GXPO_OK) return fail(nullptr, rc, "%s", msg.c_str());

    // buffers must not overlap one another
    std::vector<Interval> iv;
    for (uint32_t t = 0; t < n_tensors; ++t) {
        const gxpo_tensor &x = tensors[t];
        auto add = [&](const void *p, uint64_t bytes, const char *what) {
            if (p) iv.push_back({(uintptr_t)p, (uintptr_t)p + bytes, t, what});
        };
        add(x.theta, x.numel * 4, "theta");
        add(x.theta_probe, x.numel * 4, "theta_probe");
        add(x.m, x.numel * 4, "m");
        add(x.v, x.numel * 4, "v");
        add(x.m_alt, x.numel * 4, "m_alt");
        add(x.v_alt, x.numel * 4, "v_alt");
        add(x.model_copy, x.numel * 2, "model_copy");
    }
    std::sort(iv.begin(), iv.end(), [](const Interval &a, const Interval &b) { return a.lo < b.lo; });
    for (size_t i = 1; i < iv.size(); ++i)
        if (iv[i].lo < iv[i - 1].hi)
            return fail(nullptr, GXPO_ERR_INVALID_ARG, "%s of tensor %u overlaps %s of tensor %u", iv[i].what, iv[i].t,
                        iv[i - 1].what, iv[i - 1].t);

    // from here on the GPU is needed
    int device = -1;
    hipError_t he = hipGetDevice(&device);
    if (he != hipSuccess) return fail_hip(nullptr, he, "hipGetDevice");
    for (const Interval &x : iv) {
        rc = check_device_range(nullptr, (const void *)x.lo, x.hi - x.lo, x.what, x.t);
        if (rc != GXPO_OK) return rc;
    }

    gxpo_ctx *ctx = new (std::nothrow) gxpo_ctx();
    if (!ctx) return fail(nullptr, GXPO_ERR_NOMEM, "out of host memory");
    ctx->cfg = *cfg;
    ctx->n = n_tensors;
    ctx->n_acc = (cfg->diagnostics || cfg->clip_norm > 0.0) ? (uint32_t)kNumAcc : 1u;
    ctx->device = device;
    ctx->alternating = tensors[0].m_alt != nullptr;
    ctx->tensors.assign(tensors, tensors + n_tensors);
    ctx->options.assign(n_tensors, gxpo_tensor_options{1.0, 1.0});
    ctx->blk_start = blk_start;
    ctx->owned = iv;
    ctx->n_blocks = blk_start[n_tensors];
    for (auto &s : ctx->shadow) s.assign(n_tensors, nullptr);
    ctx->st.struct_size = sizeof(gxpo_state);
    ctx->st.phase = GXPO_PHASE_IDLE;
    ctx->st.s_star = -1;

    // runs of partials, per tensor, for the fixed-order reduction
    std::vector<SegRec> segs;
    std::vector<uint32_t> tensor_seg_start(n_tensors + 1, 0);
    for (uint32_t t = 0; t < n_tensors; ++t) {
        tensor_seg_start[t] = (uint32_t)segs.size();
        for (uint32_t b = blk_start[t]; b < blk_start[t + 1]; b += kSegPartials)
            segs.push_back({b, std::min(kSegPartials, blk_start[t + 1] - b)});
    }
    tensor_seg_start[n_tensors] = (uint32_t)segs.size();
    ctx->n_segs = (uint32_t)segs.size();

    std::vector<TensorRec> tab(n_tensors);
    for (uint32_t t = 0; t < n_tensors; ++t) tab[t] = ctx->record(t);
    std::vector<uint32_t> coarse;
    if (n_tensors > 1) {
        coarse.resize(((size_t)ctx->n_blocks >> kCoarseShift) + 1);
        uint32_t t = 0;
        for (size_t c = 0; c < coarse.size(); ++c) {
            const uint64_t b = (uint64_t)c << kCoarseShift;
            while (t + 1 < n_tensors && blk_start[t + 1] <= b) ++t;
            coarse[c] = t;
        }
    }

    auto up = [&](void *dst, const void *src, size_t bytes) { return hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice); };
    rc = dev_alloc(ctx, &ctx->d_tab, n_tensors);
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_blk_start, (size_t)n_tensors + 1);
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_coarse, coarse.size());
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_grads, (size_t)kGradRoles * n_tensors);
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_partial, (size_t)ctx->n_acc * partial_pitch(ctx->n_blocks));
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_seg, segs.size());
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_tensor_seg_start, (size_t)n_tensors + 1);
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_seg_sum, (size_t)ctx->n_acc * segs.size());
    if (rc == GXPO_OK) rc = dev_alloc(ctx, &ctx->d_result, (size_t)ctx->n_acc * ((size_t)n_tensors + 1));
    if (rc == GXPO_OK && cfg->clip_norm > 0.0) rc = dev_alloc(ctx, &ctx->d_clip, 3);
    if (rc != GXPO_OK) { release(ctx); return rc; }
    he = hipHostMalloc((void **)&ctx->h_result, sizeof(double) * ctx->n_acc * ((size_t)n_tensors + 1), hipHostMallocDefault);
    if (he == hipSuccess) he = hipHostMalloc((void **)&ctx->h_stage, sizeof(void *) * (size_t)kStageSlots * n_tensors, hipHostMallocDefault);
    for (int i = 0; he == hipSuccess && i < kStageSlots; ++i) he = hipEventCreateWithFlags(&ctx->stage_event[i], hipEventDisableTiming);
    if (he == hipSuccess) he = up(ctx->d_tab, tab.data(), sizeof(TensorRec) * n_tensors);
    if (he == hipSuccess) he = up(ctx->d_blk_start, blk_start.data(), sizeof(uint32_t) * (n_tensors + 1));
    if (he == hipSuccess && !coarse.empty()) he = up(ctx->d_coarse, coarse.data(), sizeof(uint32_t) * coarse.size());
    if (he == hipSuccess) he = up(ctx->d_seg, segs.data(), sizeof(SegRec) * segs.size());
    if (he == hipSuccess) he = up(ctx->d_tensor_seg_start, tensor_seg_start.data(), sizeof(uint32_t) * (n_tensors + 1));
    if (he == hipSuccess) he = hipMemset(ctx->d_grads, 0, sizeof(void *) * kGradRoles * n_tensors);
    if (he == hipSuccess) he = hipMemset(ctx->d_result, 0, sizeof(double) * ctx->n_acc * (n_tensors + 1));
    if (he == hipSuccess) he = hipDeviceSynchronize();
    if (he != hipSuccess) { release(ctx); return fail_hip(nullptr, he, "gxpo_init device set-up"); }
    *out = ctx;
    return GXPO_OK;
}

void gxpo_destroy(gxpo_ctx *ctx) { release(ctx); }

int gxpo_fast_steps(gxpo_ctx *ctx, int which, const void *const *grads, void *stream) {
    int rc = check_call(ctx, grads, "gxpo_fast_steps");
    if (rc != GXPO_OK) return rc;
    const uint32_t n_fast = ctx->cfg.explicit_steps ? ctx->cfg.explicit_steps : 2u;
    if (which < 0 || (uint32_t)which >= n_fast)
        return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_fast_steps: which must be in [0, %u)", n_fast);
    gxpo_state &st = ctx->st;
    if (is_fallback_phase(st)) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_fast_steps: the gate has tripped (s* = %lld), use gxpo_fallback_step", (long long)st.s_star);
    const bool in_order = which == 0 ? st.phase == GXPO_PHASE_IDLE : (st.phase == GXPO_PHASE_FAST1 && ctx->fast_done == (uint32_t)which);
    if (!in_order) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_fast_steps(%d) called in phase %u after %u fast steps", which, st.phase, ctx->fast_done);
    const bool fused = ctx->cfg.fuse_step2 != 0 && !ctx->cfg.explicit_steps;
    const bool copy_at_probe = (ctx->cfg.copy_mask & GXPO_COPY_AT_PROBE) != 0;
    for (uint32_t t = 0; t < ctx->n; ++t) {
        const gxpo_tensor &x = ctx->tensors[t];
        if (!x.theta_probe && !(fused && copy_at_probe && x.model_copy))
            return fail(ctx, GXPO_ERR_INVALID_ARG,
                        "tensor %u has no theta_probe: the active phase needs it unless fuse_step2 is set and theta^{t,1} goes to model_copy", t);
    }
    if (which == 1 && !ctx->cfg.explicit_steps) {
        // the extrapolation reads g0 and g1 side by side: g1 must not have been written over g0
        const uint64_t gbytes = ctx->cfg.grad_dtype == GXPO_GRAD_F32 ? 4u : 2u;
        for (uint32_t t = 0; t < ctx->n; ++t) {
            const uintptr_t a = (uintptr_t)ctx->shadow[kRoleG0][t], b = (uintptr_t)grads[t];
            const uint64_t bytes = ctx->tensors[t].numel * gbytes;
            if (b && a < b + bytes && b < a + bytes)
                return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_fast_steps(1): g1 of tensor %u overlaps g0, which gxpo_extrapolate still needs", t);
        }
    }
    hipStream_t s = (hipStream_t)stream;
    GradArg d_g{};
    rc = stage_grads(ctx, which == 0 ? kRoleG0 : kRoleG1, grads, s, &d_g);
    if (rc != GXPO_OK) return rc;
    const int64_t step_no = st.optim_steps + 1;
    rc = clip_prepass(ctx, d_g, which == 0 ? kAccClipG0 : kAccClipG1, which == 0 ? kClipG0 : kClipG1, s);
    if (rc != GXPO_OK) return rc;
    if (which == 1 && fused) {
        ctx->pending_g1.assign(grads, grads + ctx->n);
        ctx->pending_step2 = step_no;
    } else {
        const StepParams p = make_step_params(ctx->cfg, step_no);
        // the first fast step reads the current set and writes theta^{t,1} into the other set's parameter buffer
        // (alternating state: whichever of theta / theta_probe is not current); the unfused second step works on theta_probe
        const int src = which == 0 ? ctx->cur_set() : kSrcProbe;
        const int dst = (which == 0 && ctx->st.current_set) ? kSrcTheta : kSrcProbe;
        // the trainer differentiates at theta^{t,1}; with explicit lookahead at every probe iterate
        const int wc = ((which == 0 || ctx->cfg.explicit_steps) && copy_at_probe) ? 1 : 0;
        // fused schedule: the probe pass only previews the step, the moments are advanced by gxpo_extrapolate
        const int write_moments = fused ? 0 : 1;
        GXPO_HIP(ctx, launch_step(ctx->layout(), (int)ctx->cfg.optimizer, (int)ctx->cfg.grad_dtype, d_g, p, src, dst,
                                  write_moments, wc, nullptr, GradArg{}, ctx->d_clip, which == 0 ? kClipG0 : kClipG1, s));
        if (fused) {
            ctx->pending_g0.assign(grads, grads + ctx->n);
            ctx->pending_step1 = step_no;
        }
    }
    st.optim_steps = step_no;
    st.backward_passes += 1;
    ctx->fast_done = (uint32_t)which + 1;
    st.phase = ctx->fast_done == n_fast ? GXPO_PHASE_FAST2 : GXPO_PHASE_FAST1;
    return GXPO_OK;
}

int gxpo_extrapolate(gxpo_ctx *ctx, const void *const *g0, const void *const *g1, void *stream) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (ctx->cfg.explicit_steps) {
        // explicit lookahead: the probe trajectory was walked for real, only the reposition is left
        static const void *const no_grads[1] = {nullptr};
        int rc0 = check_call(ctx, no_grads, "gxpo_extrapolate");
        if (rc0 != GXPO_OK) return rc0;
        if (ctx->st.phase != GXPO_PHASE_FAST2) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_extrapolate called in phase %u", ctx->st.phase);
        const int wc0 = (ctx->cfg.copy_mask & GXPO_COPY_AT_TILDE) ? 1 : 0;
        GXPO_HIP(ctx, launch_reposition(ctx->layout(), (float)ctx->cfg.alpha, wc0, (hipStream_t)stream));
        ctx->st.phase = GXPO_PHASE_REPOSITIONED;
        return GXPO_OK;
    }
    int rc = check_call(ctx, g0, "gxpo_extrapolate");
    if (rc != GXPO_OK) return rc;
    if (!g1) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_extrapolate: g1 list is NULL");
    gxpo_state &st = ctx->st;
    if (st.phase != GXPO_PHASE_FAST2) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_extrapolate called in phase %u", st.phase);
    hipStream_t s = (hipStream_t)stream;
    if (ctx->cfg.fuse_step2)
        for (uint32_t t = 0; t < ctx->n; ++t) {
            if (g0[t] != ctx->pending_g0[t])
                return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_extrapolate: g0 of tensor %u differs from the one given to gxpo_fast_steps(0)", t);
            if (g1[t] != ctx->pending_g1[t])
                return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_extrapolate: g1 of tensor %u differs from the one given to gxpo_fast_steps(1)", t);
        }
    GradArg d_g0{}, d_g1{};
    rc = stage_grads(ctx, kRoleG0, g0, s, &d_g0);
    if (rc == GXPO_OK) rc = stage_grads(ctx, kRoleG1, g1, s, &d_g1);
    if (rc != GXPO_OK) return rc;
    const ExtrapParams e = make_extrap_params(ctx->cfg);
    const int wc = (ctx->cfg.copy_mask & GXPO_COPY_AT_TILDE) ? 1 : 0;
    double *diag = ctx->cfg.diagnostics ? ctx->d_partial : nullptr;
    if (ctx->cfg.fuse_step2) {
        const StepParams p1 = make_step_params(ctx->cfg, ctx->pending_step1);
        const StepParams p2 = make_step_params(ctx->cfg, ctx->pending_step2);
        GXPO_HIP(ctx, launch_fused_steps_extrapolate(ctx->layout(), (int)ctx->cfg.optimizer, (int)ctx->cfg.grad_dtype, d_g0, d_g1,
                                                     p1, p2, e, ctx->cur_set(), ctx->next_set(), wc, diag, ctx->d_clip, s));
        ctx->advance_set();
    } else {
        GXPO_HIP(ctx, launch_extrapolate(ctx->layout(), (int)ctx->cfg.grad_dtype, d_g0, d_g1, e, wc, diag, ctx->d_clip, s));
    }
    if (diag)
        GXPO_HIP(ctx, launch_finalize(ctx->d_partial, ctx->n_blocks, ctx->d_seg, ctx->n_segs, ctx->d_tensor_seg_start, ctx->n,
                                      ctx->d_seg_sum, ctx->d_result, kAccG0Sq, kNumExtrapAcc, s));
    st.phase = GXPO_PHASE_REPOSITIONED;
    return GXPO_OK;
}

int gxpo_slow_step(gxpo_ctx *ctx, const void *const *g_slow, void *stream) {
    int rc = check_call(ctx, g_slow, "gxpo_slow_step");
    if (rc != GXPO_OK) return rc;
    gxpo_state &st = ctx->st;
    if (st.phase != GXPO_PHASE_REPOSITIONED) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_slow_step called in phase %u", st.phase);
    hipStream_t s = (hipStream_t)stream;
    GradArg d_g{};
    rc = stage_grads(ctx, kRoleSlow, g_slow, s, &d_g);
    if (rc != GXPO_OK) return rc;
    const int64_t step_no = st.optim_steps + 1;
    const StepParams p = make_step_params(ctx->cfg, step_no);
    const int wc = (ctx->cfg.copy_mask & GXPO_COPY_AT_FINAL) ? 1 : 0;
    // diagnostics: <g0, g_slow> needs g0 once more; its pointers are still staged from the extrapolation pass
    GradArg dot{};
    bool cos_valid = false;
    if (ctx->cfg.diagnostics) {
        cos_valid = true;
        for (uint32_t t = 0; t < ctx->n; ++t)
            if (g_slow[t] == ctx->shadow[kRoleG0][t]) cos_valid = false;      // g0 has been overwritten by g_slow
        if (cos_valid) dot = GradArg{ctx->d_grads + (size_t)kRoleG0 * ctx->n, ctx->shadow[kRoleG0][0]};
    }
    // with clipping the norm has to exist before the pass; otherwise it is accumulated inside it
    rc = clip_prepass(ctx, d_g, kAccSlowSq, kClipSlow, s);
    if (rc != GXPO_OK) return rc;
    double *partial = (ctx->d_clip && !cos_valid) ? nullptr : ctx->d_partial;
    GXPO_HIP(ctx, launch_step(ctx->layout(), (int)ctx->cfg.optimizer, (int)ctx->cfg.grad_dtype, d_g, p, ctx->cur_set(), ctx->next_set(), 1, wc,
                              partial, dot, ctx->d_clip, kClipSlow, s));
    ctx->advance_set();
    if (partial)
        GXPO_HIP(ctx, launch_finalize(ctx->d_partial, ctx->n_blocks, ctx->d_seg, ctx->n_segs, ctx->d_tensor_seg_start, ctx->n,
                                      ctx->d_seg_sum, ctx->d_result, kAccSlowSq, cos_valid ? 2 : 1, s));
    ctx->have_norms = true;
    ctx->have_diag = ctx->cfg.diagnostics != 0;
    ctx->cos_valid = cos_valid;
    ctx->diag_t = st.t;
    st.optim_steps = step_no;
    st.backward_passes += 1;
    st.phase = GXPO_PHASE_SLOW_DONE;
    return GXPO_OK;
}

static int fetch_result(gxpo_ctx *ctx, hipStream_t s, uint32_t n_acc = 1) {
    GXPO_HIP(ctx, hipMemcpyAsync(ctx->h_result, ctx->d_result, sizeof(double) * n_acc * ((size_t)ctx->n + 1), hipMemcpyDeviceToHost, s));
    GXPO_HIP(ctx, hipStreamSynchronize(s));
    return GXPO_OK;
}

int gxpo_gate(gxpo_ctx *ctx, gxpo_gate_info *out, void *stream) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    gxpo_state &st = ctx->st;
    if (st.phase != GXPO_PHASE_SLOW_DONE) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_gate called in phase %u", st.phase);
    int rc = fetch_result(ctx, (hipStream_t)stream);
    if (rc != GXPO_OK) return rc;
    const double norm = std::sqrt(ctx->h_result[0]);
    rc = gxpo_host_gate_step(&ctx->cfg, &st, norm, out);
    if (rc != GXPO_OK) return fail(ctx, rc, "gate state is corrupt");
    st.phase = GXPO_PHASE_IDLE;
    return GXPO_OK;
}

int gxpo_fallback_step(gxpo_ctx *ctx, const void *const *g0, void *stream) {
    int rc = check_call(ctx, g0, "gxpo_fallback_step");
    if (rc != GXPO_OK) return rc;
    gxpo_state &st = ctx->st;
    if (st.phase != GXPO_PHASE_IDLE) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_fallback_step called in phase %u", st.phase);
    if (!is_fallback_phase(st)) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_fallback_step: the gate has not tripped (t = %lld)", (long long)st.t);
    hipStream_t s = (hipStream_t)stream;
    GradArg d_g{};
    rc = stage_grads(ctx, kRoleG0, g0, s, &d_g);
    if (rc != GXPO_OK) return rc;
    const int64_t step_no = st.optim_steps + 1;
    const StepParams p = make_step_params(ctx->cfg, step_no);
    const int wc = (ctx->cfg.copy_mask & GXPO_COPY_AT_FINAL) ? 1 : 0;
    rc = clip_prepass(ctx, d_g, kAccClipG0, kClipG0, s);
    if (rc != GXPO_OK) return rc;
    GXPO_HIP(ctx, launch_step(ctx->layout(), (int)ctx->cfg.optimizer, (int)ctx->cfg.grad_dtype, d_g, p, ctx->cur_set(), ctx->next_set(), 1, wc,
                              nullptr, GradArg{}, ctx->d_clip, kClipG0, s));
    ctx->advance_set();
    st.optim_steps = step_no;
    st.backward_passes += 1;
    st.t += 1;
    return GXPO_OK;
}

int gxpo_tensor_norms(gxpo_ctx *ctx, double *out_host, void *stream) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!out_host) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_tensor_norms: out is NULL");
    if (!ctx->have_norms) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_tensor_norms: no slow step has run yet");
    int rc = fetch_result(ctx, (hipStream_t)stream);
    if (rc != GXPO_OK) return rc;
    for (uint32_t t = 0; t < ctx->n; ++t) out_host[t] = std::sqrt(ctx->h_result[1 + t]);
    return GXPO_OK;
}

int gxpo_get_diagnostics(gxpo_ctx *ctx, gxpo_diagnostics *out, void *stream) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!out) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_get_diagnostics: out is NULL");
    if (!ctx->cfg.diagnostics) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_get_diagnostics: the context was created without diagnostics");
    if (!ctx->have_diag) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_get_diagnostics: no active step has completed its slow step yet");
    int rc = fetch_result(ctx, (hipStream_t)stream, kNumAcc);
    if (rc != GXPO_OK) return rc;
    const size_t pitch = (size_t)ctx->n + 1;
    auto total = [&](int acc) { return ctx->h_result[(size_t)acc * pitch]; };
    const double nan = std::numeric_limits<double>::quiet_NaN();
    double n_total = 0.0;
    for (const gxpo_tensor &x : ctx->tensors) n_total += (double)x.numel;
    const double n_act = total(kAccActive);
    gxpo_diagnostics d{};
    d.norm_g0 = std::sqrt(total(kAccG0Sq));
    d.norm_g1 = std::sqrt(total(kAccG1Sq));
    d.norm_g_slow = std::sqrt(total(kAccSlowSq));
    d.cos_g0_g_slow = (ctx->cos_valid && d.norm_g0 > 0.0 && d.norm_g_slow > 0.0) ? total(kAccG0Slow) / (d.norm_g0 * d.norm_g_slow) : nan;
    if (n_act > 0.0) {
        const double mean_shifted = total(kAccR) / n_act;             // mean of r - 1
        const double var = total(kAccR2) / n_act - mean_shifted * mean_shifted;
        d.retention_mean = 1.0 + mean_shifted;
        d.retention_std = std::sqrt(var > 0.0 ? var : 0.0);
        d.scale_mean = total(kAccScale) / n_act;
    } else {
        d.retention_mean = d.retention_std = d.scale_mean = nan;
    }
    d.inactive_fraction = 1.0 - n_act / n_total;
    d.displacement_ratio = total(kAccD2) > 0.0 ? std::sqrt(total(kAccDK) / total(kAccD2)) : nan;
    d.t = ctx->diag_t;
    *out = d;
    return GXPO_OK;
}

int gxpo_current_params(const gxpo_ctx *ctx, float **out_host) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!out_host) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_current_params: out is NULL");
    for (uint32_t t = 0; t < ctx->n; ++t) out_host[t] = ctx->st.current_set ? ctx->tensors[t].theta_probe : ctx->tensors[t].theta;
    return GXPO_OK;
}

int gxpo_get_state(const gxpo_ctx *ctx, gxpo_state *out) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!out) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_get_state: out is NULL");
    *out = ctx->st;
    return GXPO_OK;
}

int gxpo_set_state(gxpo_ctx *ctx, const gxpo_state *in) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!in) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_state: state is NULL");
    if (in->struct_size != sizeof(gxpo_state)) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_state: struct_size mismatch");
    if (ctx->st.phase != GXPO_PHASE_IDLE) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_set_state: a training step is in progress");
    if (in->phase != GXPO_PHASE_IDLE) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_state: only an IDLE state can be restored");
    if (in->t < 0 || in->optim_steps < 0 || in->backward_passes < 0 || in->s_star < -1)
        return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_state: negative counter");
    if (in->window_len > ctx->cfg.window) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_state: window_len exceeds the configured window");
    if (in->current_set > (ctx->alternating ? 1u : 0u))
        return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_state: current_set %u, but the tensors %s", in->current_set,
                    ctx->alternating ? "have two buffer sets (0 or 1)" : "have no second buffer set (m_alt, v_alt)");
    ctx->st = *in;
    return GXPO_OK;
}

int gxpo_update_config(gxpo_ctx *ctx, const gxpo_config *cfg) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    std::string msg;
    int rc = check_config(cfg, msg);
    if (rc != GXPO_OK) return fail(ctx, rc, "gxpo_update_config: %s", msg.c_str());
    if (ctx->st.phase != GXPO_PHASE_IDLE) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_update_config: a training step is in progress");
    const gxpo_config &o = ctx->cfg;
    const bool same_shape = cfg->optimizer == o.optimizer && cfg->grad_dtype == o.grad_dtype && cfg->fuse_step2 == o.fuse_step2 &&
                            cfg->diagnostics == o.diagnostics &&
                            cfg->explicit_steps == o.explicit_steps && (cfg->clip_norm > 0.0) == (o.clip_norm > 0.0);
    if (!same_shape)
        return fail(ctx, GXPO_ERR_INVALID_ARG,
                    "gxpo_update_config: optimizer, grad_dtype, fuse_step2, diagnostics, explicit_steps and "
                    "clipping on/off are fixed at gxpo_init");
    gxpo_state &st = ctx->st;
    if (st.window_len > cfg->window) {       // keep the most recent norms
        const uint32_t drop = st.window_len - cfg->window;
        std::memmove(&st.window[0], &st.window[drop], sizeof(double) * cfg->window);
        st.window_len = cfg->window;
    }
    ctx->cfg = *cfg;
    return GXPO_OK;
}

int gxpo_set_tensor_options(gxpo_ctx *ctx, const gxpo_tensor_options *opts) {
    if (!ctx) return GXPO_ERR_INVALID_ARG;
    if (!opts) return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_tensor_options: options are NULL");
    if (ctx->st.phase != GXPO_PHASE_IDLE) return fail(ctx, GXPO_ERR_BAD_STATE, "gxpo_set_tensor_options: a training step is in progress");
    for (uint32_t t = 0; t < ctx->n; ++t) {
        const double a = opts[t].lr_scale, b = opts[t].weight_decay_scale;
        if (!(a >= 0.0) || !std::isfinite(a) || !(b >= 0.0) || !std::isfinite(b))
            return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_tensor_options: tensor %u: multipliers must be finite and >= 0", t);
    }
    int dev = -1;
    GXPO_HIP(ctx, hipGetDevice(&dev));
    if (dev != ctx->device)
        return fail(ctx, GXPO_ERR_INVALID_ARG, "gxpo_set_tensor_options: current device %d is not the context's device %d", dev, ctx->device);
    const std::vector<gxpo_tensor_options> before = ctx->options;
    ctx->options.assign(opts, opts + ctx->n);
    std::vector<TensorRec> tab(ctx->n);
    for (uint32_t t = 0; t < ctx->n; ++t) tab[t] = ctx->record(t);
    // kernels of earlier calls may still be reading the table
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(ctx->d_tab, tab.data(), sizeof(TensorRec) * ctx->n, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        ctx->options = before;
        return fail_hip(ctx, e, "gxpo_set_tensor_options: table upload");
    }
    return GXPO_OK;
}

int gxpo_slow_step_noalloc(const gxpo_config *cfg, const gxpo_tensor *tensor, int64_t optim_step, const void *g_slow,
                           double *sum_sq_out_device, void *stream) {
    std::string msg;
    int rc = check_config(cfg, msg);
    if (rc != GXPO_OK) return fail(nullptr, rc, "gxpo_slow_step_noalloc: %s", msg.c_str());
    if (cfg->clip_norm > 0.0 || cfg->diagnostics)
        return fail(nullptr, GXPO_ERR_UNSUPPORTED, "gxpo_slow_step_noalloc: clipping and diagnostics need the workspace of a context");
    if (!tensor || !g_slow || !sum_sq_out_device) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: NULL argument");
    if (optim_step < 1) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: optim_step must be >= 1");
    const gxpo_tensor &x = *tensor;
    const bool adam = cfg->optimizer == GXPO_OPT_ADAMW;
    if (x.numel == 0) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: numel is 0");
    if (x.numel > GXPO_NOALLOC_MAX_NUMEL)
        return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: numel %llu exceeds the built-in workspace (at most %llu elements); use a context",
                    (unsigned long long)x.numel, (unsigned long long)GXPO_NOALLOC_MAX_NUMEL);
    if (!x.theta) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: theta is NULL");
    if (adam && (!x.m || !x.v)) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: AdamW needs m and v");
    if (!adam && (x.m || x.v)) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: m and v must be NULL for plain GD");
    const bool wc = (cfg->copy_mask & GXPO_COPY_AT_FINAL) && x.model_copy;
    const uint64_t gbytes = cfg->grad_dtype == GXPO_GRAD_F32 ? 4u : 2u;
    // every buffer the kernels touch: alignment, device range, and no overlap between any two
    struct Buf { const void *p; uint64_t bytes; uintptr_t align; const char *what; };
    const Buf bufs[6] = {{x.theta, x.numel * 4, 16, "theta"},
                         {x.m, x.numel * 4, 16, "m"},
                         {x.v, x.numel * 4, 16, "v"},
                         {wc ? x.model_copy : nullptr, x.numel * 2, 8, "model_copy"},
                         {g_slow, x.numel * gbytes, cfg->grad_dtype == GXPO_GRAD_F32 ? (uintptr_t)16 : (uintptr_t)8, "g_slow"},
                         {sum_sq_out_device, 8, 8, "sum_sq_out"}};
    for (const Buf &b : bufs)
        if (b.p && (uintptr_t)b.p % b.align)
            return fail(nullptr, GXPO_ERR_ALIGNMENT, "gxpo_slow_step_noalloc: %s is not %u-byte aligned", b.what, (unsigned)b.align);
    for (int i = 0; i < 6; ++i)
        for (int j = i + 1; j < 6; ++j) {
            if (!bufs[i].p || !bufs[j].p) continue;
            const uintptr_t a = (uintptr_t)bufs[i].p, b = (uintptr_t)bufs[j].p;
            if (a < b + bufs[j].bytes && b < a + bufs[i].bytes)
                return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_slow_step_noalloc: %s overlaps %s", bufs[i].what, bufs[j].what);
        }
    for (const Buf &b : bufs) {
        if (!b.p) continue;
        rc = check_device_range(nullptr, b.p, b.bytes, b.what, 0);
        if (rc != GXPO_OK) return rc;
    }
    Layout L{};
    L.n_tensors = 1;
    L.n_blocks = (uint32_t)((x.numel + kWaveElems - 1) / kWaveElems);
    L.single = TensorRec{x.theta, nullptr, x.m, x.v, wc ? x.model_copy : nullptr, nullptr, nullptr, x.numel, 1.0f, 1.0f};
    const StepParams p = make_step_params(*cfg, optim_step);
    hipError_t e = launch_slow_step_noalloc(L, (int)cfg->optimizer, (int)cfg->grad_dtype, GradArg{nullptr, g_slow}, p, wc ? 1 : 0,
                                            sum_sq_out_device, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(nullptr, e, "gxpo_slow_step_noalloc");
    return GXPO_OK;
}

int gxpo_stream_copy(void *dst_device, const void *src_device, uint64_t bytes, void *stream) {
    if (!dst_device || !src_device) return fail(nullptr, GXPO_ERR_INVALID_ARG, "gxpo_stream_copy: NULL pointer");
    if (bytes % 16 || (uintptr_t)dst_device % 16 || (uintptr_t)src_device % 16)
        return fail(nullptr, GXPO_ERR_ALIGNMENT, "gxpo_stream_copy: pointers and size must be multiples of 16");
    int rc = check_device_range(nullptr, src_device, bytes, "copy source", 0);
    if (rc == GXPO_OK) rc = check_device_range(nullptr, dst_device, bytes, "copy destination", 0);
    if (rc != GXPO_OK) return rc;
    hipError_t e = launch_stream_copy(dst_device, src_device, bytes, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(nullptr, e, "gxpo_stream_copy launch");
    return GXPO_OK;
}

}  // extern "C"
