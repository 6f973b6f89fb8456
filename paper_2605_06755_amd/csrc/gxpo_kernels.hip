// gfx950 kernels of the GXPO update engine.
//
// Every pass is a pure HBM stream: no element needs a neighbour, nothing is
// reused, so the kernels are built around how MI355X moves bytes best:
//
//  * one-shot blocks of one wavefront: each lane owns 4 consecutive elements
//    (one 128-bit access per fp32 stream, one 64-bit access per bf16 stream)
//    and the block retires after a single load -> compute -> store round.
//    Blocks are dispatched in index order, so the set of DRAM pages in flight
//    stays a narrow moving front.  Measured on this part with the stand-alone
//    probe (csrc/hbm_probe.hip): 81.6 % of peak against 68-73 % for blocks of
//    2 or 4 wavefronts, 68 % for lanes that own 8 elements (two 128-bit
//    accesses per fp32 stream, one per bf16 stream) and 57-70 % for
//    grid-stride loops; 128-bit accesses for bf16 streams by half of the
//    lanes plus a cross-lane hand-over are slower than the 64-bit ones too.
//  * buffer instructions with the streaming cache policy (sc1 + nt): the data
//    is touched once per pass, there is nothing for L2 / MALL to keep (81 %
//    of peak against 74 % with the default policy, 75 % for non-temporal
//    global accesses).  The
//    buffer descriptor of each stream covers exactly the block's span, so the
//    hardware range check makes the ragged last block of a tensor safe:
//    out-of-range lanes load 0 and their stores are dropped.
//  * the block -> (tensor, offset) map is two or three scalar loads (coarse
//    index + short scan); a single flat tensor skips it and takes every
//    pointer straight from the kernel arguments.
//
// Arithmetic is fp32 with the optimizer constants prepared in double on the
// host; only the sum of squares of g_slow is accumulated in fp64.
#include "gxpo_internal.h"

namespace gxpo {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// cache-policy bits of gfx94x/gfx950 buffer instructions: sc0 = 1, nt = 2, sc1 = 16
constexpr int kStreamPolicy = 16 | 2;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t span_rsrc(const void *base, uint32_t bytes) {
    // raw (unstructured) buffer: stride 0, 32-bit data format; range-checked against `bytes`
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// ---- 4-element lane loads / stores -------------------------------------------------------
// `full` is block-uniform: true when the block's span holds all of its elements, so
// every lane may use one wide access.  Otherwise each element goes through its own
// range-checked access.

__device__ __forceinline__ f32x4 load_f32(__amdgpu_buffer_rsrc_t r, uint32_t elem, bool full) {
    if (full) {
        u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(elem * 4u), 0, kStreamPolicy);
        return __builtin_bit_cast(f32x4, x);
    }
    f32x4 o;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        unsigned x = __builtin_amdgcn_raw_buffer_load_b32(r, (int)((elem + k) * 4u), 0, kStreamPolicy);
        o[k] = __builtin_bit_cast(float, x);
    }
    return o;
}

__device__ __forceinline__ void store_f32(__amdgpu_buffer_rsrc_t r, uint32_t elem, bool full, f32x4 v) {
    if (full) {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)(elem * 4u), 0, kStreamPolicy);
        return;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float lane_value = v[k];   // a scalar copy: bit-casting the vector element in place reads element 0
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, lane_value), r, (int)((elem + k) * 4u), 0, kStreamPolicy);
    }
}

__device__ __forceinline__ f32x4 load_bf16(__amdgpu_buffer_rsrc_t r, uint32_t elem, bool full) {
    f32x4 o;
    if (full) {
        u32x2 x = __builtin_amdgcn_raw_buffer_load_b64(r, (int)(elem * 2u), 0, kStreamPolicy);
        o[0] = __builtin_bit_cast(float, x[0] << 16);
        o[1] = __builtin_bit_cast(float, x[0] & 0xffff0000u);
        o[2] = __builtin_bit_cast(float, x[1] << 16);
        o[3] = __builtin_bit_cast(float, x[1] & 0xffff0000u);
        return o;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        unsigned x = __builtin_amdgcn_raw_buffer_load_b16(r, (int)((elem + k) * 2u), 0, kStreamPolicy);
        o[k] = __builtin_bit_cast(float, x << 16);
    }
    return o;
}

__device__ __forceinline__ unsigned bf16_bits(float f) {
    // conversion in the compiler's native bf16 type: round to nearest even
    __bf16 h = (__bf16)f;
    return (unsigned)__builtin_bit_cast(unsigned short, h);
}

__device__ __forceinline__ void store_bf16(__amdgpu_buffer_rsrc_t r, uint32_t elem, bool full, f32x4 v) {
    if (full) {
        u32x2 x;
        x[0] = bf16_bits(v[0]) | (bf16_bits(v[1]) << 16);
        x[1] = bf16_bits(v[2]) | (bf16_bits(v[3]) << 16);
        __builtin_amdgcn_raw_buffer_store_b64(x, r, (int)(elem * 2u), 0, kStreamPolicy);
        return;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)bf16_bits(v[k]), r, (int)((elem + k) * 2u), 0, kStreamPolicy);
}

template <int GDT> __device__ __forceinline__ __amdgpu_buffer_rsrc_t grad_rsrc(const void *g, uint64_t e0, uint32_t cnt) {
    if (GDT == 0) return span_rsrc((const float *)g + e0, cnt * 4u);
    return span_rsrc((const unsigned short *)g + e0, cnt * 2u);
}
__device__ __forceinline__ const void *grad_ptr(const GradArg &g, const Layout &L, uint32_t tensor) {
    return L.n_tensors > 1 ? g.table[tensor] : g.single;
}
template <int GDT> __device__ __forceinline__ f32x4 load_grad(__amdgpu_buffer_rsrc_t r, uint32_t elem, bool full) {
    if (GDT == 0) return load_f32(r, elem, full);
    return load_bf16(r, elem, full);
}

// ---- which part of which tensor this block owns ---------------------------------------
struct Span {
    TensorRec rec;
    uint32_t tensor;
    uint64_t e0;       // first element of the block inside the tensor
    uint32_t cnt;      // elements of the tensor inside the block's span (<= elems per block)
    bool full;
};

__device__ __forceinline__ Span locate(const Layout &L, uint32_t b) {
    constexpr uint32_t kBlockElems = kWaveElems;
    uint32_t t = 0;
    if (L.n_tensors > 1) {
        t = L.coarse[b >> kCoarseShift];
        while (L.blk_start[t + 1] <= b) ++t;      // blk_start[n_tensors] == n_blocks > b
    }
    Span s;
    s.tensor = t;
    uint32_t first_block = 0;
    if (L.n_tensors > 1) {
        s.rec = L.tab[t];
        first_block = L.blk_start[t];
    } else {
        s.rec = L.single;                          // straight from the kernel arguments
    }
    s.e0 = (uint64_t)(b - first_block) * kBlockElems;
    const uint64_t rem = s.rec.numel - s.e0;
    s.cnt = rem < kBlockElems ? (uint32_t)rem : kBlockElems;
    s.full = s.cnt == kBlockElems;
    return s;
}

// ---- OptimStep on one element (Algorithm 1's OptimStep) ---------------------------------
// Returns the amount to subtract from theta; updates the moments in place.
//   GD    : eta * g
//   AdamW : lr*wd*theta + lr/(1-beta1^s) * m / (sqrt(v)/sqrt(1-beta2^s) + eps)
// Keeping the update separate from theta lets callers form theta - update with one
// rounding, and lets the fused pass subtract it from a displacement instead.
template <int OPT>
__device__ __forceinline__ float optim_update(float theta, float &m, float &v, float g, const StepParams &p) {
    if (OPT == 0) return p.lr * g;
    m = fmaf(p.beta1, m, p.one_minus_beta1 * g);
    v = fmaf(p.beta2, v, p.one_minus_beta2 * g * g);
    const float denom = fmaf(sqrtf(v), p.rsqrt_bias2, p.eps);
    return fmaf(p.lr_wd, theta, p.step_size * (m / denom));
}

// The step constants of one tensor: its parameter group scales the learning rate and the
// decoupled decay.  Multipliers of exactly 1 leave every constant bit-identical.
__device__ __forceinline__ StepParams for_tensor(StepParams p, const TensorRec &rec) {
    p.lr *= rec.lr_scale;
    p.step_size *= rec.lr_scale;
    p.lr_wd *= rec.lr_wd_scale;
    return p;
}

// ---- extrapolation factor (Eqs. (4), (7); Algorithm 1 "Extrapolation factor") -------------
// scale = S_K(r)/S_2(r) with r = g1/g0, written so that nothing cancels:
//   K even: S_K/S_2 = sum_{j<K/2} r^{2j}
//   K odd : S_K/S_2 = sum_{j<(K-1)/2} r^{2j} + r^{K-1}/(1+r),   1 + r = (g0+g1)/g0
// g0 + g1 is rounded once from exact inputs, so the pole at r = -1 is approached
// with full relative accuracy.  Off the active set, and at r == -1 where S_2
// vanishes, the observed displacement is kept (scale = 1).
struct ScaleInfo {
    float scale;     // the factor applied to the observed displacement
    float r;         // retention ratio after the clamp (meaningful only when active)
    bool active;     // |g0| > delta
};

// g0, g1 are the gradients as loaded, c0, c1 their clipping factors (1 when clipping is off
// or inactive).  The fast steps consumed g0*c0 and g1*c1; the ratio is formed from those.
__device__ __forceinline__ ScaleInfo extrap_scale_info(float g0, float c0, float g1, float c1, const ExtrapParams &e) {
    const float g0c = g0 * c0, g1c = g1 * c1;
    const float r = g1c / g0c;
    const float rc = fminf(fmaxf(r, -e.r_max), e.r_max);
    const float x = rc * rc;
    float series = 1.0f, power = 1.0f;
    for (uint32_t j = 1; j < e.half; ++j) {
        series = fmaf(series, x, 1.0f);
        power *= x;
    }
    float scale = series;
    if (e.odd) {
        power *= x;                                   // r^(K-1)
        const bool clamped = rc != r;
        // g0*c0 + g1*c1 with one rounding: exact product inside the fma plus the exact
        // rounding error of the other product (both vanish when the factors are 1)
        const float sum = fmaf(g0, c0, g1c) + fmaf(g1, c1, -g1c);
        const float num = clamped ? 1.0f : g0c;
        const float den = clamped ? 1.0f + rc : sum;
        scale = fmaf(power, num / den, series);
    }
    const bool active = fabsf(g0c) > e.delta;
    const bool use = active && (rc != -1.0f);
    return ScaleInfo{use ? scale : 1.0f, rc, active};
}

// Sum over the 64 lanes of a wavefront with DPP moves (no LDS traffic, no bpermute): inside
// each row of 16 lanes two quad permutes and two row rotations leave the row total in every
// lane; row_bcast:15 then adds row k-1's total into rows 1 and 3, row_bcast:31 adds lane 31's
// value into rows 2 and 3, so lane 63 holds the total, which is broadcast.  The order of the
// additions is fixed by the lane numbers.  All 64 lanes must be active.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ double dpp_fetch(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xf, false);     // lanes outside ROW_MASK receive 0
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xf, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum(double x) {
    x += dpp_fetch<0xb1, 0xf>(x);      // quad_perm:[1,0,3,2]
    x += dpp_fetch<0x4e, 0xf>(x);      // quad_perm:[2,3,0,1]
    x += dpp_fetch<0x124, 0xf>(x);     // row_ror:4
    x += dpp_fetch<0x128, 0xf>(x);     // row_ror:8
    x += dpp_fetch<0x142, 0xa>(x);     // row_bcast:15 into rows 1 and 3
    x += dpp_fetch<0x143, 0xc>(x);     // row_bcast:31 into rows 2 and 3
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), 63);
    return __hiloint2double(hi, lo);
}

// Adds the N per-lane values over the block (one wavefront) and stores them as this block's
// partials of accumulators first_acc .. first_acc + N - 1 (fixed order: the lane butterfly).
template <int N>
__device__ __forceinline__ void store_block_sums(double (&acc)[N], double *__restrict__ partial, int first_acc, uint32_t n_blocks,
                                                 uint32_t block) {
    const size_t pitch = partial_pitch(n_blocks);
    const uint32_t slot = partial_slot(block, partial_stride(n_blocks));
#pragma unroll
    for (int a = 0; a < N; ++a) acc[a] = wave_sum(acc[a]);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int a = 0; a < N; ++a) partial[(size_t)(first_acc + a) * pitch + slot] = acc[a];
    }
}

// Per-lane accumulators of the extrapolation-pass diagnostics.  The two gradient norms must
// match an fp64 reference to ~1e-12 and stay in fp64.  The other statistics are means and
// ratios of fp32 quantities (r, scale and the displacements are formed in fp32 to begin
// with): they are summed in fp32 inside a block (256 terms, pairwise over the lanes)
// and in fp64 from the block partial on; the active count is an integer.  That keeps the
// diagnostics from turning the pass ALU-bound (fp64 adds and 64-bit lane exchanges are the
// expensive part of a block's reduction).
struct ExtrapDiag {
    double g0_sq = 0.0, g1_sq = 0.0;
    float rm1_sum = 0.0f, rm1_sq = 0.0f, scale_sum = 0.0f, d2_sq = 0.0f, dK_sq = 0.0f;
    uint32_t active = 0;
};

// `in_range`: the coordinate exists (lanes past the ragged end of a tensor loaded zeros; their
// gradients add nothing, but a zero-state AdamW step with eps = 0 is 0/0, which must not reach the sums).
__device__ __forceinline__ void add_extrap_diag(ExtrapDiag &d, float g0, float g1, const ScaleInfo &si, float disp2, bool in_range) {
    d.g0_sq = fma((double)g0, (double)g0, d.g0_sq);
    d.g1_sq = fma((double)g1, (double)g1, d.g1_sq);
    const float rm1 = si.r - 1.0f;          // centred on the common case r ~ 1: no cancellation in the variance
    d.active += si.active ? 1u : 0u;
    d.rm1_sum += si.active ? rm1 : 0.0f;
    d.rm1_sq = si.active ? fmaf(rm1, rm1, d.rm1_sq) : d.rm1_sq;
    d.scale_sum += si.active ? si.scale : 0.0f;
    const float d2 = in_range ? disp2 : 0.0f;
    const float dK = in_range ? si.scale * disp2 : 0.0f;
    d.d2_sq = fmaf(d2, d2, d.d2_sq);
    d.dK_sq = fmaf(dK, dK, d.dK_sq);
}

// 32-bit versions of the wave reduction above (same lane pattern, same fixed order).
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_fetch(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_fetch<0xb1, 0xf>(x);
    x += dpp_fetch<0x4e, 0xf>(x);
    x += dpp_fetch<0x124, 0xf>(x);
    x += dpp_fetch<0x128, 0xf>(x);
    x += dpp_fetch<0x142, 0xa>(x);
    x += dpp_fetch<0x143, 0xc>(x);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xb1, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4e, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x124, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// Block totals of the eight extrapolation-pass accumulators -> this block's partials of
// accumulators kAccG0Sq .. kAccDK (fixed order: the lane butterfly).
__device__ __forceinline__ void store_extrap_diag(const ExtrapDiag &d, double *__restrict__ partial, uint32_t n_blocks, uint32_t block) {
    double acc[kNumExtrapAcc];
    acc[kAccG0Sq - kAccG0Sq] = wave_sum(d.g0_sq);
    acc[kAccG1Sq - kAccG0Sq] = wave_sum(d.g1_sq);
    acc[kAccActive - kAccG0Sq] = (double)wave_sum(d.active);
    acc[kAccR - kAccG0Sq] = (double)wave_sum(d.rm1_sum);
    acc[kAccR2 - kAccG0Sq] = (double)wave_sum(d.rm1_sq);
    acc[kAccScale - kAccG0Sq] = (double)wave_sum(d.scale_sum);
    acc[kAccD2 - kAccG0Sq] = (double)wave_sum(d.d2_sq);
    acc[kAccDK - kAccG0Sq] = (double)wave_sum(d.dK_sq);
    const size_t pitch = partial_pitch(n_blocks);
    const uint32_t slot = partial_slot(block, partial_stride(n_blocks));
    if (threadIdx.x == 0) {
#pragma unroll
        for (int a = 0; a < kNumExtrapAcc; ++a) partial[(size_t)(kAccG0Sq + a) * pitch + slot] = acc[a];
    }
}

// ============================================================================
// OptimStep pass: fast step 1 (theta -> probe), unfused fast step 2
// (probe -> probe), slow step (theta -> theta, + sum of squares), fallback step
// (theta -> theta).  28 B/param with fp32 gradients (16 read, 12 written).
//
// As the probe of the fused schedule (write_moments == 0) it only previews the
// step: theta^{t,1} is written for the trainer, the advanced moments are
// dropped because the fused pass recomputes them from the same inputs
// (20 B/param: 16 read, 4 written; 18 when only the bf16 copy is written).
// ============================================================================
template <int OPT, int GDT>
__global__ __launch_bounds__(64) void k_optim_step(Layout L, GradArg grads, StepParams p_all, int src, int dst,
                                                       int write_moments, int write_copy, double *__restrict__ partial,
                                                       GradArg dot_with, const float *__restrict__ clip, int clip_index) {
    const Span s = locate(L, blockIdx.x);
    const StepParams p = for_tensor(p_all, s.rec);
    const uint32_t elem = threadIdx.x * kLaneElems;
    const uint32_t bytes = s.cnt * 4u;
    const float *src_ptr = ((src & kSrcProbe) ? s.rec.probe : s.rec.theta) + s.e0;
    float *dst_base = (dst & kSrcProbe) ? s.rec.probe : s.rec.theta;     // a NULL probe: nobody wants fp32 theta^{t,1}
    const auto r_src = span_rsrc(src_ptr, bytes);
    const auto r_g = grad_rsrc<GDT>(grad_ptr(grads, L, s.tensor), s.e0, s.cnt);

    f32x4 th = load_f32(r_src, elem, s.full);
    f32x4 g = load_grad<GDT>(r_g, elem, s.full);
    f32x4 m = {0, 0, 0, 0}, v = {0, 0, 0, 0};
    if (OPT == 1) {
        const bool alt = (src & kMomentsAlt) != 0;
        m = load_f32(span_rsrc((alt ? s.rec.m_alt : s.rec.m) + s.e0, bytes), elem, s.full);
        v = load_f32(span_rsrc((alt ? s.rec.v_alt : s.rec.v) + s.e0, bytes), elem, s.full);
    }
    const float coef = clip ? clip[clip_index] : 1.0f;          // global-norm clipping factor of this gradient
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float mk = m[k], vk = v[k];
        th[k] = th[k] - optim_update<OPT>(th[k], mk, vk, g[k] * coef, p);
        m[k] = mk;
        v[k] = vk;
    }
    if (dst_base) store_f32(span_rsrc(dst_base + s.e0, bytes), elem, s.full, th);
    if (OPT == 1 && write_moments) {
        const bool alt = (dst & kMomentsAlt) != 0;
        store_f32(span_rsrc((alt ? s.rec.m_alt : s.rec.m) + s.e0, bytes), elem, s.full, m);
        store_f32(span_rsrc((alt ? s.rec.v_alt : s.rec.v) + s.e0, bytes), elem, s.full, v);
    }
    if (write_copy && s.rec.copy) {
        const auto r_c = span_rsrc((unsigned short *)s.rec.copy + s.e0, s.cnt * 2u);
        store_bf16(r_c, elem, s.full, th);
    }
    if (partial) {
        // out-of-range lanes loaded g = 0 and add nothing
        double acc[2] = {0.0, 0.0};
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[0] = fma((double)g[k], (double)g[k], acc[0]);
        const void *other = dot_with.single;
        if (L.n_tensors > 1) other = dot_with.table ? dot_with.table[s.tensor] : nullptr;
        if (other) {        // diagnostics: <g0, g_slow>, g0 re-read (+4 B/param)
            const f32x4 o = load_grad<GDT>(grad_rsrc<GDT>(other, s.e0, s.cnt), elem, s.full);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[1] = fma((double)o[k], (double)g[k], acc[1]);
            store_block_sums<2>(acc, partial, kAccSlowSq, L.n_blocks, blockIdx.x);
        } else {
            double only[1] = {acc[0]};
            store_block_sums<1>(only, partial, kAccSlowSq, L.n_blocks, blockIdx.x);
        }
    }
}

// ============================================================================
// Extrapolate + reposition alone (Algorithm 1 "Active coordinates" ... "Reposition"):
//   theta <- theta + alpha * scale * (theta_probe - theta)
// 20 B/param with fp32 gradients (16 read, 4 written).
// ============================================================================
template <int GDT, bool DIAG>
__global__ __launch_bounds__(64) void k_extrapolate(Layout L, GradArg g0s, GradArg g1s, ExtrapParams e,
                                                        int write_copy, double *__restrict__ diag_partial,
                                                        const float *__restrict__ clip) {
    const Span s = locate(L, blockIdx.x);
    const uint32_t elem = threadIdx.x * kLaneElems;
    const uint32_t bytes = s.cnt * 4u;
    const auto r_th = span_rsrc(s.rec.theta + s.e0, bytes);
    const auto r_pr = span_rsrc(s.rec.probe + s.e0, bytes);
    const auto r_g0 = grad_rsrc<GDT>(grad_ptr(g0s, L, s.tensor), s.e0, s.cnt);
    const auto r_g1 = grad_rsrc<GDT>(grad_ptr(g1s, L, s.tensor), s.e0, s.cnt);
    f32x4 th0 = load_f32(r_th, elem, s.full);
    f32x4 th2 = load_f32(r_pr, elem, s.full);
    f32x4 g0 = load_grad<GDT>(r_g0, elem, s.full);
    f32x4 g1 = load_grad<GDT>(r_g1, elem, s.full);
    const float c0 = clip ? clip[kClipG0] : 1.0f, c1 = clip ? clip[kClipG1] : 1.0f;
    ExtrapDiag diag;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const ScaleInfo si = extrap_scale_info(g0[k], c0, g1[k], c1, e);
        const float disp2 = th2[k] - th0[k];
        if (DIAG) add_extrap_diag(diag, g0[k], g1[k], si, disp2, elem + k < s.cnt);
        th0[k] = fmaf(e.alpha * si.scale, disp2, th0[k]);
    }
    store_f32(r_th, elem, s.full, th0);
    if (write_copy && s.rec.copy) {
        const auto r_c = span_rsrc((unsigned short *)s.rec.copy + s.e0, s.cnt * 2u);
        store_bf16(r_c, elem, s.full, th0);
    }
    if (DIAG) store_extrap_diag(diag, diag_partial, L.n_blocks, blockIdx.x);
}

// ============================================================================
// Reposition alone (explicit lookahead): theta <- theta + alpha (theta_probe - theta).
// 12 B/param (8 read, 4 written).
// ============================================================================
__global__ __launch_bounds__(64) void k_reposition(Layout L, float alpha, int write_copy) {
    const Span s = locate(L, blockIdx.x);
    const uint32_t elem = threadIdx.x * kLaneElems;
    const uint32_t bytes = s.cnt * 4u;
    const auto r_th = span_rsrc(s.rec.theta + s.e0, bytes);
    const auto r_pr = span_rsrc(s.rec.probe + s.e0, bytes);
    f32x4 th0 = load_f32(r_th, elem, s.full);
    const f32x4 thn = load_f32(r_pr, elem, s.full);
#pragma unroll
    for (int k = 0; k < 4; ++k) th0[k] = fmaf(alpha, thn[k] - th0[k], th0[k]);
    store_f32(r_th, elem, s.full, th0);
    if (write_copy && s.rec.copy) {
        const auto r_c = span_rsrc((unsigned short *)s.rec.copy + s.e0, s.cnt * 2u);
        store_bf16(r_c, elem, s.full, th0);
    }
}

// ============================================================================
// Fused: both fast steps' state update + extrapolate + reposition.
//
// The first fast step was only previewed by the probe pass (theta^{t,1} went
// to the trainer, nothing else was stored).  This pass replays it from the
// same inputs (theta^t, m, v, g0 and the step-1 constants give bit-identical
// theta^{t,1}, m, v, because the same fp32 operations run in the same order),
// takes the second fast step on top, and extrapolates.  theta^{t,1},
// theta^{t,2}, r and scale live only in registers; the two-step displacement
// is formed as (theta^{t,1} - theta^t) - update_2, i.e. from the exact
// difference of two fp32 iterates, not from a rounded theta^{t,2}.
// Recomputing costs ALU time the pass does not have to wait for; it saves the
// write and re-read of m, v (16 B) and the re-read of theta^{t,1} (4 B):
// 32 B/param with fp32 gradients (20 read, 12 written).
// ============================================================================
template <int OPT, int GDT, bool DIAG>
__global__ __launch_bounds__(64) void k_fused_steps_extrapolate(Layout L, GradArg g0s, GradArg g1s, StepParams p1_all,
                                                                    StepParams p2_all, ExtrapParams e, int src, int dst,
                                                                    int write_copy, double *__restrict__ diag_partial,
                                                                    const float *__restrict__ clip) {
    const Span s = locate(L, blockIdx.x);
    const StepParams p1 = for_tensor(p1_all, s.rec), p2 = for_tensor(p2_all, s.rec);
    const uint32_t elem = threadIdx.x * kLaneElems;
    const uint32_t bytes = s.cnt * 4u;
    const auto r_th = span_rsrc(((src & kSrcProbe) ? s.rec.probe : s.rec.theta) + s.e0, bytes);
    const auto r_g0 = grad_rsrc<GDT>(grad_ptr(g0s, L, s.tensor), s.e0, s.cnt);
    const auto r_g1 = grad_rsrc<GDT>(grad_ptr(g1s, L, s.tensor), s.e0, s.cnt);
    f32x4 th0 = load_f32(r_th, elem, s.full);
    f32x4 g0 = load_grad<GDT>(r_g0, elem, s.full);
    f32x4 m = {0, 0, 0, 0}, v = {0, 0, 0, 0};
    if (OPT == 1) {
        const bool alt = (src & kMomentsAlt) != 0;
        m = load_f32(span_rsrc((alt ? s.rec.m_alt : s.rec.m) + s.e0, bytes), elem, s.full);
        v = load_f32(span_rsrc((alt ? s.rec.v_alt : s.rec.v) + s.e0, bytes), elem, s.full);
    }
    f32x4 g1 = load_grad<GDT>(r_g1, elem, s.full);
    const float c0 = clip ? clip[kClipG0] : 1.0f, c1 = clip ? clip[kClipG1] : 1.0f;
    ExtrapDiag diag;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float mk = m[k], vk = v[k];
        const float g0c = g0[k] * c0, g1c = g1[k] * c1;           // what the fast steps consume (clipped)
        const float th1 = th0[k] - optim_update<OPT>(th0[k], mk, vk, g0c, p1);    // theta^{t,1}, as the probe pass stored it
        const float upd2 = optim_update<OPT>(th1, mk, vk, g1c, p2);
        m[k] = mk;
        v[k] = vk;
        const float disp2 = (th1 - th0[k]) - upd2;                // theta^{t,2} - theta^t
        const ScaleInfo si = extrap_scale_info(g0[k], c0, g1[k], c1, e);
        if (DIAG) add_extrap_diag(diag, g0[k], g1[k], si, disp2, elem + k < s.cnt);
        th0[k] = fmaf(e.alpha * si.scale, disp2, th0[k]);
    }
    store_f32(span_rsrc(((dst & kSrcProbe) ? s.rec.probe : s.rec.theta) + s.e0, bytes), elem, s.full, th0);
    if (OPT == 1) {
        const bool alt = (dst & kMomentsAlt) != 0;
        store_f32(span_rsrc((alt ? s.rec.m_alt : s.rec.m) + s.e0, bytes), elem, s.full, m);
        store_f32(span_rsrc((alt ? s.rec.v_alt : s.rec.v) + s.e0, bytes), elem, s.full, v);
    }
    if (write_copy && s.rec.copy) {
        const auto r_c = span_rsrc((unsigned short *)s.rec.copy + s.e0, s.cnt * 2u);
        store_bf16(r_c, elem, s.full, th0);
    }
    if (DIAG) store_extrap_diag(diag, diag_partial, L.n_blocks, blockIdx.x);
}

// ============================================================================
// Norm pre-pass for gradient clipping: sum of squares of one gradient list
// (read-only, 4 or 2 B/param), same block plan and reduction as the slow step.
// ============================================================================
// A launched block covers kSumsqGroup consecutive blocks of the plan (a single 1 KiB read per
// launched block would be bound by the block dispatch rate, not by HBM); it still writes one
// partial per plan block, so the reduction that follows is the same.
constexpr uint32_t kSumsqGroup = 4;

template <int GDT>
__global__ __launch_bounds__(64) void k_sumsq(Layout L, GradArg grads, double *__restrict__ partial, int acc_index) {
    const uint32_t elem = threadIdx.x * kLaneElems;
    const uint32_t first = blockIdx.x * kSumsqGroup;
    f32x4 g[kSumsqGroup];
#pragma unroll
    for (uint32_t i = 0; i < kSumsqGroup; ++i) {
        g[i] = f32x4{0, 0, 0, 0};
        if (first + i < L.n_blocks) {
            const Span s = locate(L, first + i);
            g[i] = load_grad<GDT>(grad_rsrc<GDT>(grad_ptr(grads, L, s.tensor), s.e0, s.cnt), elem, s.full);
        }
    }
#pragma unroll
    for (uint32_t i = 0; i < kSumsqGroup; ++i) {
        if (first + i < L.n_blocks) {
            double acc[1] = {0.0};
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[0] = fma((double)g[i][k], (double)g[i][k], acc[0]);
            store_block_sums<1>(acc, partial, acc_index, L.n_blocks, first + i);
        }
    }
}

__global__ void k_clip_coefficient(const double *__restrict__ result_all, uint32_t n_tensors, int acc, double max_norm,
                                   float *__restrict__ clip, int clip_index) {
    const double norm = sqrt(result_all[(size_t)acc * (1 + n_tensors)]);
    const double c = max_norm / (norm + 1e-6);
    clip[clip_index] = (float)(c < 1.0 ? c : 1.0);          // a NaN norm gives c = NaN -> 1: the step then propagates the NaN
}

// ============================================================================
// Fixed-order reduction of the per-block partial sums.
// Stage 1: one block per run of <= kSegPartials partials of one tensor.
// Stage 2: one wavefront per tensor adds that tensor's run sums (lane-strided,
// then over the lanes).  Stage 3, only for lists of several tensors: one
// wavefront adds the tensor sums the same way.  The order of every addition is
// fixed by the shapes alone.
// ============================================================================
constexpr int kFinalThreads = 256;

__global__ __launch_bounds__(kFinalThreads) void k_reduce_runs(const double *__restrict__ partial_all, uint32_t n_blocks, int first_acc,
                                                             const SegRec *__restrict__ seg, double *__restrict__ seg_sum_all) {
    // blockIdx.x: run, blockIdx.y: accumulator
    const uint32_t stride = partial_stride(n_blocks);
    const double *partial = partial_all + (size_t)(first_acc + blockIdx.y) * partial_pitch(n_blocks);
    double *seg_sum = seg_sum_all + (size_t)(first_acc + blockIdx.y) * gridDim.x;
    // no table: a single tensor, whose runs follow from the block count alone
    const uint32_t run_first = blockIdx.x * kSegPartials;
    const SegRec sr = seg ? seg[blockIdx.x] : SegRec{run_first, n_blocks - run_first < kSegPartials ? n_blocks - run_first : kSegPartials};
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < sr.count; i += kFinalThreads) acc += partial[partial_slot(sr.first + i, stride)];
    acc = wave_sum(acc);
    __shared__ double wave_part[kFinalThreads / 64];
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kFinalThreads / 64; ++w) total += wave_part[w];
        seg_sum[blockIdx.x] = total;
    }
}

__global__ __launch_bounds__(kFinalThreads) void k_reduce_tensors(const double *__restrict__ seg_sum_all, uint32_t n_segs, int first_acc,
                                                                const uint32_t *__restrict__ tensor_seg_start, uint32_t n_tensors,
                                                                double *__restrict__ result_all) {
    // blockIdx.x: group of kFinalThreads / 64 tensors, blockIdx.y: accumulator.  One wavefront per
    // tensor: lane l adds runs l, l + 64, ... in order, then the lanes are summed.
    const double *seg_sum = seg_sum_all + (size_t)(first_acc + blockIdx.y) * n_segs;
    double *result = result_all + (size_t)(first_acc + blockIdx.y) * (1 + n_tensors);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t t = blockIdx.x * (kFinalThreads / 64) + (threadIdx.x >> 6);
    if (t >= n_tensors) return;                          // whole wavefronts leave together
    double acc = 0.0;
    const uint32_t run_lo = tensor_seg_start ? tensor_seg_start[t] : 0u;           // no table: one tensor owning every run
    const uint32_t run_hi = tensor_seg_start ? tensor_seg_start[t + 1] : n_segs;
    for (uint32_t i = run_lo + lane; i < run_hi; i += 64) acc += seg_sum[i];
    acc = wave_sum(acc);
    if (lane == 0) {
        result[1 + t] = acc;
        if (n_tensors == 1) result[0] = acc;             // nothing left to add: the total is this tensor's sum
    }
}

// Stage 3 (lists of several tensors): one wavefront per accumulator adds the tensor sums,
// lane-strided in index order, then over the lanes.
__global__ __launch_bounds__(64) void k_reduce_total(uint32_t n_tensors, int first_acc, double *__restrict__ result_all) {
    double *result = result_all + (size_t)(first_acc + blockIdx.x) * (1 + n_tensors);
    double total = 0.0;
    for (uint32_t t = threadIdx.x; t < n_tensors; t += 64) total += result[1 + t];
    total = wave_sum(total);
    if (threadIdx.x == 0) result[0] = total;
}

// ============================================================================
// Plain streaming copy with the engine's access pattern (measurement reference).
// ============================================================================
__global__ __launch_bounds__(64) void k_stream_copy(const float *__restrict__ src, float *__restrict__ dst, uint64_t n_elems) {
    const uint64_t e0 = (uint64_t)blockIdx.x * kWaveElems;
    const uint64_t rem = n_elems - e0;
    const uint32_t cnt = rem < kWaveElems ? (uint32_t)rem : kWaveElems;
    const auto r_s = span_rsrc(src + e0, cnt * 4u);
    const auto r_d = span_rsrc(dst + e0, cnt * 4u);
    const uint32_t elem = threadIdx.x * kLaneElems;
    // n_elems is a multiple of 4, so a lane's 4 elements are all inside or all outside the span
    store_f32(r_d, elem, true, load_f32(r_s, elem, true));
}

}  // namespace

hipError_t launch_step(const Layout &L, int optimizer, int grad_dtype, const GradArg &g, const StepParams &p, int src, int dst,
                       int write_moments, int write_copy, double *partial, const GradArg &dot, const float *clip, int clip_index,
                       hipStream_t st) {
    const dim3 grid(L.n_blocks), block(64);
    if (optimizer == 0 && grad_dtype == 0) k_optim_step<0, 0><<<grid, block, 0, st>>>(L, g, p, src, dst, write_moments, write_copy, partial, dot, clip, clip_index);
    else if (optimizer == 0) k_optim_step<0, 1><<<grid, block, 0, st>>>(L, g, p, src, dst, write_moments, write_copy, partial, dot, clip, clip_index);
    else if (grad_dtype == 0) k_optim_step<1, 0><<<grid, block, 0, st>>>(L, g, p, src, dst, write_moments, write_copy, partial, dot, clip, clip_index);
    else k_optim_step<1, 1><<<grid, block, 0, st>>>(L, g, p, src, dst, write_moments, write_copy, partial, dot, clip, clip_index);
    return hipGetLastError();
}

hipError_t launch_extrapolate(const Layout &L, int grad_dtype, const GradArg &g0, const GradArg &g1, const ExtrapParams &e,
                              int write_copy, double *diag, const float *clip, hipStream_t st) {
    const dim3 grid(L.n_blocks), block(64);
    if (diag) {
        if (grad_dtype == 0) k_extrapolate<0, true><<<grid, block, 0, st>>>(L, g0, g1, e, write_copy, diag, clip);
        else k_extrapolate<1, true><<<grid, block, 0, st>>>(L, g0, g1, e, write_copy, diag, clip);
    } else {
        if (grad_dtype == 0) k_extrapolate<0, false><<<grid, block, 0, st>>>(L, g0, g1, e, write_copy, nullptr, clip);
        else k_extrapolate<1, false><<<grid, block, 0, st>>>(L, g0, g1, e, write_copy, nullptr, clip);
    }
    return hipGetLastError();
}

namespace {
template <bool DIAG>
hipError_t fused_launch(const Layout &L, int optimizer, int grad_dtype, const GradArg &g0, const GradArg &g1, const StepParams &p1,
                        const StepParams &p2, const ExtrapParams &e, int src, int dst, int write_copy, double *diag, const float *clip,
                        hipStream_t st) {
    const dim3 grid(L.n_blocks), block(64);
    if (optimizer == 0 && grad_dtype == 0) k_fused_steps_extrapolate<0, 0, DIAG><<<grid, block, 0, st>>>(L, g0, g1, p1, p2, e, src, dst, write_copy, diag, clip);
    else if (optimizer == 0) k_fused_steps_extrapolate<0, 1, DIAG><<<grid, block, 0, st>>>(L, g0, g1, p1, p2, e, src, dst, write_copy, diag, clip);
    else if (grad_dtype == 0) k_fused_steps_extrapolate<1, 0, DIAG><<<grid, block, 0, st>>>(L, g0, g1, p1, p2, e, src, dst, write_copy, diag, clip);
    else k_fused_steps_extrapolate<1, 1, DIAG><<<grid, block, 0, st>>>(L, g0, g1, p1, p2, e, src, dst, write_copy, diag, clip);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_fused_steps_extrapolate(const Layout &L, int optimizer, int grad_dtype, const GradArg &d_g0, const GradArg &d_g1,
                                          const StepParams &p1, const StepParams &p2, const ExtrapParams &e, int src, int dst,
                                          int write_copy, double *d_diag_partial, const float *d_clip, hipStream_t stream) {
    return d_diag_partial ? fused_launch<true>(L, optimizer, grad_dtype, d_g0, d_g1, p1, p2, e, src, dst, write_copy, d_diag_partial, d_clip, stream)
                          : fused_launch<false>(L, optimizer, grad_dtype, d_g0, d_g1, p1, p2, e, src, dst, write_copy, nullptr, d_clip, stream);
}

hipError_t launch_sumsq(const Layout &L, int grad_dtype, const GradArg &g, double *partial, int acc, hipStream_t st) {
    const dim3 grid((L.n_blocks + kSumsqGroup - 1) / kSumsqGroup), block(64);
    if (grad_dtype == 0) k_sumsq<0><<<grid, block, 0, st>>>(L, g, partial, acc);
    else k_sumsq<1><<<grid, block, 0, st>>>(L, g, partial, acc);
    return hipGetLastError();
}

hipError_t launch_clip_coefficient(const double *d_result, uint32_t n_tensors, int acc, double max_norm, float *d_clip,
                                   int clip_index, hipStream_t stream) {
    k_clip_coefficient<<<dim3(1), dim3(1), 0, stream>>>(d_result, n_tensors, acc, max_norm, d_clip, clip_index);
    return hipGetLastError();
}

hipError_t launch_reposition(const Layout &L, float alpha, int write_copy, hipStream_t stream) {
    k_reposition<<<dim3(L.n_blocks), dim3(64), 0, stream>>>(L, alpha, write_copy);
    return hipGetLastError();
}

hipError_t launch_finalize(const double *d_partial, uint32_t n_blocks, const SegRec *d_seg, uint32_t n_segs,
                           const uint32_t *d_tensor_seg_start, uint32_t n_tensors, double *d_seg_sum, double *d_result,
                           int first_acc, int n_acc, hipStream_t stream) {
    k_reduce_runs<<<dim3(n_segs, n_acc), dim3(kFinalThreads), 0, stream>>>(d_partial, n_blocks, first_acc, d_seg, d_seg_sum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint32_t tensors_per_block = kFinalThreads / 64;
    k_reduce_tensors<<<dim3((n_tensors + tensors_per_block - 1) / tensors_per_block, n_acc), dim3(kFinalThreads), 0, stream>>>(
        d_seg_sum, n_segs, first_acc, d_tensor_seg_start, n_tensors, d_result);
    e = hipGetLastError();
    if (e != hipSuccess || n_tensors == 1) return e;
    k_reduce_total<<<dim3(n_acc), dim3(64), 0, stream>>>(n_tensors, first_acc, d_result);
    return hipGetLastError();
}

// ============================================================================
// Slow step + norm for callers that cannot allocate: the reduction workspace is
// a file-scope device array instead of memory from gxpo_init.  Each GPU holds
// its own copy of the array at its own address; the address is looked up once
// per device and kept.  Nothing in the array has to start at zero: every block
// of a launch writes its own partial, the reduction reads exactly the partials,
// run sums and results the launch wrote, so what an earlier (larger) call left
// behind is never read.
// ============================================================================
constexpr size_t kNoAllocRuns = (kNoAllocMaxBlocks + kSegPartials - 1) / kSegPartials;
constexpr size_t kNoAllocDoubles = (size_t)8 * ((kNoAllocMaxBlocks + 7u) >> 3) + kNoAllocRuns + 2;
static __device__ __align__(256) double scratch[kNoAllocDoubles];

namespace {
constexpr int kMaxDevices = 64;
double *g_scratch_ptr[kMaxDevices];            // device address of `scratch` on each GPU, nullptr until looked up
}  // namespace

hipError_t launch_slow_step_noalloc(const Layout &L, int optimizer, int grad_dtype, const GradArg &g, const StepParams &p,
                                    int write_copy, double *d_sum_sq_out, hipStream_t stream) {
    if (L.n_tensors != 1 || L.n_blocks == 0 || L.n_blocks > kNoAllocMaxBlocks) return hipErrorInvalidValue;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    double *ws = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!ws) {
        // `scratch` names the array for the host only; kernels need this GPU's address of it
        e = hipGetSymbolAddress((void **)&ws, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ws) return hipErrorInvalidSymbol;
        __atomic_store_n(&g_scratch_ptr[dev], ws, __ATOMIC_RELEASE);
    }
    double *partial = ws;
    double *run_sum = ws + partial_pitch(kNoAllocMaxBlocks);
    double *result = run_sum + kNoAllocRuns;
    e = launch_step(L, optimizer, grad_dtype, g, p, kSrcTheta, kSrcTheta, 1, write_copy, partial, GradArg{}, nullptr, 0, stream);
    if (e != hipSuccess) return e;
    const uint32_t n_runs = (L.n_blocks + kSegPartials - 1) / kSegPartials;
    e = launch_finalize(partial, L.n_blocks, nullptr, n_runs, nullptr, 1, run_sum, result, kAccSlowSq, 1, stream);
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(d_sum_sq_out, result, sizeof(double), hipMemcpyDeviceToDevice, stream);
}

hipError_t launch_stream_copy(void *dst, const void *src, uint64_t bytes, hipStream_t stream) {
    const uint64_t n_elems = bytes / 4;
    const uint64_t blocks = (n_elems + kWaveElems - 1) / kWaveElems;
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    k_stream_copy<<<dim3((uint32_t)blocks), dim3(64), 0, stream>>>((const float *)src, (float *)dst, n_elems);
    return hipGetLastError();
}

}  // namespace gxpo
