// Internal interface between the host side of the library (gxpo_host.cpp) and
// its gfx950 kernels (gxpo_kernels.hip).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gxpo {

// One wavefront handles 64 lanes x 4 consecutive elements of one tensor.
constexpr uint32_t kLaneElems = 4;
constexpr uint32_t kWaveElems = 64 * kLaneElems;
// The coarse block->tensor index has one entry per 2^kCoarseShift blocks.
constexpr uint32_t kCoarseShift = 6;
// Partials of one tensor are reduced in runs of at most this many.
constexpr uint32_t kSegPartials = 8192;

struct TensorRec {          // device copy of one gxpo_tensor
    float *theta;
    float *probe;
    float *m;
    float *v;
    void *copy;             // bf16 model copy or nullptr
    float *m_alt;           // second buffers for the moments (alternating state) or nullptr
    float *v_alt;
    uint64_t numel;
    float lr_scale;         // parameter group: multiplies the step size (1 = the context's lr)
    float lr_wd_scale;      // lr_scale * weight_decay_scale: multiplies lr * weight_decay
};

// How the 1-D grid covers the ragged tensor list: tensor t owns blocks
// [blk_start[t], blk_start[t+1]); coarse[b >> kCoarseShift] is the tensor that
// owns block (b >> kCoarseShift) << kCoarseShift.
struct Layout {
    const TensorRec *tab;
    const uint32_t *blk_start;
    const uint32_t *coarse;
    uint32_t n_tensors;
    uint32_t n_blocks;
    TensorRec single;       // copy of tab[0]; used instead of the tables when n_tensors == 1
};

// Per-block partial sums are stored XCD-major: blocks are handed to the 8 XCDs
// round-robin, so block b's partial goes to slot (b % 8) * stride + b / 8 and
// each XCD's L2 sees its own partials as one dense, growing run of doubles
// (full-line write-backs instead of eight XCDs each writing 8 bytes of a line).
__host__ __device__ inline uint32_t partial_stride(uint32_t n_blocks) { return (n_blocks + 7u) >> 3; }
__host__ __device__ inline uint32_t partial_slot(uint32_t block, uint32_t stride) { return (block & 7u) * stride + (block >> 3); }

// One gradient list as a kernel argument: the device pointer table, plus the
// pointer itself when there is a single tensor (saves a dependent load).
struct GradArg {
    const void *const *table;
    const void *single;
};

// OptimStep constants, derived in double on the host, rounded once to fp32.
struct StepParams {
    float beta1, one_minus_beta1;
    float beta2, one_minus_beta2;
    float lr_wd;            // lr * weight_decay
    float step_size;        // lr / (1 - beta1^s)
    float rsqrt_bias2;      // 1 / sqrt(1 - beta2^s)
    float eps;
    float lr;               // plain GD
};

struct ExtrapParams {
    float alpha;
    float delta;            // fp32(delta)
    float r_max;            // fp32(r_max), +inf = no clamp
    uint32_t half;          // K/2 (K even) or (K-1)/2 (K odd)
    uint32_t odd;           // K & 1
};

struct SegRec {             // a run of per-block partials inside one tensor
    uint32_t first;
    uint32_t count;
};

// Which buffers a pass reads (src) and writes (dst): bit 0 picks the parameter buffer (theta or
// theta_probe), bit 1 the moments (m, v or m_alt, v_alt).  With alternating state the two sets
// {theta, m, v} and {theta_probe, m_alt, v_alt} are kSetMain and kSetAlt.
enum { kSrcTheta = 0, kSrcProbe = 1, kMomentsAlt = 2, kSetMain = 0, kSetAlt = kSrcProbe | kMomentsAlt };

// Reduction accumulators.  Each owns one XCD-major array of per-block partials,
// `partial_pitch(n_blocks)` doubles apart.  Only kAccSlowSq exists unless the
// context was created with diagnostics.
enum {
    kAccSlowSq = 0,    // sum g_slow^2                      (slow step)
    kAccG0Slow = 1,    // sum g0 * g_slow                   (slow step, diagnostics)
    kAccG0Sq = 2,      // sum g0^2                          (extrapolation pass, diagnostics; so are all below)
    kAccG1Sq = 3,      // sum g1^2
    kAccActive = 4,    // number of active coordinates
    kAccR = 5,         // sum over the active set of (r - 1)
    kAccR2 = 6,        // sum over the active set of (r - 1)^2
    kAccScale = 7,     // sum over the active set of scale
    kAccD2 = 8,        // sum (theta^{t,2} - theta^t)^2
    kAccDK = 9,        // sum (theta^{t,K} - theta^t)^2
    kAccClipG0 = 10,   // sum g0^2, pre-pass for gradient clipping (also the fallback step's gradient)
    kAccClipG1 = 11,   // sum g1^2, pre-pass for gradient clipping
    kNumAcc = 12
};
constexpr int kNumExtrapAcc = kAccDK - kAccG0Sq + 1;

// Gradient clipping: coef points to three device floats (for g0, g1, g_slow), each
// min(1, max_norm / (||g|| + 1e-6)), written by the norm pre-pass; nullptr = no clipping.
enum { kClipG0 = 0, kClipG1 = 1, kClipSlow = 2 };
__host__ __device__ inline size_t partial_pitch(uint32_t n_blocks) { return (size_t)8 * ((n_blocks + 7u) >> 3); }

// All launchers enqueue on `stream` and return the launch status.
// d_partial: nullptr = no reduction; otherwise sum g^2 goes to accumulator kAccSlowSq and, when
// d_g0_for_dot holds a list, sum g0*g to kAccG0Slow.
hipError_t launch_step(const Layout &L, int optimizer, int grad_dtype,
                       const GradArg &d_grads, const StepParams &p,
                       int src, int dst, int write_moments, int write_copy, double *d_partial,
                       const GradArg &d_g0_for_dot, const float *d_clip, int clip_index, hipStream_t stream);

// sum of squares of one gradient list into accumulator `acc` (read-only pass, 4 or 2 B/param)
hipError_t launch_sumsq(const Layout &L, int grad_dtype, const GradArg &d_grads, double *d_partial, int acc,
                        hipStream_t stream);

// d_clip[clip_index] = min(1, max_norm / (sqrt(result of accumulator acc) + 1e-6))
hipError_t launch_clip_coefficient(const double *d_result, uint32_t n_tensors, int acc, double max_norm, float *d_clip,
                                   int clip_index, hipStream_t stream);

// d_diag_partial (both extrapolation launchers): nullptr, or the partial arrays; then the pass
// also fills accumulators kAccG0Sq .. kAccDK.
hipError_t launch_extrapolate(const Layout &L, int grad_dtype,
                              const GradArg &d_g0, const GradArg &d_g1,
                              const ExtrapParams &e, int write_copy, double *d_diag_partial, const float *d_clip,
                              hipStream_t stream);

// theta <- theta + alpha (theta_probe - theta), nothing else (explicit lookahead).
hipError_t launch_reposition(const Layout &L, float alpha, int write_copy, hipStream_t stream);

// p1 / p2: constants of the first / second fast step (both are applied here).  src / dst: the set (kSetMain or
// kSetAlt) the pass reads theta^t, m, v from and the set it writes theta~, m, v to; equal = in place.
hipError_t launch_fused_steps_extrapolate(const Layout &L, int optimizer, int grad_dtype,
                                          const GradArg &d_g0, const GradArg &d_g1,
                                          const StepParams &p1, const StepParams &p2, const ExtrapParams &e,
                                          int src, int dst, int write_copy, double *d_diag_partial, const float *d_clip,
                                          hipStream_t stream);

// Reduces accumulators [first_acc, first_acc + n_acc).  For accumulator a:
// result[a * (1 + n_tensors)] = sum over all tensors, result[a * (1 + n_tensors) + 1 + t] = tensor t.
hipError_t launch_finalize(const double *d_partial, uint32_t n_blocks, const SegRec *d_seg, uint32_t n_segs,
                           const uint32_t *d_tensor_seg_start, uint32_t n_tensors,
                           double *d_seg_sum, double *d_result, int first_acc, int n_acc, hipStream_t stream);

hipError_t launch_stream_copy(void *dst, const void *src, uint64_t bytes, hipStream_t stream);

// Slow step + sum of squares of one flat tensor with the reduction workspace in a file-scope device
// array (no allocation anywhere): at most kNoAllocMaxBlocks blocks.  The sum lands in *d_sum_sq_out.
constexpr uint32_t kNoAllocMaxBlocks = 1u << 20;
hipError_t launch_slow_step_noalloc(const Layout &L, int optimizer, int grad_dtype, const GradArg &g, const StepParams &p,
                                    int write_copy, double *d_sum_sq_out, hipStream_t stream);

}  // namespace gxpo
