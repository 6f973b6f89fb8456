// hbm_probe -- stand-alone measurements behind the engine's launch shape, cache policy, buffer
// phases and rank-aware placement on MI355X (gfx950).  Not part of libgxpo.so: a small program
// that streams synthetic arrays with the engine's access pattern and prints GB/s, so that every
// design choice quoted in the documentation can be re-measured with one command:
//
//     hbm_probe shape      one-wave one-shot blocks vs wider blocks, 8 elements per lane, grid-stride loops
//     hbm_probe policy     cache-policy bits of the buffer accesses, and plain global accesses
//     hbm_probe phase      base addresses of the streams modulo 64 KiB
//     hbm_probe ranks      one read stream moved across a 200 GiB allocation (DRAM rank regions)
//     hbm_probe bf16       the fused pass with two bf16 gradient streams: 64-bit vs 128-bit accesses
//     hbm_probe chunks     512 MiB physical chunks (virtual-memory API): which pairs and triples of chunks slow each other down
//     hbm_probe sets       the same chunks sorted by rank: which ranks a pass should read from and write to (in place / out of place)
//
// The pass modelled is the AdamW-shaped step: read theta, m, v, g; write theta', m, v (28 B per
// element with fp32 gradients), arithmetic reduced to a few multiply-adds (the real arithmetic
// changes the time by < 0.2 %).  Arrays hold pseudo-random data (all-zero data streams faster).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define CK(x)                                                                                   \
    do {                                                                                        \
        hipError_t e_ = (x);                                                                    \
        if (e_ != hipSuccess) {                                                                 \
            printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__);      \
            exit(1);                                                                            \
        }                                                                                       \
    } while (0)

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void *base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
template <int POL> __device__ __forceinline__ f4 ld(__amdgpu_buffer_rsrc_t r, int off) {
    return __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, POL));
}
template <int POL> __device__ __forceinline__ void st(__amdgpu_buffer_rsrc_t r, int off, f4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, v), r, off, 0, POL);
}
__device__ __forceinline__ void math(f4 &T, f4 &M, f4 &V, f4 G) {
    M = M * 0.9f + G;
    V = V * 0.99f + G * G;
    T = T + M * 1e-6f + V * 1e-7f;
}
__device__ __forceinline__ unsigned span_bytes(size_t n, size_t e0, unsigned block_elems) {
    const size_t rem = n - e0;
    return (unsigned)(rem < block_elems ? rem : block_elems) * 4u;
}

// one-shot blocks of WPB wavefronts, EPL elements per lane (EPL 8: two 128-bit accesses, 1 KiB apart), policy POL
template <int WPB, int EPL, int POL>
__global__ __launch_bounds__(64 * WPB) void k_step(const float *th_in, float *th_out, float *m, float *v, const float *g, size_t n) {
    constexpr unsigned BE = 64 * WPB * EPL;
    const size_t e0 = (size_t)blockIdx.x * BE;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, BE);
    const auto rt = rsrc(th_in + e0, bytes), ro = rsrc(th_out + e0, bytes), rm = rsrc(m + e0, bytes), rv = rsrc(v + e0, bytes),
               rg = rsrc(g + e0, bytes);
    f4 T[EPL / 4], M[EPL / 4], V[EPL / 4], G[EPL / 4];
#pragma unroll
    for (int j = 0; j < EPL / 4; ++j) {
        const int off = (j * 64 * WPB + threadIdx.x) * 16;
        T[j] = ld<POL>(rt, off), M[j] = ld<POL>(rm, off), V[j] = ld<POL>(rv, off), G[j] = ld<POL>(rg, off);
    }
#pragma unroll
    for (int j = 0; j < EPL / 4; ++j) {
        const int off = (j * 64 * WPB + threadIdx.x) * 16;
        math(T[j], M[j], V[j], G[j]);
        st<POL>(ro, off, T[j]), st<POL>(rm, off, M[j]), st<POL>(rv, off, V[j]);
    }
}

// the same step with the two moments in ONE array, interleaved per block: 1 KiB of m, then 1 KiB of v (one stream fewer)
__global__ __launch_bounds__(64) void k_step_mv(const float *th_in, float *th_out, float *mv, const float *g, size_t n) {
    const size_t e0 = (size_t)blockIdx.x * 256;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, 256);
    const int off = threadIdx.x * 16;
    const auto rm = rsrc(mv + 2 * e0, bytes), rv = rsrc(mv + 2 * e0 + 256, bytes);
    f4 T = ld<18>(rsrc(th_in + e0, bytes), off), M = ld<18>(rm, off), V = ld<18>(rv, off), G = ld<18>(rsrc(g + e0, bytes), off);
    math(T, M, V, G);
    st<18>(rsrc(th_out + e0, bytes), off, T), st<18>(rm, off, M), st<18>(rv, off, V);
}

// persistent blocks that walk the arrays with a grid stride
template <int WPB>
__global__ __launch_bounds__(64 * WPB) void k_step_stride(const float *th_in, float *th_out, float *m, float *v, const float *g, size_t n) {
    constexpr unsigned BE = 64 * WPB * 4;
    for (size_t e0 = (size_t)blockIdx.x * BE; e0 < n; e0 += (size_t)gridDim.x * BE) {
        const unsigned bytes = span_bytes(n, e0, BE);
        const auto rt = rsrc(th_in + e0, bytes), ro = rsrc(th_out + e0, bytes), rm = rsrc(m + e0, bytes), rv = rsrc(v + e0, bytes),
                   rg = rsrc(g + e0, bytes);
        const int off = threadIdx.x * 16;
        f4 T = ld<18>(rt, off), M = ld<18>(rm, off), V = ld<18>(rv, off), G = ld<18>(rg, off);
        math(T, M, V, G);
        st<18>(ro, off, T), st<18>(rm, off, M), st<18>(rv, off, V);
    }
}

// plain global accesses (no buffer descriptors); NT selects non-temporal builtins
template <bool NT>
__global__ __launch_bounds__(64) void k_step_global(const f4 *th_in, f4 *th_out, f4 *m, f4 *v, const f4 *g, size_t n4) {
    const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= n4) return;
    f4 T, M, V, G;
    if (NT) {
        T = __builtin_nontemporal_load(th_in + i), M = __builtin_nontemporal_load(m + i), V = __builtin_nontemporal_load(v + i),
        G = __builtin_nontemporal_load(g + i);
    } else {
        T = th_in[i], M = m[i], V = v[i], G = g[i];
    }
    math(T, M, V, G);
    if (NT) {
        __builtin_nontemporal_store(T, th_out + i), __builtin_nontemporal_store(M, m + i), __builtin_nontemporal_store(V, v + i);
    } else {
        th_out[i] = T, m[i] = M, v[i] = V;
    }
}

// in-place step: read theta, m, v, g; write theta, m, v (the slow step's shape)
__global__ __launch_bounds__(64) void k_slow(float *th, float *m, float *v, const float *g, size_t n) {
    const size_t e0 = (size_t)blockIdx.x * 256;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, 256);
    const int off = threadIdx.x * 16;
    const auto rt = rsrc(th + e0, bytes), rm = rsrc(m + e0, bytes), rv = rsrc(v + e0, bytes);
    f4 T = ld<18>(rt, off), M = ld<18>(rm, off), V = ld<18>(rv, off), G = ld<18>(rsrc(g + e0, bytes), off);
    math(T, M, V, G);
    st<18>(rt, off, T), st<18>(rm, off, M), st<18>(rv, off, V);
}

__global__ __launch_bounds__(64) void k_copy(const float *src, float *dst, size_t n) {
    const size_t e0 = (size_t)blockIdx.x * 256;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, 256);
    st<18>(rsrc(dst + e0, bytes), threadIdx.x * 16, ld<18>(rsrc(src + e0, bytes), threadIdx.x * 16));
}

// the slow step's shape out of place: read theta, m, v, g; write theta', m', v' elsewhere
__global__ __launch_bounds__(64) void k_slow_oop(const float *th, const float *m, const float *v, const float *g, float *th2, float *m2,
                                                  float *v2, size_t n) {
    const size_t e0 = (size_t)blockIdx.x * 256;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, 256);
    const int off = threadIdx.x * 16;
    f4 T = ld<18>(rsrc(th + e0, bytes), off), M = ld<18>(rsrc(m + e0, bytes), off), V = ld<18>(rsrc(v + e0, bytes), off);
    const f4 G = ld<18>(rsrc(g + e0, bytes), off);
    math(T, M, V, G);
    st<18>(rsrc(th2 + e0, bytes), off, T), st<18>(rsrc(m2 + e0, bytes), off, M), st<18>(rsrc(v2 + e0, bytes), off, V);
}

// two streams read and written in place at the same element offset
__global__ __launch_bounds__(64) void k_rmw2(float *a, float *b, size_t n) {
    const size_t e0 = (size_t)blockIdx.x * 256;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, 256);
    const int off = threadIdx.x * 16;
    const auto ra = rsrc(a + e0, bytes), rb = rsrc(b + e0, bytes);
    const f4 A = ld<18>(ra, off), B = ld<18>(rb, off);
    st<18>(ra, off, A * 0.999f + B * 1e-6f), st<18>(rb, off, B * 0.999f + A * 1e-6f);
}

__device__ __forceinline__ f4 widen(unsigned a, unsigned b) {
    f4 o;
    o[0] = __builtin_bit_cast(float, a << 16), o[1] = __builtin_bit_cast(float, a & 0xffff0000u);
    o[2] = __builtin_bit_cast(float, b << 16), o[3] = __builtin_bit_cast(float, b & 0xffff0000u);
    return o;
}
// the fused pass's shape: read theta, m, v, g0, g1; write theta, m, v.  MODE 0: fp32 gradients; 1: bf16 gradients, one
// 64-bit access per lane; 2: bf16, lanes 0..31 issue 128-bit accesses and the data is handed to the owning lanes.
template <int MODE>
__global__ __launch_bounds__(64) void k_fused(float *th, float *m, float *v, const void *g0, const void *g1, size_t n) {
    const size_t e0 = (size_t)blockIdx.x * 256;
    if (e0 >= n) return;
    const unsigned bytes = span_bytes(n, e0, 256);
    const int off = threadIdx.x * 16;
    const auto rt = rsrc(th + e0, bytes), rm = rsrc(m + e0, bytes), rv = rsrc(v + e0, bytes);
    auto grad = [&](const void *g) -> f4 {
        if (MODE == 0) return ld<18>(rsrc((const float *)g + e0, bytes), off);
        const auto rg = rsrc((const unsigned short *)g + e0, bytes / 2);
        if (MODE == 1) {
            const u2 x = __builtin_amdgcn_raw_buffer_load_b64(rg, threadIdx.x * 8, 0, 18);
            return widen(x[0], x[1]);
        }
        u4 x = {0, 0, 0, 0};
        if (threadIdx.x < 32) x = __builtin_amdgcn_raw_buffer_load_b128(rg, threadIdx.x * 16, 0, 18);
        const int src = (threadIdx.x >> 1) * 4;
        const unsigned a0 = __builtin_amdgcn_ds_bpermute(src, x[0]), a1 = __builtin_amdgcn_ds_bpermute(src, x[1]);
        const unsigned a2 = __builtin_amdgcn_ds_bpermute(src, x[2]), a3 = __builtin_amdgcn_ds_bpermute(src, x[3]);
        return (threadIdx.x & 1) ? widen(a2, a3) : widen(a0, a1);
    };
    f4 T = ld<18>(rt, off), M = ld<18>(rm, off), V = ld<18>(rv, off);
    const f4 G = grad(g0), H = grad(g1);
    math(T, M, V, G + H * 0.1f);
    st<18>(rt, off, T), st<18>(rm, off, M), st<18>(rv, off, V);
}

__global__ void k_fill(float *p, size_t n, unsigned seed) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        unsigned x = (unsigned)i * 2654435761u + seed;
        x ^= x >> 15, x *= 2246822519u, x ^= x >> 13;
        p[i] = ((int)(x >> 9) - (1 << 22)) * (0.02f / (1 << 22));
    }
}

// best of three batches of `iters` launches, in GB/s
template <typename F> static double gbps(F launch, double bytes, int iters = 8) {
    static hipEvent_t a, b;
    static bool made = false;
    if (!made) {
        CK(hipEventCreate(&a));
        CK(hipEventCreate(&b));
        made = true;
    }
    launch();
    double best = 0;
    for (int r = 0; r < 3; ++r) {
        CK(hipEventRecord(a));
        for (int i = 0; i < iters; ++i) launch();
        CK(hipEventRecord(b));
        CK(hipEventSynchronize(b));
        float ms;
        CK(hipEventElapsedTime(&ms, a, b));
        best = std::max(best, bytes * iters / ms / 1e6);
    }
    CK(hipGetLastError());
    return best;
}

static const size_t MiB = 1ull << 20, GiB = 1ull << 30;
static char *arena(size_t bytes) {
    char *base;
    CK(hipMalloc(&base, bytes + GiB));
    base += (GiB - (size_t)base % GiB) % GiB;
    k_fill<<<16384, 256>>>((float *)base, bytes / 4, 7);
    CK(hipDeviceSynchronize());
    CK(hipGetLastError());
    return base;
}
static void line(const char *what, double g) {
    printf("  %-84s %7.0f GB/s  %5.1f %% of 8 TB/s\n", what, g, g / 80.0);
    fflush(stdout);
}

// five arrays of n elements, 2 MiB-multiple pitch, moments 32 KiB out of phase unless told otherwise
struct Five { float *a[5]; };
static Five place(char *base, size_t pitch, const size_t *phase) {
    Five f;
    for (int k = 0; k < 5; ++k) f.a[k] = (float *)(base + k * pitch + phase[k]);
    return f;
}

static int run_shape() {
    const size_t n = 1540000000ull, pitch = ((n * 4 + 2 * MiB - 1) / (2 * MiB) + 1) * 2 * MiB;
    char *base = arena(pitch * 5);
    const size_t ph[5] = {0, 0, 32768, 32768, 0};
    const Five f = place(base, pitch, ph);
    printf("launch shape, AdamW-shaped step (28 B/element), n = %zu fp32 per array, moments +32 KiB\n", n);
    auto nb = [&](unsigned be) { return (unsigned)((n + be - 1) / be); };
    line("one-shot blocks, 1 wavefront, 4 elements per lane  [the engine's shape]", gbps([&] { k_step<1, 4, 18><<<nb(256), 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("one-shot blocks, 2 wavefronts", gbps([&] { k_step<2, 4, 18><<<nb(512), 128>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("one-shot blocks, 4 wavefronts", gbps([&] { k_step<4, 4, 18><<<nb(1024), 256>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("one-shot blocks, 1 wavefront, 8 elements per lane (two 128-bit accesses per stream)", gbps([&] { k_step<1, 8, 18><<<nb(512), 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    for (int per_cu : {4, 8, 16, 32})
        {
            char what[96];
            snprintf(what, sizeof what, "grid-stride loop, 1-wavefront blocks, %d blocks per CU", per_cu);
            line(what, gbps([&] { k_step_stride<1><<<256 * per_cu, 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
        }
    line("grid-stride loop, 4-wavefront blocks, 8 blocks per CU", gbps([&] { k_step_stride<4><<<256 * 8, 256>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    // the interleaved array takes the place of m and v: 8n bytes from m's start end before the gradient array begins
    line("1 wavefront, 4 elements per lane, m and v interleaved per block in one array", gbps([&] { k_step_mv<<<nb(256), 64>>>(f.a[0], f.a[1], f.a[2], f.a[4], n); }, 28.0 * n));
    line("plain copy, same shape (8 B/element)", gbps([&] { k_copy<<<nb(256), 64>>>(f.a[0], f.a[1], n); }, 8.0 * n));
    return 0;
}

static int run_policy() {
    const size_t n = 1540000000ull, pitch = ((n * 4 + 2 * MiB - 1) / (2 * MiB) + 1) * 2 * MiB;
    char *base = arena(pitch * 5);
    const size_t ph[5] = {0, 0, 32768, 32768, 0};
    const Five f = place(base, pitch, ph);
    const unsigned nb = (unsigned)((n + 255) / 256);
    printf("cache policy of the accesses, AdamW-shaped step, n = %zu\n", n);
    line("buffer accesses, sc1 + nt (streaming)  [the engine's policy]", gbps([&] { k_step<1, 4, 18><<<nb, 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("buffer accesses, nt only", gbps([&] { k_step<1, 4, 2><<<nb, 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("buffer accesses, sc1 only", gbps([&] { k_step<1, 4, 16><<<nb, 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("buffer accesses, default policy", gbps([&] { k_step<1, 4, 0><<<nb, 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    line("global accesses, non-temporal", gbps([&] { k_step_global<true><<<(unsigned)((n / 4 + 63) / 64), 64>>>((const f4 *)f.a[0], (f4 *)f.a[1], (f4 *)f.a[2], (f4 *)f.a[3], (const f4 *)f.a[4], n / 4); }, 28.0 * n));
    line("global accesses, default", gbps([&] { k_step_global<false><<<(unsigned)((n / 4 + 63) / 64), 64>>>((const f4 *)f.a[0], (f4 *)f.a[1], (f4 *)f.a[2], (f4 *)f.a[3], (const f4 *)f.a[4], n / 4); }, 28.0 * n));
    return 0;
}

static int run_phase() {
    const size_t n = 1540000000ull, pitch = ((n * 4 + 2 * MiB - 1) / (2 * MiB) + 1) * 2 * MiB;
    char *base = arena(pitch * 5);
    const unsigned nb = (unsigned)((n + 255) / 256);
    printf("base addresses modulo 64 KiB (KiB: theta_in, theta_out, m, v, g), AdamW-shaped step, n = %zu\n", n);
    const int combos[][5] = {{0, 0, 0, 0, 0},    {0, 0, 32, 32, 0},  {0, 32, 32, 32, 0}, {0, 0, 32, 32, 32}, {0, 32, 0, 32, 0},
                             {0, 0, 16, 48, 0},  {0, 16, 32, 48, 8}, {0, 8, 16, 24, 32}, {0, 0, 32, 0, 0},   {0, 4, 32, 36, 8}};
    for (const auto &c : combos) {
        size_t ph[5];
        for (int k = 0; k < 5; ++k) ph[k] = (size_t)c[k] * 1024;
        const Five f = place(base, pitch, ph);
        char what[96];
        snprintf(what, sizeof what, "phases %2d %2d %2d %2d %2d KiB%s", c[0], c[1], c[2], c[3], c[4], (c[2] == 32 && c[3] == 32 && !c[1] && !c[4]) ? "  [the layout rule]" : "");
        line(what, gbps([&] { k_step<1, 4, 18><<<nb, 64>>>(f.a[0], f.a[1], f.a[2], f.a[3], f.a[4], n); }, 28.0 * n));
    }
    return 0;
}

static int run_ranks() {
    const size_t n = 1ull << 27;                                    // 512 MiB windows
    const int span = 200;
    char *base = arena((size_t)(span + 8) * GiB);
    const unsigned nb = (unsigned)(n / 256);
    auto at = [&](int gib, size_t ph = 0) { return (float *)(base + (size_t)gib * GiB + ph); };
    printf("one 208 GiB allocation; slow-step shape (read theta, m, v, g; write theta, m, v) on 512 MiB windows:\n"
           "theta, m, v fixed at offsets ref, ref+1, ref+2 GiB, the gradient window at offset x.  Columns: ref = 0, 100, 195 GiB.\n"
           "A window in the same DRAM rank as the reference runs ~4 %% faster than one in another rank.\n"
           "   x GiB     ref 0   ref 100   ref 195   |  copy 0 -> x   all four at x..x+3\n");
    const int refs[3] = {0, 100, 195};
    for (int x = 3; x <= span; ++x) {
        printf("  %5d ", x);
        for (int r : refs) {
            if (x >= r - 1 && x <= r + 3) {
                printf("        - ");
                continue;
            }
            printf("   %6.0f ", gbps([&] { k_slow<<<nb, 64>>>(at(r), at(r + 1, 32768), at(r + 2, 32768), at(x), n); }, 28.0 * n, 5));
        }
        printf("  |   %6.0f      %6.0f\n", gbps([&] { k_copy<<<nb, 64>>>(at(0), at(x), n); }, 8.0 * n, 5),
               gbps([&] { k_slow<<<nb, 64>>>(at(x), at(x + 1, 32768), at(x + 2, 32768), at(x + 3), n); }, 28.0 * n, 5));
        fflush(stdout);
    }
    return 0;
}

static int run_bf16() {
    const size_t n = 1ull << 29, pitch = 2 * GiB + 2 * MiB;
    char *base = arena(pitch * 5);
    float *th = (float *)base, *m = (float *)(base + pitch + 32768), *v = (float *)(base + 2 * pitch + 32768);
    void *g0 = base + 3 * pitch, *g1 = base + 4 * pitch;
    const unsigned nb = (unsigned)(n / 256);
    printf("fused pass shape (read theta, m, v, g0, g1; write theta, m, v), n = %zu\n", n);
    line("fp32 gradients, 128-bit accesses (32 B/element)", gbps([&] { k_fused<0><<<nb, 64>>>(th, m, v, g0, g1, n); }, 32.0 * n));
    line("bf16 gradients, one 64-bit access per lane (28 B/element)  [the engine's]", gbps([&] { k_fused<1><<<nb, 64>>>(th, m, v, g0, g1, n); }, 28.0 * n));
    line("bf16 gradients, 128-bit accesses by half the lanes + cross-lane hand-over", gbps([&] { k_fused<2><<<nb, 64>>>(th, m, v, g0, g1, n); }, 28.0 * n));
    return 0;
}

static void percentiles(std::vector<double> v, const char *what) {
    std::sort(v.begin(), v.end());
    auto q = [&](double f) { return v[(size_t)(f * (v.size() - 1))]; };
    printf("  %-52s min %5.0f  5%% %5.0f  25%% %5.0f  median %5.0f  75%% %5.0f  95%% %5.0f  max %5.0f GB/s\n", what, v.front(), q(0.05), q(0.25), q(0.5),
           q(0.75), q(0.95), v.back());
    fflush(stdout);
}

static int run_chunks() {
    const size_t H = 512 * MiB;
    const int slots = 192;                                          // 96 GiB
    const size_t n = (H - 64 * 1024) / 4;                           // windows start at a chunk's first byte (+ phase) and end inside it
    const unsigned nb = (unsigned)((n + 255) / 256);
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned, prop.location.type = hipMemLocationTypeDevice, prop.location.id = 0;
    hipMemAccessDesc acc = {};
    acc.location = prop.location, acc.flags = hipMemAccessFlagsProtReadWrite;
    static hipMemGenericAllocationHandle_t h[slots];
    for (int i = 0; i < slots; ++i) CK(hipMemCreate(&h[i], H, &prop, 0));
    void *va;
    CK(hipMemAddressReserve(&va, slots * H, 2 * MiB, nullptr, 0));
    for (int i = 0; i < slots; ++i) CK(hipMemMap((char *)va + i * H, H, 0, h[i], 0));
    CK(hipMemSetAccess(va, slots * H, &acc, 1));
    char *base = (char *)va;
    k_fill<<<16384, 256>>>((float *)base, slots * H / 4, 7);
    CK(hipDeviceSynchronize());
    auto P = [&](int chunk, size_t phase = 0) { return (float *)(base + (size_t)chunk * H + phase); };   // phase <= 32 KiB: inside the chunk
    printf("%d chunks of 512 MiB from hipMemCreate, mapped in creation order; windows of %zu elements at the start of a chunk\n", slots, n);

    // chunks that share chunk 0's DRAM rank: gradient window in the candidate against theta, m, v in chunks 0, 1, 2
    std::vector<int> pool;
    {
        std::vector<double> r(slots, 0.0);
        for (int c = 3; c < slots; ++c) r[c] = gbps([&] { k_slow<<<nb, 64>>>(P(0), P(1, 32768), P(2, 32768), P(c), n); }, 28.0 * n, 3);
        std::vector<double> s(r.begin() + 3, r.end());
        std::sort(s.begin(), s.end());
        const double top = s[s.size() * 3 / 4];
        for (int c = 3; c < slots; ++c)
            if (r[c] > 0.975 * top) pool.push_back(c);
        printf("%zu of the chunks 3..%d share the rank of chunks 0-2 (gradient window there within 2.5 %% of the fast level)\n", pool.size(), slots - 1);
    }
    if (pool.size() < 48) {
        printf("too few chunks in one rank for the rest of this probe\n");
        return 1;
    }

    printf("pairs: two streams, both read and written in place, same phase; reference chunk against every chunk of the pool\n");
    for (int ref : {pool[0], pool[1], pool[40]}) {
        std::vector<double> r;
        std::vector<int> who, slow;
        for (int c : pool)
            if (c != ref) who.push_back(c), r.push_back(gbps([&] { k_rmw2<<<nb, 64>>>(P(ref), P(c), n); }, 16.0 * n, 3));
        char t[96];
        snprintf(t, sizeof t, "reference chunk %d", ref);
        percentiles(r, t);
        std::vector<double> s = r;
        std::sort(s.begin(), s.end());
        const double med = s[s.size() / 2];
        printf("    partners below 96 %% of the median:");
        for (size_t i = 0; i < r.size(); ++i)
            if (r[i] < 0.96 * med) printf(" %d", who[i]), slow.push_back(who[i]);
        printf("   (%zu of %zu)\n", slow.size(), r.size());
        // the same partners with the partner 32 KiB out of phase, and as a plain copy reference -> partner
        std::vector<double> ph, cp;
        for (int c : slow) ph.push_back(gbps([&] { k_rmw2<<<nb, 64>>>(P(ref), P(c, 32768), n); }, 16.0 * n, 3)),
            cp.push_back(gbps([&] { k_copy<<<nb, 64>>>(P(ref), P(c), n); }, 8.0 * n, 3));
        if (!slow.empty()) percentiles(ph, "    those partners, 32 KiB out of phase"), percentiles(cp, "    those partners, copy reference -> partner");
    }

    printf("triples: slow-step shape, theta, m, v (moments +32 KiB) and the gradient in four chunks drawn at random from the pool\n");
    {
        unsigned x = 12345;
        auto rnd = [&](int m) { x = x * 1664525u + 1013904223u; return (int)((x >> 8) % (unsigned)m); };
        std::vector<double> r, again;
        for (int t = 0; t < 600; ++t) {
            int c[4];
            for (int k = 0; k < 4; ++k) {
                bool fresh;
                do {
                    c[k] = pool[rnd((int)pool.size())], fresh = true;
                    for (int j = 0; j < k; ++j) fresh = fresh && c[j] != c[k];
                } while (!fresh);
            }
            r.push_back(gbps([&] { k_slow<<<nb, 64>>>(P(c[0]), P(c[1], 32768), P(c[2], 32768), P(c[3]), n); }, 28.0 * n, 3));
            if (t % 20 == 0) again.push_back(gbps([&] { k_slow<<<nb, 64>>>(P(c[0]), P(c[1], 32768), P(c[2], 32768), P(c[3]), n); }, 28.0 * n, 3) - r.back());
        }
        percentiles(r, "600 random quadruples");
        double s2 = 0;
        for (double d : again) s2 += d * d;
        printf("  the same quadruple measured twice differs by %.0f GB/s (rms over %zu)\n", std::sqrt(s2 / again.size()), again.size());
    }
    CK(hipDeviceSynchronize());
    CK(hipMemUnmap(va, slots * H));
    for (int i = 0; i < slots; ++i) CK(hipMemRelease(h[i]));
    CK(hipMemAddressFree(va, slots * H));
    return 0;
}

static int run_sets() {
    const size_t H = 512 * MiB;
    size_t free_b, total_b;
    CK(hipMemGetInfo(&free_b, &total_b));
    const int slots = (int)std::min<size_t>(560, (free_b - 4 * GiB) / H);      // all three ranks, if the device is otherwise empty
    const size_t n = (H - 64 * 1024) / 4;
    const unsigned nb = (unsigned)((n + 255) / 256);
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned, prop.location.type = hipMemLocationTypeDevice, prop.location.id = 0;
    hipMemAccessDesc acc = {};
    acc.location = prop.location, acc.flags = hipMemAccessFlagsProtReadWrite;
    std::vector<hipMemGenericAllocationHandle_t> h(slots);
    for (int i = 0; i < slots; ++i) CK(hipMemCreate(&h[i], H, &prop, 0));
    void *va;
    CK(hipMemAddressReserve(&va, slots * H, 2 * MiB, nullptr, 0));
    for (int i = 0; i < slots; ++i) CK(hipMemMap((char *)va + i * H, H, 0, h[i], 0));
    CK(hipMemSetAccess(va, slots * H, &acc, 1));
    char *base = (char *)va;
    k_fill<<<16384, 256>>>((float *)base, slots * H / 4, 7);
    CK(hipDeviceSynchronize());
    auto P = [&](int chunk, size_t phase = 0) { return (float *)(base + (size_t)chunk * H + phase); };
    // ranks by timing: the gradient window in the candidate against theta, m, v in quarter windows of one reference chunk
    const size_t nq = n / 4 - 16384;
    const unsigned nbq = (unsigned)((nq + 255) / 256);
    std::vector<int> rank(slots, -1), members[3];
    int found = 0;
    for (int ref = 0; ref >= 0 && found < 3;) {
        std::vector<double> r(slots, 0.0), sorted;
        for (int c = 0; c < slots; ++c)
            if (rank[c] < 0 && c != ref)
                r[c] = gbps([&] { k_slow<<<nbq, 64>>>(P(ref), P(ref, 128 * MiB + 32768), P(ref, 256 * MiB + 32768), P(c, 384 * MiB), nq); }, 28.0 * nq, 6),
                sorted.push_back(r[c]);
        rank[ref] = found;
        if (sorted.size() > 8) {
            // the reference's rank is the fast cluster: two-means on the rates; one cluster if the centres are within 2.5 %
            std::sort(sorted.begin(), sorted.end());
            double lo = sorted.front(), hi = sorted.back(), cut = 0;
            for (int it = 0; it < 10; ++it) {
                cut = 0.5 * (lo + hi);
                double sl = 0, sh = 0;
                size_t nl = 0, nh = 0;
                for (double y : sorted) (y <= cut ? (sl += y, ++nl) : (sh += y, ++nh));
                if (!nl || !nh) break;
                lo = sl / nl, hi = sh / nh;
            }
            cut = hi - lo > 0.025 * hi ? 0.5 * (lo + hi) : 0;
            printf("  reference chunk %d: %zu candidates, cluster centres %.0f / %.0f GB/s\n", ref, sorted.size(), lo, hi);
            for (int c = 0; c < slots; ++c)
                if (rank[c] < 0 && r[c] > cut) rank[c] = found;
        }
        ++found;
        // next reference: the slowest chunk still unlabelled, the one least likely to be a straggler of this rank
        ref = -1;
        for (int c = 0; c < slots; ++c)
            if (rank[c] < 0 && (ref < 0 || r[c] < r[ref])) ref = c;
    }
    for (int c = 0; c < slots; ++c)
        if (rank[c] >= 0) members[rank[c]].push_back(c);
    printf("%d chunks of 512 MiB; by rank: %zu, %zu, %zu\n", slots, members[0].size(), members[1].size(), members[2].size());
    if (members[0].size() < 16 || members[1].size() < 16 || members[2].size() < 16) {
        printf("fewer than three ranks with 16 chunks each: run this on an otherwise empty device\n");
        return 1;
    }
    struct Layout { const char *name; int rd[4]; int wr[3]; };       // rank of theta, m, v, g; rank of theta', m', v' (-1: in place)
    const Layout layouts[] = {
        {"in place, everything in rank A                     [the engine's default]", {0, 0, 0, 0}, {-1, -1, -1}},
        {"in place, theta A, m A, v B, gradient A", {0, 0, 1, 0}, {-1, -1, -1}},
        {"in place, theta A, m B, v C, gradient A", {0, 1, 2, 0}, {-1, -1, -1}},
        {"out of place, read A, write A A A", {0, 0, 0, 0}, {0, 0, 0}},
        {"out of place, read A, write B B B                  [alternating state]", {0, 0, 0, 0}, {1, 1, 1}},
        {"out of place, read A, write B C C", {0, 0, 0, 0}, {1, 2, 2}},
        {"out of place, read A, write A B C", {0, 0, 0, 0}, {0, 1, 2}},
        {"out of place, read B C C (gradient B), write A A A [what would have to follow]", {1, 2, 2, 1}, {0, 0, 0}},
    };
    unsigned x = 4711;
    auto rnd = [&](int m) { x = x * 1664525u + 1013904223u; return (int)((x >> 8) % (unsigned)m); };
    printf("slow-step shape (read theta, m, v, gradient; write three streams), 120 random choices of chunks per line, GB/s:\n");
    for (const Layout &L : layouts) {
        std::vector<double> r;
        for (int t = 0; t < 120; ++t) {
            int used[7], nu = 0, rd[4], wr[3] = {0, 0, 0};
            auto one = [&](int k) {
                int c;
                bool fresh;
                do {
                    c = members[k][rnd((int)members[k].size())], fresh = true;
                    for (int j = 0; j < nu; ++j) fresh = fresh && used[j] != c;
                } while (!fresh);
                return used[nu++] = c;
            };
            for (int k = 0; k < 4; ++k) rd[k] = one(L.rd[k]);
            if (L.wr[0] < 0) {
                r.push_back(gbps([&] { k_slow<<<nb, 64>>>(P(rd[0]), P(rd[1], 32768), P(rd[2], 32768), P(rd[3]), n); }, 28.0 * n, 3));
            } else {
                for (int k = 0; k < 3; ++k) wr[k] = one(L.wr[k]);
                r.push_back(gbps([&] { k_slow_oop<<<nb, 64>>>(P(rd[0]), P(rd[1], 32768), P(rd[2], 32768), P(rd[3]), P(wr[0]), P(wr[1], 32768),
                                                              P(wr[2], 32768), n); }, 28.0 * n, 3));
            }
        }
        double mean = 0;
        for (double y : r) mean += y;
        char what[128];
        snprintf(what, sizeof what, "%-82s mean %5.0f", L.name, mean / r.size());
        percentiles(r, what);
    }
    CK(hipDeviceSynchronize());
    CK(hipMemUnmap(va, slots * H));
    for (int i = 0; i < slots; ++i) CK(hipMemRelease(h[i]));
    CK(hipMemAddressFree(va, slots * H));
    return 0;
}

int main(int argc, char **argv) {
    const char *what = argc > 1 ? argv[1] : "";
    if (!strcmp(what, "shape")) return run_shape();
    if (!strcmp(what, "policy")) return run_policy();
    if (!strcmp(what, "phase")) return run_phase();
    if (!strcmp(what, "ranks")) return run_ranks();
    if (!strcmp(what, "bf16")) return run_bf16();
    if (!strcmp(what, "chunks")) return run_chunks();
    if (!strcmp(what, "sets")) return run_sets();
    printf("usage: hbm_probe shape | policy | phase | ranks | bf16 | chunks | sets\n");
    return 2;
}
