// Internal helpers shared by the LRQMM HIP kernels (gfx950 only).
// Compiled with -ffp-contract=off: a*b+c is never fused implicitly; every FMA
// in this library is written as fmaf()/fma() on purpose.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define LRQ_WAVE 64

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Quantizer parameters of one call (Eq. (quantA)): qmax as float, clamp range, rounding mode.
struct QuantParams {
    float qmaxf;   // 2^(bits-1) - 1
    float lo;      // -qmax - 1
    float hi;      // qmax
    int round_mode;
};

static inline QuantParams make_quant_params(int bits, int round_mode) {
    QuantParams q;
    int qm = (1 << (bits - 1)) - 1;
    q.qmaxf = (float)qm;
    q.lo = (float)(-qm - 1);
    q.hi = (float)qm;
    q.round_mode = round_mode;
    return q;
}

// lambda = fl32(qmax / amax), s = fl32(amax / qmax); zero group when amax < 1e-30.
__device__ __forceinline__ void make_scales(float amax, float qmaxf, float& lam, float& s) {
    if (amax >= 1e-30f) {
        lam = qmaxf / amax;
        s = amax / qmaxf;
    } else {
        lam = 0.0f;
        s = 0.0f;
    }
}

// code = clamp(round(fl32(lambda * x))) as a float holding an integer value.
__device__ __forceinline__ float quant_code(float x, float lam, const QuantParams& q) {
    float t = x * lam;
    float c = (q.round_mode == 0) ? floorf(t) : rintf(t);
    return fminf(fmaxf(c, q.lo), q.hi);
}

// The same residual with the rounding mode fixed at compile time (callers branch once on
// q.round_mode around a block of these instead of selecting per element).
template <int ROUND_MODE>
__device__ __forceinline__ float quant_residual_m(float x, float lam, float s, const QuantParams& q) {
    const float t = x * lam;
    const float c = ROUND_MODE == 0 ? floorf(t) : rintf(t);
    return fmaf(-fminf(fmaxf(c, q.lo), q.hi), s, x);
}

// residual x - code * s with a single rounding.
__device__ __forceinline__ float quant_residual(float x, float lam, float s, const QuantParams& q) {
    float c = quant_code(x, lam, q);
    return fmaf(-c, s, x);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// 16-byte global load of 4 consecutive floats when allowed, else guarded scalar loads.
// `k` is the first column, valid columns are [0, cols).  Rows out of range give zeros.
// The vector path is branch free (clamped address, then a select): a load under a branch
// makes the compiler wait for every outstanding load, which defeats software prefetching.
// It needs cols % 4 == 0, cols >= 4 and a valid row pointer even when row_ok is false.
template <bool VEC>
__device__ __forceinline__ float4 load4f(const float* __restrict__ rowp, int k, int cols, bool row_ok) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (VEC) {
        const int kc = min(k, cols - 4);
        const float4 t = *reinterpret_cast<const float4*>(rowp + kc);
        const bool ok = row_ok && k < cols;
        v.x = ok ? t.x : 0.f;
        v.y = ok ? t.y : 0.f;
        v.z = ok ? t.z : 0.f;
        v.w = ok ? t.w : 0.f;
    } else {
        if (!row_ok) return v;
        if (k + 0 < cols) v.x = rowp[k + 0];
        if (k + 1 < cols) v.y = rowp[k + 1];
        if (k + 2 < cols) v.z = rowp[k + 2];
        if (k + 3 < cols) v.w = rowp[k + 3];
    }
    return v;
}

// Branch-free float4 load from a vector padded to a multiple of 4: element k .. k+3 when
// k < n, zeros otherwise (n >= 4, n % 4 == 0 after padding).
__device__ __forceinline__ float4 load4_padded(const float* __restrict__ p, int k, int n) {
    const int kc = max(0, min(k, n - 4));
    const float4 t = *reinterpret_cast<const float4*>(p + kc);
    const bool ok = k < n;
    return make_float4(ok ? t.x : 0.f, ok ? t.y : 0.f, ok ? t.z : 0.f, ok ? t.w : 0.f);
}

// ---- float32 values as sums of bfloat16 planes (for the bf16 matrix cores) ----
// A float32 value is the exact sum of three bfloat16 planes (8 + 8 + 8 significant bits: round to nearest,
// subtract, repeat); products of such sums are evaluated plane by plane, each product exact, accumulated in
// float32 by the matrix core.
typedef __bf16 v8bf16 __attribute__((ext_vector_type(8)));
struct Planes3 {
    v8bf16 p1, p2, p3;
};
typedef __bf16 v2bf16 __attribute__((ext_vector_type(2)));
typedef float v2f32 __attribute__((ext_vector_type(2)));
// Two values per conversion instruction; a bfloat16 is the upper half of its float32, so the
// converted pair is widened again with a shift and a mask.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f32){a, b}, v2bf16));
}
// PL planes are formed (1, 2 or 3); the members beyond PL stay unset and must not be used.
template <int PL = 3>
__device__ __forceinline__ Planes3 split_planes(const float (&r)[8]) {
    uint32_t w1[4], w2[4], w3[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float a = r[2 * e], b = r[2 * e + 1];
        const uint32_t h = pack_bf16x2(a, b);
        w1[e] = h;
        if (PL >= 2) {
            const float ra = a - __uint_as_float(h << 16);              // exact
            const float rb = b - __uint_as_float(h & 0xffff0000u);
            const uint32_t m = pack_bf16x2(ra, rb);
            w2[e] = m;
            if (PL >= 3) {
                const float ra2 = ra - __uint_as_float(m << 16);            // exact
                const float rb2 = rb - __uint_as_float(m & 0xffff0000u);
                w3[e] = pack_bf16x2(ra2, rb2);
            }
        }
    }
    typedef uint32_t v4u32 __attribute__((ext_vector_type(4)));
    Planes3 o;
    o.p1 = __builtin_bit_cast(v8bf16, (v4u32){w1[0], w1[1], w1[2], w1[3]});
    if (PL >= 2) o.p2 = __builtin_bit_cast(v8bf16, (v4u32){w2[0], w2[1], w2[2], w2[3]});
    if (PL >= 3) o.p3 = __builtin_bit_cast(v8bf16, (v4u32){w3[0], w3[1], w3[2], w3[3]});
    return o;
}

#define LRQ_CHECK_LAUNCH()                                   \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return LRQMM_ERR_HIP; \
    } while (0)
