// Counter-based Gaussian test matrix for the randomized range finder (paper:
// Background 2.1, stage 1 of the RSVD description; the sampling itself is left to
// the cited literature -- this library draws i.i.d. N(0,1) entries).
//
// Element (i, j) depends only on (seed, stream, i, j).  All floating-point steps
// are exactly rounded IEEE float64 operations (+ - * /) in a fixed order, with
// contraction disabled, so the float32 result is reproducible bit for bit by any
// implementation that follows the same sequence.
#include "kernels.h"

#pragma clang fp contract(off)

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// ln(k / 2^24), k in [1, 2^24]: k = m 2^e, m in [sqrt(1/2), sqrt(2)),
// ln m = 2 atanh((m-1)/(m+1)) through s^21.
__device__ static double ln_ratio24(uint32_t k) {
    int e = 32 - __clz((int)k);
    double m = ldexp((double)k, -e);   // [0.5, 1), exact
    if (m < 0.7071067811865476) {
        m = m * 2.0;
        e -= 1;
    }
    const double s = (m - 1.0) / (m + 1.0);
    const double s2 = s * s;
    double p = 1.0 / 21.0;
    p = p * s2 + 1.0 / 19.0;
    p = p * s2 + 1.0 / 17.0;
    p = p * s2 + 1.0 / 15.0;
    p = p * s2 + 1.0 / 13.0;
    p = p * s2 + 1.0 / 11.0;
    p = p * s2 + 1.0 / 9.0;
    p = p * s2 + 1.0 / 7.0;
    p = p * s2 + 1.0 / 5.0;
    p = p * s2 + 1.0 / 3.0;
    p = p * s2 + 1.0;
    const double lnm = (2.0 * s) * p;
    return lnm + (double)(e - 24) * 0.6931471805599453;
}

// sqrt(x) for x >= 0: two Heron steps from the correctly rounded float32 root.
__device__ static double heron_sqrt(double x) {
    const double y0 = (double)__fsqrt_rn((float)x);
    if (!(y0 > 0.0)) return 0.0;
    const double y1 = 0.5 * (y0 + x / y0);
    return 0.5 * (y1 + x / y1);
}

// sin and cos on [0, pi/4]: Taylor through x^17 / x^16.
__device__ static void sincos_small(double x, double& sn, double& cs) {
    const double x2 = x * x;
    double ps = 1.0 / 355687428096000.0;
    ps = ps * x2 + (-1.0 / 1307674368000.0);
    ps = ps * x2 + 1.0 / 6227020800.0;
    ps = ps * x2 + (-1.0 / 39916800.0);
    ps = ps * x2 + 1.0 / 362880.0;
    ps = ps * x2 + (-1.0 / 5040.0);
    ps = ps * x2 + 1.0 / 120.0;
    ps = ps * x2 + (-1.0 / 6.0);
    ps = ps * x2 + 1.0;
    double pc = 1.0 / 20922789888000.0;
    pc = pc * x2 + (-1.0 / 87178291200.0);
    pc = pc * x2 + 1.0 / 479001600.0;
    pc = pc * x2 + (-1.0 / 3628800.0);
    pc = pc * x2 + 1.0 / 40320.0;
    pc = pc * x2 + (-1.0 / 720.0);
    pc = pc * x2 + 1.0 / 24.0;
    pc = pc * x2 + (-1.0 / 2.0);
    pc = pc * x2 + 1.0;
    sn = x * ps;
    cs = pc;
}

__device__ static float gaussian_at(uint64_t key, uint32_t i, uint32_t j) {
    const uint64_t ctr = ((uint64_t)i << 32) | (uint64_t)j;
    const uint64_t h = mix64(ctr + key);
    const uint32_t k1 = (uint32_t)(h >> 40) + 1u;          // 1 .. 2^24
    const uint32_t k2 = (uint32_t)(h >> 16) & 0xFFFFFFu;   // 0 .. 2^24-1
    const double rad = heron_sqrt(-2.0 * ln_ratio24(k1));
    const uint32_t octant = k2 >> 21;
    const uint32_t rem = k2 & 0x1FFFFFu;
    const uint32_t r = (octant & 1u) ? (0x200000u - rem) : rem;
    const double phi = 6.283185307179586 * ((double)r / 16777216.0);
    double sn, cs;
    sincos_small(phi, sn, cs);
    const bool use_sin = (octant == 1u) | (octant == 2u) | (octant == 5u) | (octant == 6u);
    const bool neg = (octant >= 2u) & (octant <= 5u);
    double t = use_sin ? sn : cs;
    t = neg ? -t : t;
    return (float)(rad * t);
}

// Workgroups [0, nb_sketch) fill the sketch; the following ones (if any) derive the step
// vectors lambda = qmax/amax, s = amax/qmax of the operand the sketch is for, so that the
// preparation of a factorization is one launch.
__global__ void fill_sketch_kernel(uint64_t key, int rows, int cols, int ld, float* __restrict__ omega,
                                   int nb_sketch, const float* __restrict__ amax, int n, int npad, float qmaxf,
                                   float* __restrict__ lam, float* __restrict__ s,
                                   uint32_t* __restrict__ zero_words, int zero_n) {
    if ((int)blockIdx.x >= nb_sketch) {
        const int i = ((int)blockIdx.x - nb_sketch) * blockDim.x + threadIdx.x;
        if (zero_words) {       // the trailing workgroups clear words instead (column maxima before their merge)
            if (i < zero_n) zero_words[i] = 0u;
            return;
        }
        if (i >= npad) return;
        float l = 0.0f, st = 0.0f;
        if (i < n) make_scales(amax[i], qmaxf, l, st);
        lam[i] = l;
        s[i] = st;
        return;
    }
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)rows * ld;
    if (idx >= total) return;
    const uint32_t i = (uint32_t)(idx / ld), j = (uint32_t)(idx % ld);
    omega[idx] = (j < (uint32_t)cols) ? gaussian_at(key, i, j) : 0.0f;
}

__global__ void pad_copy_kernel(const float* __restrict__ src, int rows, int cols, int ld,
                                float* __restrict__ dst) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)rows * ld;
    if (idx >= total) return;
    const int i = (int)(idx / ld), j = (int)(idx % ld);
    dst[idx] = (j < cols) ? src[(size_t)i * cols + j] : 0.0f;
}

static uint64_t host_mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int launch_fill_sketch(uint64_t seed, int stream_id, int rows, int cols, int ld, float* omega,
                       hipStream_t st) {
    return launch_sketch_and_scales(seed, stream_id, rows, cols, ld, omega, nullptr, 0, 0, 0.f, nullptr, nullptr,
                                    st);
}

int launch_sketch_and_scales(uint64_t seed, int stream_id, int rows, int cols, int ld, float* omega,
                             const float* amax, int n, int npad, float qmaxf, float* lam, float* s,
                             hipStream_t st) {
    const uint64_t key = host_mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(stream_id + 1));
    const size_t total = (size_t)rows * ld;
    const int nb_sketch = (int)((total + 255) / 256), nb_scale = amax ? (npad + 255) / 256 : 0;
    if (nb_sketch + nb_scale == 0) return LRQMM_OK;
    hipLaunchKernelGGL(fill_sketch_kernel, dim3(nb_sketch + nb_scale), dim3(256), 0, st, key, rows, cols, ld,
                       omega, nb_sketch, amax, n, npad, qmaxf, lam, s, nullptr, 0);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_sketch_and_zero(uint64_t seed, int stream_id, int rows, int cols, int ld, float* omega,
                           uint32_t* zero_words, int zero_n, hipStream_t st) {
    const uint64_t key = host_mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(stream_id + 1));
    const size_t total = (size_t)rows * ld;
    const int nb_sketch = (int)((total + 255) / 256), nb_zero = (zero_n + 255) / 256;
    if (nb_sketch + nb_zero == 0) return LRQMM_OK;
    hipLaunchKernelGGL(fill_sketch_kernel, dim3(nb_sketch + nb_zero), dim3(256), 0, st, key, rows, cols, ld, omega,
                       nb_sketch, nullptr, 0, 0, 0.f, nullptr, nullptr, zero_words, zero_n);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_pad_copy(const float* src, int rows, int cols, int ld, float* dst, hipStream_t st) {
    const size_t total = (size_t)rows * ld;
    if (total == 0) return LRQMM_OK;
    hipLaunchKernelGGL(pad_copy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, rows,
                       cols, ld, dst);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
