// Symmetric absmax quantization (paper: Background 2.2 Eq. (quantA); floor variant
// Methodology Eq. (get_ra2); Algorithm 2, quantization step).  HBM-streaming kernels: each
// input element is read from HBM once (the second touch of a row/tile hits L2).
#include "kernels.h"

// One wavefront per row: absmax by wave reduction, then codes with 4-byte packed stores.
// Second quantization level (complete residual compensation, Eq. (gemm_r_split)): when amax0 is
// given, the value that is quantized is the residual fl32(x - code0 * s0) of the first level, whose
// scales come from amax0 (the first level's maxima of the same groups).
__device__ __forceinline__ float4 first_level_residual(float4 v, float lam0, float s0, const QuantParams& q) {
    return make_float4(quant_residual(v.x, lam0, s0, q), quant_residual(v.y, lam0, s0, q),
                       quant_residual(v.z, lam0, s0, q), quant_residual(v.w, lam0, s0, q));
}

// mode (all row kernels): ROWS_FULL computes amax and codes; ROWS_AMAX_ONLY stops after amax;
// ROWS_GIVEN_AMAX reads amax[row] (written by an earlier launch) instead of the row's own maximum.
enum { ROWS_FULL = 0, ROWS_AMAX_ONLY = 1, ROWS_GIVEN_AMAX = 2 };
template <bool VEC>
__global__ __launch_bounds__(256) void quant_rows_kernel(const float* __restrict__ X, int ldx, int rows,
                                                         int cols, QuantParams q,
                                                         int8_t* __restrict__ codes,
                                                         float* __restrict__ amax, int mode,
                                                         const float* __restrict__ amax0) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= rows) return;
    const float* xp = X + (size_t)row * ldx;
    float lam0 = 0.f, s0 = 0.f;
    if (amax0) make_scales(amax0[row], q.qmaxf, lam0, s0);
    float m = 0.0f;
    if (mode == ROWS_GIVEN_AMAX) {
        m = amax[row];
    } else {
        for (int k = lane * 4; k < cols; k += 256) {
            float4 v = load4f<VEC>(xp, k, cols, true);
            if (amax0) v = first_level_residual(v, lam0, s0, q);
            m = fmaxf(fmaxf(m, fabsf(v.x)), fmaxf(fabsf(v.y), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
        m = wave_max(m);
        if (lane == 0) amax[row] = m;
        if (mode == ROWS_AMAX_ONLY) return;
    }
    float lam, s;
    make_scales(m, q.qmaxf, lam, s);
    int8_t* cp = codes + (size_t)row * cols;
    for (int k = lane * 4; k < cols; k += 256) {
        float4 v = load4f<VEC>(xp, k, cols, true);
        if (amax0) v = first_level_residual(v, lam0, s0, q);
        int c0 = (int)quant_code(v.x, lam, q), c1 = (int)quant_code(v.y, lam, q);
        int c2 = (int)quant_code(v.z, lam, q), c3 = (int)quant_code(v.w, lam, q);
        if (VEC) {
            uint32_t p = (uint32_t)(c0 & 0xff) | ((uint32_t)(c1 & 0xff) << 8) |
                         ((uint32_t)(c2 & 0xff) << 16) | ((uint32_t)(c3 & 0xff) << 24);
            *reinterpret_cast<uint32_t*>(cp + k) = p;
        } else {
            if (k + 0 < cols) cp[k + 0] = (int8_t)c0;
            if (k + 1 < cols) cp[k + 1] = (int8_t)c1;
            if (k + 2 < cols) cp[k + 2] = (int8_t)c2;
            if (k + 3 < cols) cp[k + 3] = (int8_t)c3;
        }
    }
}

// Single-read variant: the row is kept in registers between the absmax reduction and the
// code computation (NV float4 per thread, NV <= 16), so A is fetched from HBM once.  TPR threads
// cooperate on a row: 64 (one wavefront, cols <= 4096) or 256 (a workgroup, cols <= 16384).
template <bool VEC, int TPR, int NV>
__global__ __launch_bounds__(256) void quant_rows_cached_kernel(const float* __restrict__ X, int ldx, int rows,
                                                                int cols, QuantParams q,
                                                                int8_t* __restrict__ codes,
                                                                float* __restrict__ amax, int mode,
                                                                const float* __restrict__ amax0) {
    __shared__ float wmax[4];
    const int t = threadIdx.x % TPR;
    const int row = blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    const bool row_ok = row < rows;
    const float* xp = X + (size_t)(row_ok ? row : 0) * ldx;
    float4 v[NV];
    float m = 0.0f;
    float lam0 = 0.f, s0 = 0.f;
    if (amax0) make_scales(amax0[row_ok ? row : 0], q.qmaxf, lam0, s0);
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int k = (t + TPR * u) * 4;
        v[u] = load4f<VEC>(xp, k, cols, row_ok);
        if (amax0) v[u] = first_level_residual(v[u], lam0, s0, q);     // zeros stay zeros
        m = fmaxf(fmaxf(m, fabsf(v[u].x)), fmaxf(fabsf(v[u].y), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
    }
    m = wave_max(m);
    if (TPR == 256) {
        if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
        __syncthreads();
        m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    }
    if (!row_ok) return;
    if (mode == ROWS_GIVEN_AMAX) m = amax[row];
    else if (t == 0) amax[row] = m;
    if (mode == ROWS_AMAX_ONLY) return;
    float lam, s;
    make_scales(m, q.qmaxf, lam, s);
    int8_t* cp = codes + (size_t)row * cols;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int k = (t + TPR * u) * 4;
        if (k >= cols) continue;
        const int c0 = (int)quant_code(v[u].x, lam, q), c1 = (int)quant_code(v[u].y, lam, q);
        const int c2 = (int)quant_code(v[u].z, lam, q), c3 = (int)quant_code(v[u].w, lam, q);
        if (VEC) {
            const uint32_t p = (uint32_t)(c0 & 0xff) | ((uint32_t)(c1 & 0xff) << 8) |
                               ((uint32_t)(c2 & 0xff) << 16) | ((uint32_t)(c3 & 0xff) << 24);
            *reinterpret_cast<uint32_t*>(cp + k) = p;
        } else {
            if (k + 0 < cols) cp[k + 0] = (int8_t)c0;
            if (k + 1 < cols) cp[k + 1] = (int8_t)c1;
            if (k + 2 < cols) cp[k + 2] = (int8_t)c2;
            if (k + 3 < cols) cp[k + 3] = (int8_t)c3;
        }
    }
}

__global__ void fill_u32_kernel(uint32_t* p, int n, uint32_t v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Column absmax of a row-major matrix.  A workgroup takes 256 columns and a slab of rows: a wave reads 1 KB
// of one row per instruction (each lane 4 adjacent columns), the four waves take every fourth row of the slab,
// 16 row loads in flight per lane; the waves' maxima are merged through LDS and the slabs with one unsigned
// atomic max per column on the bit pattern of |x| (exact and order independent for x >= 0).
#ifndef LRQ_ABSMAX_WGS
#define LRQ_ABSMAX_WGS 1024     // workgroups aimed at (more slabs: more atomics per column)
#endif
template <bool VEC>
__global__ __launch_bounds__(256) void absmax_cols_kernel(const float* __restrict__ X, int ldx, int rows,
                                                          int cols, int rows_per_block,
                                                          uint32_t* __restrict__ amax_bits, QuantParams q,
                                                          const float* __restrict__ amax0) {
    __shared__ float4 red[4][64];
    const int quad = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int c = (blockIdx.x * 64 + quad) * 4;
    float lam0[4] = {0.f, 0.f, 0.f, 0.f}, s0[4] = {0.f, 0.f, 0.f, 0.f};
    if (amax0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) make_scales(c + t < cols ? amax0[c + t] : 0.f, q.qmaxf, lam0[t], s0[t]);
    }
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(rows, r0 + rows_per_block);
    float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int rb = r0 + rg; rb < r1; rb += 64) {     // rows clamped into the slab: max is idempotent
        float4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = load4f<VEC>(X + (size_t)min(rb + 4 * u, r1 - 1) * ldx, c, cols, true);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (amax0)
                v[u] = make_float4(quant_residual(v[u].x, lam0[0], s0[0], q), quant_residual(v[u].y, lam0[1], s0[1], q),
                                   quant_residual(v[u].z, lam0[2], s0[2], q), quant_residual(v[u].w, lam0[3], s0[3], q));
            m.x = fmaxf(m.x, fabsf(v[u].x));
            m.y = fmaxf(m.y, fabsf(v[u].y));
            m.z = fmaxf(m.z, fabsf(v[u].z));
            m.w = fmaxf(m.w, fabsf(v[u].w));
        }
    }
    red[rg][quad] = m;
    __syncthreads();
    if (rg != 0 || c >= cols) return;
#pragma unroll
    for (int g = 1; g < 4; ++g) {
        const float4 o = red[g][quad];
        m.x = fmaxf(m.x, o.x); m.y = fmaxf(m.y, o.y); m.z = fmaxf(m.z, o.z); m.w = fmaxf(m.w, o.w);
    }
    if (c + 0 < cols) atomicMax(amax_bits + c + 0, __float_as_uint(m.x));
    if (c + 1 < cols) atomicMax(amax_bits + c + 1, __float_as_uint(m.y));
    if (c + 2 < cols) atomicMax(amax_bits + c + 2, __float_as_uint(m.z));
    if (c + 3 < cols) atomicMax(amax_bits + c + 3, __float_as_uint(m.w));
}

// Quantize a 64(k) x 64(n) tile with per-column scales and store it transposed
// (codesT is cols x rows, contiguous along the original row index k).
template <bool VEC, bool VECOUT>
__global__ __launch_bounds__(256) void quant_cols_kernel(const float* __restrict__ X, int ldx, int rows,
                                                         int cols, const float* __restrict__ amax,
                                                         QuantParams q,
                                                         int8_t* __restrict__ codesT,
                                                         const float* __restrict__ amax0,
                                                         float* __restrict__ lam_out,
                                                         float* __restrict__ s_out, int npad) {
    __shared__ __align__(16) int8_t tile[64][80];
    const int n0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n = n0 + tx * 4;
    float lam[4], stp[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        float a = (n + t < cols) ? amax[n + t] : 0.0f;
        make_scales(a, q.qmaxf, lam[t], stp[t]);
    }
    // the step vectors of this operand, zero padded to npad entries, for the kernels that follow
    if (lam_out && blockIdx.y == 0 && ty == 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (n + t < npad) {
                lam_out[n + t] = lam[t];     // zero beyond cols (amax read as 0 there)
                s_out[n + t] = stp[t];
            }
    }
    float lam0[4] = {0.f, 0.f, 0.f, 0.f}, s0[4] = {0.f, 0.f, 0.f, 0.f};
    if (amax0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) make_scales(n + t < cols ? amax0[n + t] : 0.f, q.qmaxf, lam0[t], s0[t]);
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int kl = ty + 16 * rr;
        const int k = k0 + kl;
        float4 v = load4f<VEC>(X + (size_t)min(k, rows - 1) * ldx, n, cols, k < rows);
        if (amax0)
            v = make_float4(quant_residual(v.x, lam0[0], s0[0], q), quant_residual(v.y, lam0[1], s0[1], q),
                            quant_residual(v.z, lam0[2], s0[2], q), quant_residual(v.w, lam0[3], s0[3], q));
        tile[tx * 4 + 0][kl] = (int8_t)(int)quant_code(v.x, lam[0], q);
        tile[tx * 4 + 1][kl] = (int8_t)(int)quant_code(v.y, lam[1], q);
        tile[tx * 4 + 2][kl] = (int8_t)(int)quant_code(v.z, lam[2], q);
        tile[tx * 4 + 3][kl] = (int8_t)(int)quant_code(v.w, lam[3], q);
    }
    __syncthreads();
    const int nl = threadIdx.x >> 2, chunk = threadIdx.x & 3;
    const int nn = n0 + nl;
    if (nn >= cols) return;
    const int kb = k0 + chunk * 16;
    int8_t* dst = codesT + (size_t)nn * rows + kb;
    if (VECOUT) {
        if (kb < rows) *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(&tile[nl][chunk * 16]);
    } else {
#pragma unroll
        for (int b = 0; b < 16; ++b)
            if (kb + b < rows) dst[b] = tile[nl][chunk * 16 + b];
    }
}

__global__ void scales_kernel(const float* __restrict__ amax, int n, int npad, float qmaxf,
                              float* __restrict__ lam, float* __restrict__ s) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= npad) return;
    float l = 0.0f, st = 0.0f;
    if (i < n) make_scales(amax[i], qmaxf, l, st);
    lam[i] = l;
    s[i] = st;
}

// One scale for the whole matrix (the paper's own Eq. (quantA)): every entry of amax[n] is
// replaced by the maximum of all of them.  One workgroup; max is exact and order independent.
__global__ __launch_bounds__(1024) void tensor_max_kernel(float* __restrict__ amax, int n) {
    __shared__ float wm[16];
    float m = 0.0f;
    for (int i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, amax[i]);
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
    __syncthreads();
    m = wm[0];
#pragma unroll
    for (int w = 1; w < 16; ++w) m = fmaxf(m, wm[w]);
    for (int i = threadIdx.x; i < n; i += 1024) amax[i] = m;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static int rows_launch(const float* X, int ldx, int rows, int cols, QuantParams q, int8_t* codes, float* amax,
                       int mode, const float* amax0, hipStream_t st);

int launch_quantize_rows(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor,
                         const float* amax0, int8_t* codes, float* amax, hipStream_t st) {
    if (!per_tensor) return rows_launch(X, ldx, rows, cols, q, codes, amax, ROWS_FULL, amax0, st);
    // one scale per matrix: row maxima, their maximum broadcast to every row, then the codes
    int rc = rows_launch(X, ldx, rows, cols, q, codes, amax, ROWS_AMAX_ONLY, amax0, st);
    if (rc != LRQMM_OK) return rc;
    hipLaunchKernelGGL(tensor_max_kernel, dim3(1), dim3(1024), 0, st, amax, rows);
    LRQ_CHECK_LAUNCH();
    return rows_launch(X, ldx, rows, cols, q, codes, amax, ROWS_GIVEN_AMAX, amax0, st);
}

static int rows_launch(const float* X, int ldx, int rows, int cols, QuantParams q, int8_t* codes, float* amax,
                       int mode, const float* amax0, hipStream_t st) {
    const bool vec = (cols % 4 == 0) && (ldx % 4 == 0) && aligned16(X) && (((uintptr_t)codes & 3) == 0);
    if (cols <= 256 * 4 * 16) {
        // Row cached in registers: one wavefront per row up to 4096 columns, else one workgroup.
        const bool wave = cols <= 64 * 4 * 16;
        const int per = wave ? 256 : 1024;
        const int need = ceil_div(cols, per);
        dim3 grid(wave ? ceil_div(rows, 4) : rows);
#define LRQ_QR(V, T, N) hipLaunchKernelGGL((quant_rows_cached_kernel<V, T, N>), grid, dim3(256), 0, st, X, ldx, rows, cols, q, codes, amax, mode, amax0)
#define LRQ_QR_NV(V, T) do { if (need <= 1) LRQ_QR(V, T, 1); else if (need <= 2) LRQ_QR(V, T, 2); \
        else if (need <= 4) LRQ_QR(V, T, 4); else if (need <= 8) LRQ_QR(V, T, 8); else LRQ_QR(V, T, 16); } while (0)
        if (wave) { if (vec) LRQ_QR_NV(true, 64); else LRQ_QR_NV(false, 64); }
        else      { if (vec) LRQ_QR_NV(true, 256); else LRQ_QR_NV(false, 256); }
#undef LRQ_QR_NV
#undef LRQ_QR
    } else {                              // very long rows: two passes over the row
        dim3 grid(ceil_div(rows, 4));
        if (vec) hipLaunchKernelGGL(quant_rows_kernel<true>, grid, dim3(256), 0, st, X, ldx, rows, cols, q, codes, amax, mode, amax0);
        else     hipLaunchKernelGGL(quant_rows_kernel<false>, grid, dim3(256), 0, st, X, ldx, rows, cols, q, codes, amax, mode, amax0);
    }
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

static int absmax_cols_launch(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor,
                              const float* amax0, float* amax, hipStream_t st, bool amax_zeroed) {
    const bool vec = (cols % 4 == 0) && (ldx % 4 == 0) && aligned16(X);
    if (!amax_zeroed) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(ceil_div(cols, 256)), dim3(256), 0, st,
                           reinterpret_cast<uint32_t*>(amax), cols, 0u);
        LRQ_CHECK_LAUNCH();
    }
    // enough row slabs to fill the chip, at least 64 rows each (one batch of loads per lane)
    const int col_blocks = ceil_div(cols, 256);
    int slabs = max(1, min(ceil_div(rows, 64), ceil_div(LRQ_ABSMAX_WGS, col_blocks)));
    const int rows_per_block = ceil_div(rows, slabs);
    slabs = ceil_div(rows, rows_per_block);
    dim3 g1(col_blocks, slabs);
    if (vec)
        hipLaunchKernelGGL(absmax_cols_kernel<true>, g1, dim3(256), 0, st, X, ldx, rows, cols, rows_per_block,
                           reinterpret_cast<uint32_t*>(amax), q, amax0);
    else
        hipLaunchKernelGGL(absmax_cols_kernel<false>, g1, dim3(256), 0, st, X, ldx, rows, cols, rows_per_block,
                           reinterpret_cast<uint32_t*>(amax), q, amax0);
    LRQ_CHECK_LAUNCH();
    if (per_tensor) {
        hipLaunchKernelGGL(tensor_max_kernel, dim3(1), dim3(1024), 0, st, amax, cols);
        LRQ_CHECK_LAUNCH();
    }
    return LRQMM_OK;
}

int launch_absmax_cols(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor, float* amax,
                       hipStream_t st, bool amax_zeroed) {
    return absmax_cols_launch(X, ldx, rows, cols, q, per_tensor, nullptr, amax, st, amax_zeroed);
}

int launch_absmax_rows(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor, float* amax,
                       hipStream_t st) {
    int rc = rows_launch(X, ldx, rows, cols, q, nullptr, amax, ROWS_AMAX_ONLY, nullptr, st);
    if (rc != LRQMM_OK || !per_tensor) return rc;
    hipLaunchKernelGGL(tensor_max_kernel, dim3(1), dim3(1024), 0, st, amax, rows);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_quantize_cols(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor,
                         const float* amax0, int8_t* codesT, float* amax, hipStream_t st, bool amax_zeroed,
                         float* lam_out, float* s_out) {
    const bool vec = (cols % 4 == 0) && (ldx % 4 == 0) && aligned16(X);
    const bool vecout = (rows % 16 == 0) && aligned16(codesT);
    const int npad = (cols + 3) / 4 * 4;
    const int rc = absmax_cols_launch(X, ldx, rows, cols, q, per_tensor, amax0, amax, st, amax_zeroed);
    if (rc != LRQMM_OK) return rc;
    dim3 g2(ceil_div(cols, 64), ceil_div(rows, 64));
    if (vec && vecout)
        hipLaunchKernelGGL((quant_cols_kernel<true, true>), g2, dim3(256), 0, st, X, ldx, rows, cols, amax, q, codesT, amax0, lam_out, s_out, npad);
    else if (vec)
        hipLaunchKernelGGL((quant_cols_kernel<true, false>), g2, dim3(256), 0, st, X, ldx, rows, cols, amax, q, codesT, amax0, lam_out, s_out, npad);
    else if (vecout)
        hipLaunchKernelGGL((quant_cols_kernel<false, true>), g2, dim3(256), 0, st, X, ldx, rows, cols, amax, q, codesT, amax0, lam_out, s_out, npad);
    else
        hipLaunchKernelGGL((quant_cols_kernel<false, false>), g2, dim3(256), 0, st, X, ldx, rows, cols, amax, q, codesT, amax0, lam_out, s_out, npad);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_tick(uint32_t* word, hipStream_t st) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, st, word, 1, 0u);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_scales(const float* amax, int n, int npad, float qmaxf, float* lam, float* s,
                  hipStream_t st) {
    hipLaunchKernelGGL(scales_kernel, dim3(ceil_div(npad, 256)), dim3(256), 0, st, amax, n, npad, qmaxf, lam, s);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
