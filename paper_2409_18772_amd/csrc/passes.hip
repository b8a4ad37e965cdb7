// Streaming products with the quantization residual R = X - Dequant(Quant(X))
// (paper: Algorithm 2, dequantization and residual steps, for R; Background 2.1 / Algorithm 1 for the
// products R.Omega, R^T Q, R Z, Q^T R of the randomized range finder), and the
// code-matrix products in the compensation terms of Algorithm 2 (A~ W and V^T B~).
//
// R is never stored: each pass re-reads the float32 operand once from HBM and
// regenerates the residual in registers from the per-group scales.  The
// tall-skinny contraction runs on the fp32 matrix cores (v_mfma_f32_16x16x4_f32);
// since the reduction index may be visited in any order, each lane loads 16
// contiguous bytes and the MFMA k-index is permuted to match.
//
// MFMA 16x16x4 f32 operand layout (lane l): A[i = l%16][k = l/16],
// B[k = l/16][j = l%16], D[i = 4*(l/16)+v][j = l%16] for v = 0..3.
#include <type_traits>
#include "kernels.h"

#define KCHUNK 128   // reduction elements staged per LDS step in the N-type kernels
#define KSUB (KCHUNK / 16)   // float4 loads per lane per chunk

__device__ __forceinline__ v4f mfma16(float a, float b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Register image of one thread's share of W[k0 .. k0+KC)[0..LP) (row-major, ld = LP).
template <int NT, int KC = KCHUNK>
struct WStage {
    static constexpr int LP = NT * 16;
    static constexpr int N4 = KC * LP / 4 / 256;   // float4 per thread (LP multiple of 16)
    float4 v[N4];
    __device__ __forceinline__ void load(const float* __restrict__ W, int k0, int kend) {
#pragma unroll
        for (int u = 0; u < N4; ++u) {
            const int e = (threadIdx.x + 256 * u) * 4;
            const int kk = e / LP, n = e % LP;
            const int kr = min(k0 + kk, kend - 1);          // branch free: clamp, then select
            const float4 t = *reinterpret_cast<const float4*>(W + (size_t)kr * LP + n);
            const bool ok = k0 + kk < kend;
            v[u] = make_float4(ok ? t.x : 0.f, ok ? t.y : 0.f, ok ? t.z : 0.f, ok ? t.w : 0.f);
        }
    }
    __device__ __forceinline__ void store(float* __restrict__ wl) const {   // LDS row stride LP+4
#pragma unroll
        for (int u = 0; u < N4; ++u) {
            const int e = (threadIdx.x + 256 * u) * 4;
            const int kk = e / LP, n = e % LP;
            *reinterpret_cast<float4*>(wl + kk * (LP + 4) + n) = v[u];
        }
    }
};

// Quantization fused into the first residual product (the sketch pass): with the group maxima known, one
// read of the operand yields both its codes and Y = R.Omega.  amax: the group maxima (rows of X for AXIS 0,
// columns for AXIS 1); lam_out / s_out: the step vectors lambda = qmax/amax, s = amax/qmax that the later
// passes read; codes: rows x cols row-major (AXIS 0) or transposed, cols x rows (AXIS 1).  Guard-free shapes
// only: rows a multiple of 64 besides the FULLK conditions, 16-byte aligned codes.
struct QOut {
    const float* amax;
    float* lam_out;
    float* s_out;
    int8_t* codes;
};

// ---------------------------------------------------------------------------
// N-type: partial[split][rows][LP] = R[:, k-range] . W[k-range, :]
// grid (ceil(rows/64), splits); 4 waves x 16 rows.  Per KCHUNK columns: the W chunk goes
// through double-buffered LDS, and both the next chunk of X and of W are already in
// flight (in registers) while the matrix cores work on the current one.
// ---------------------------------------------------------------------------
template <int NT, int AXIS, bool VEC>
__global__ __launch_bounds__(256) void resid_mul_n_kernel(
    const float* __restrict__ X, int ldx, int rows, int cols, const float* __restrict__ lam,
    const float* __restrict__ sc, QuantParams q, const float* __restrict__ W, int chunk,
    float* __restrict__ partial, QOut) {
    constexpr int LP = NT * 16;
    // wide sketches stage 64-deep chunks: 128 x (LP + 4) floats twice would leave one workgroup per CU
    constexpr int KC = NT <= 3 ? KCHUNK : KCHUNK / 2;
    constexpr int KS = KC / 16;          // float4 loads per lane per chunk
    __shared__ __align__(16) float wl[2][KC * (LP + 4)];
    __shared__ __align__(16) float sl[2][2 * KC];   // per-column lambda | step of the chunk (AXIS 1)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int row = blockIdx.x * 64 + wave * 16 + r;
    const bool row_ok = row < rows;
    const float* xp = X + (size_t)(row_ok ? row : 0) * ldx;
    const int kb = blockIdx.y * chunk;
    const int ke = min(cols, kb + chunk);
    float lam_r = 0.f, s_r = 0.f;
    if (AXIS == 0 && row_ok) {
        lam_r = lam[row];
        s_r = sc[row];
    }
    v4f acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = (v4f){0.f, 0.f, 0.f, 0.f};

    float4 xr[KS];
    float scale_reg = 0.f;     // this thread's element of the chunk's lambda (t < 128) or step vector
    WStage<NT, KC> ws;
    auto load_x = [&](int k0) {
#pragma unroll
        for (int j = 0; j < KS; ++j) xr[j] = load4f<VEC>(xp, k0 + 16 * j + 4 * g, ke, row_ok);
        if (AXIS == 1) {
            const int t = threadIdx.x & (KC - 1);
            const int kc = min(k0 + t, ke - 1);
            const float v = ((threadIdx.x & KC) == 0) ? lam[kc] : sc[kc];
            scale_reg = (k0 + t < ke) ? v : 0.f;
        }
    };
    if (kb < ke) {
        load_x(kb);
        ws.load(W, kb, ke);
    }
    int buf = 0;
    for (int k0 = kb; k0 < ke; k0 += KC, buf ^= 1) {
        ws.store(wl[buf]);
        if (AXIS == 1 && threadIdx.x < 2 * KC) sl[buf][threadIdx.x] = scale_reg;
        __syncthreads();             // wl[buf], sl[buf] complete; the other buffers no longer read
        float res[KS][4];
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            float4 l4, s4;
            if (AXIS == 0) {
                l4 = make_float4(lam_r, lam_r, lam_r, lam_r);
                s4 = make_float4(s_r, s_r, s_r, s_r);
            } else {
                l4 = *reinterpret_cast<const float4*>(&sl[buf][16 * j + 4 * g]);
                s4 = *reinterpret_cast<const float4*>(&sl[buf][KC + 16 * j + 4 * g]);
            }
            res[j][0] = quant_residual(xr[j].x, l4.x, s4.x, q);
            res[j][1] = quant_residual(xr[j].y, l4.y, s4.y, q);
            res[j][2] = quant_residual(xr[j].z, l4.z, s4.z, q);
            res[j][3] = quant_residual(xr[j].w, l4.w, s4.w, q);
        }
        if (k0 + KC < ke) {      // next chunk's loads fly during this chunk's MFMAs
            load_x(k0 + KC);
            ws.load(W, k0 + KC, ke);
        }
        const float* wb = wl[buf];
#pragma unroll
        for (int j = 0; j < KS; ++j) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* wrow = wb + (16 * j + 4 * g + t) * (LP + 4) + r;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma16(res[j][t], wrow[16 * nt], acc[nt]);
            }
        }
    }
    float* out = partial + (size_t)blockIdx.y * rows * LP;
    const int orow0 = blockIdx.x * 64 + wave * 16 + 4 * g;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (orow0 + v < rows) out[(size_t)(orow0 + v) * LP + 16 * nt + r] = acc[nt][v];
}

template <int ROUND_MODE>
__device__ __forceinline__ float quant_code_residual(float x, float lam, float s, const QuantParams& q, float& code) {
    const float t = x * lam;
    const float c = ROUND_MODE == 0 ? floorf(t) : rintf(t);
    code = fminf(fmaxf(c, q.lo), q.hi);
    return fmaf(-code, s, x);
}

// ---------------------------------------------------------------------------
// Row quantization (Eq. (quantA), one scale per row of A) and the sketch product Y = R.Omega (Algorithm 1, the
// sample matrix) from ONE read of the operand, for short rows (cols <= 576, a multiple of 16) and sketches
// padded to 16 columns.  A tile is 16 rows; workgroups of 8 waves are persistent, take a contiguous run of
// tiles, and load tile i+1 into a second register set while tile i is worked on.
//   * Wave w reads rows 2w and 2w+1 of the tile, adjacent lanes adjacent 16-byte pieces (NV float4 per lane), so
//     global loads and the code stores are fully coalesced and a row's maximum is a reduction inside one wave.
//   * The residuals go to LDS as a 16-row tile (row stride = 4 mod 64 floats: the 64 lanes of a matrix-core operand
//     read 64 different banks).  For the product the waves split the reduction: wave w always takes the same
//     columns, so its sketch operands stay in registers (4 NV values) for the life of the workgroup.
//   * The eight partial products of a tile meet in LDS and are added in the order of the waves, so the result
//     does not depend on the launch.  Two barriers per tile.
//   * A finished 16 x 16 tile of Y stays in LDS until the next barrier, where threads 0-255 add its Y^T Y to the
//     workgroup's float64 Gram matrix (also in LDS); at the end each workgroup leaves gpart[block][16][16], which
//     is what the orthonormalization needs next: no separate pass over Y forms it.
// amax, lam_out, s_out and the codes carry the bits the separate quantization kernel writes.
// ---------------------------------------------------------------------------
template <int NS>     // matrix-core steps (of 4 columns) per wave: ceil(cols / 32)
__global__ __launch_bounds__(512, 4) void quant_sketch_rows_kernel(
    const float* __restrict__ X, int ldx, int rows, int cols, QuantParams q, const float* __restrict__ W,
    float* __restrict__ Y, double* __restrict__ gpart, float* __restrict__ amax, float* __restrict__ lam_out,
    float* __restrict__ s_out, int8_t* __restrict__ codes) {
    constexpr int NV = (NS + 3) / 4;                     // 16-byte pieces per lane: ceil(cols / 128)
    extern __shared__ __align__(16) float rt[];          // residual tile: 16 rows of ldr floats
    __shared__ float pacc[8][256];
    __shared__ float yt[16][17];                         // the last finished tile of Y (rows past the end: zeros)
    __shared__ double gl[256];                           // the workgroup's Y^T Y so far, entry (t / 16, t % 16) by thread t
    if (threadIdx.x < 256) gl[threadIdx.x] = 0.0;        // (kept in LDS: no register lives across the tile loop for it)
    auto gram_tile = [&] {
        if (threadIdx.x < 256) {
            const int ga = threadIdx.x >> 4, gb = threadIdx.x & 15;
            double gacc = gl[threadIdx.x];
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) gacc = fma((double)yt[rr][ga], (double)yt[rr][gb], gacc);
            gl[threadIdx.x] = gacc;
        }
    };
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int cpr = cols >> 2;                           // 16-byte pieces, and steps, per row
    const int ldr = cols + ((68 - (cols & 63)) & 63);
    const int spw = (cpr + 7) >> 3;                      // steps per wave (= NS)
    const int s0 = min(cpr, wave * spw), s1 = min(cpr, s0 + spw);
    const int ntiles = (rows + 15) >> 4;
    const int t0 = (int)((long long)blockIdx.x * ntiles / gridDim.x);
    const int t1 = (int)((long long)(blockIdx.x + 1) * ntiles / gridDim.x);
    if (t0 >= t1) return;                                // uniform
    float wreg[NS];      // B operands: Omega[4 s + g][r] for the wave's steps
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const float v = W[(size_t)(4 * min(s0 + i, cpr - 1) + g) * 16 + r];
        wreg[i] = s0 + i < s1 ? v : 0.f;
    }
    // piece u of a lane: number lane + 64 u of the wave's two rows
    auto piece = [&](int u, int& rl, int& cc) {
        const int c = lane + 64 * u;
        rl = c >= cpr ? 1 : 0;
        cc = c - (rl ? cpr : 0);
        return c < 2 * cpr;
    };
    // No guard on the values: rows past the end read row 0 and only reach their own maxima, codes and output
    // rows, none of which is stored; pieces past the two rows read piece 0 and are not used.
    auto load_tile = [&](float4 (&x)[NV], int tile) {
        const int row0 = tile * 16 + 2 * wave;
        const float* p0 = X + (size_t)(row0 < rows ? row0 : 0) * ldx;
        const float* p1 = X + (size_t)(row0 + 1 < rows ? row0 + 1 : 0) * ldx;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            int rl, cc;
            const bool valid = piece(u, rl, cc);
            x[u] = *reinterpret_cast<const float4*>((rl ? p1 : p0) + 4 * (valid ? cc : 0));
        }
    };
    auto process = [&](const float4 (&x)[NV], int tile) {
        const int row0 = tile * 16 + 2 * wave;
        float m0 = 0.f, m1 = 0.f;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            int rl, cc;
            const bool valid = piece(u, rl, cc);
            const float mm = fmaxf(fmaxf(fabsf(x[u].x), fabsf(x[u].y)), fmaxf(fabsf(x[u].z), fabsf(x[u].w)));
            if (valid && rl == 0) m0 = fmaxf(m0, mm);
            if (valid && rl == 1) m1 = fmaxf(m1, mm);
        }
        m0 = wave_max(m0);
        m1 = wave_max(m1);
        float lam0, sc0, lam1, sc1;
        make_scales(m0, q.qmaxf, lam0, sc0);
        make_scales(m1, q.qmaxf, lam1, sc1);
        if (lane < 2 && row0 + lane < rows) {
            amax[row0 + lane] = lane ? m1 : m0;
            lam_out[row0 + lane] = lane ? lam1 : lam0;
            s_out[row0 + lane] = lane ? sc1 : sc0;
        }
        auto quantize = [&](auto mode) {         // one uniform branch on the rounding mode per tile
            constexpr int RM = decltype(mode)::value;
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                int rl, cc;
                if (!piece(u, rl, cc)) continue;
                const float lam_r = rl ? lam1 : lam0, s_r = rl ? sc1 : sc0;
                float c0, c1, c2, c3;
                float4 res;
                res.x = quant_code_residual<RM>(x[u].x, lam_r, s_r, q, c0);
                res.y = quant_code_residual<RM>(x[u].y, lam_r, s_r, q, c1);
                res.z = quant_code_residual<RM>(x[u].z, lam_r, s_r, q, c2);
                res.w = quant_code_residual<RM>(x[u].w, lam_r, s_r, q, c3);
                const int i0 = (int)c0, i1 = (int)c1, i2 = (int)c2, i3 = (int)c3;
                const uint32_t pk = (uint32_t)(i0 & 0xff) | ((uint32_t)(i1 & 0xff) << 8) |
                                    ((uint32_t)(i2 & 0xff) << 16) | ((uint32_t)(i3 & 0xff) << 24);
                if (row0 + rl < rows) *reinterpret_cast<uint32_t*>(codes + (size_t)(row0 + rl) * cols + 4 * cc) = pk;
                *reinterpret_cast<float4*>(rt + (2 * wave + rl) * ldr + 4 * cc) = res;
            }
        };
        if (q.round_mode == 0) quantize(std::integral_constant<int, 0>{});
        else quantize(std::integral_constant<int, 1>{});
        __syncthreads();        // the tile's residuals are in LDS; the last tile's partial products have been read
        if (tile > t0) gram_tile();     // the previous tile of Y is in LDS too
        v4f acc = (v4f){0.f, 0.f, 0.f, 0.f};
        const float* ap = rt + r * ldr + 4 * s0 + g;
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (s0 + i < s1) acc = mfma16(ap[4 * i], wreg[i], acc);      // the same for all lanes of a wave
#pragma unroll
        for (int v = 0; v < 4; ++v) pacc[wave][(4 * g + v) * 16 + r] = acc[v];
        __syncthreads();        // the eight partial products are in LDS; the residual tile has been read
        if (threadIdx.x < 256) {
            float sum = pacc[0][threadIdx.x];
#pragma unroll
            for (int w = 1; w < 8; ++w) sum += pacc[w][threadIdx.x];
            const int orow = tile * 16 + (threadIdx.x >> 4);
            if (orow < rows) Y[(size_t)orow * 16 + (threadIdx.x & 15)] = sum;
            yt[threadIdx.x >> 4][threadIdx.x & 15] = orow < rows ? sum : 0.f;
        }
    };
    float4 xa[NV], xb[NV];
    int tile = t0;
    load_tile(xa, tile);
    while (true) {          // two tiles per round: the register sets swap roles
        load_tile(xb, min(tile + 1, t1 - 1));
        process(xa, tile);
        if (++tile >= t1) break;
        load_tile(xa, min(tile + 1, t1 - 1));
        process(xb, tile);
        if (++tile >= t1) break;
    }
    __syncthreads();
    gram_tile();
    if (threadIdx.x < 256) gpart[(size_t)blockIdx.x * 256 + threadIdx.x] = gl[threadIdx.x];
}

// ---------------------------------------------------------------------------
// The same product on the bf16 matrix cores.  A float32 value is the exact sum of three
// bfloat16 planes (8 + 8 + 8 significant bits: round to nearest, subtract, repeat), and the
// product of two such sums is evaluated with the six plane products whose weight is at least
// 2^-16 of the leading one (r1 w1, r1 w2, r2 w1, r1 w3, r2 w2, r3 w1), each exact, accumulated
// in float32 by the matrix core: the dropped products are below 2^-24 of the leading one,
// the size of the float32 accumulation rounding itself.  Six v_mfma_f32_16x16x32_bf16 take
// 96 cycles per 32 k against 256 for eight v_mfma_f32_16x16x4_f32, and these kernels are
// bound by the matrix cores as soon as two of them share the chip.
// Operand layout (lane l): A[i = l%16][k = 8(l/16) .. +8], B[k = 8(l/16) .. +8][j = l%16],
// D[i = 4(l/16)+v][j = l%16].  The 8 k-slots of lane group g in a 32-deep step are the
// columns 4g .. 4g+3 and 16+4g .. 16+4g+3 of that step (two 16-byte loads of X); W is staged
// in LDS as three planes [plane][n][k] with k in that slot order, so a B operand is one
// 16-byte LDS read.
// ---------------------------------------------------------------------------
// acc[m][n] += a[m] . b[n] for NA x NB independent accumulators: the six plane products are
// the outer loop (smallest terms first), so consecutive matrix instructions never depend on
// each other.
// Reduced precision (the compensation terms "in half precision", Methodology, after Eq. (gemm_r_split)):
// with PL = 2 planes per operand the three products of weight >= 2^-8 are formed (relative error of a
// product 2^-16), with PL = 1 the leading product alone (2^-8, plain bfloat16 operands).
template <int NA, int NB, int PL = 3>
__device__ __forceinline__ void mfma_planes(const Planes3 (&a)[NA], const Planes3 (&b)[NB], v4f (&acc)[NA][NB]) {
#define LRQ_PP(PA, PB)                                                                               \
    _Pragma("unroll") for (int m = 0; m < NA; ++m) _Pragma("unroll") for (int n = 0; n < NB; ++n)     \
        acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m].PA, b[n].PB, acc[m][n], 0, 0, 0);
    if constexpr (PL >= 3) {
        LRQ_PP(p3, p1)
        LRQ_PP(p2, p2)
        LRQ_PP(p1, p3)
    }
    if constexpr (PL >= 2) {
        LRQ_PP(p2, p1)
        LRQ_PP(p1, p2)
    }
    LRQ_PP(p1, p1)
#undef LRQ_PP
}

// One thread's share of the chunk W[k0 .. k0+KC)[0..LP): units (n, group), a unit being the 8
// rows of W that form one lane group's k-slots of one 32-deep step, for one column n.
template <int NT, int KC, int PL = 3>
struct WStageBf16 {
    static constexpr int LP = NT * 16;
    static constexpr int LDK = KC + 8;                      // plane row stride in bfloat16
    static constexpr int UNITS = LP * (KC / 8);
    static constexpr int NU = (UNITS + 255) / 256;
    float v[NU][8];
    int off[NU];        // this thread's units: offset of their first element inside a chunk of W
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int unit = min((int)threadIdx.x + 256 * u, UNITS - 1);
            const int n = unit % LP, grp = unit / LP;
            off[u] = (32 * (grp >> 2) + 4 * (grp & 3)) * LP + n;
        }
    }
    // whole chunk inside the reduction range: no clamps, constant offsets from one base
    __device__ __forceinline__ void load_full(const float* __restrict__ W, int k0) {
        const float* p = W + (size_t)k0 * LP;
#pragma unroll
        for (int u = 0; u < NU; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[u][e] = p[off[u] + ((e & 3) + 16 * (e >> 2)) * LP];
    }
    __device__ __forceinline__ void load(const float* __restrict__ W, int k0, int kend) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int unit = min((int)threadIdx.x + 256 * u, UNITS - 1);
            const int n = unit % LP, grp = unit / LP;        // grp = 4 (step in chunk) + lane group
            const int kbase = k0 + 32 * (grp >> 2) + 4 * (grp & 3);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = kbase + (e & 3) + 16 * (e >> 2);
                const float t = W[(size_t)min(k, kend - 1) * LP + n];   // branch free: clamp, then select
                v[u][e] = k < kend ? t : 0.f;
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t* __restrict__ wl) const {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int unit = (int)threadIdx.x + 256 * u;
            if (unit < UNITS) {
                const int n = unit % LP, grp = unit / LP;
                const Planes3 pl = split_planes<PL>(v[u]);
                uint16_t* dst = wl + n * LDK + 8 * grp;
                *reinterpret_cast<v8bf16*>(dst) = pl.p1;
                if (PL >= 2) *reinterpret_cast<v8bf16*>(dst + LP * LDK) = pl.p2;
                if (PL >= 3) *reinterpret_cast<v8bf16*>(dst + 2 * LP * LDK) = pl.p3;
            }
        }
    }
};

// residual x - code s and the code itself (the arithmetic of quant_code / quant_residual_m)
// FULLK: the vector path with cols and the split length multiples of the chunk depth, so no
// load in the loop needs a guard along the reduction (rows past the end read row 0 and are not stored).
template <int NT, int AXIS, bool VEC, bool FULLK = false, int PL = 3, bool QOUT = false>
__global__ __launch_bounds__(256) void resid_mul_n_bf16_kernel(
    const float* __restrict__ X, int ldx, int rows, int cols, const float* __restrict__ lam,
    const float* __restrict__ sc, QuantParams q, const float* __restrict__ W, int chunk,
    float* __restrict__ partial, QOut qo) {
    static_assert(!QOUT || FULLK, "the fused quantization exists for the guard-free shapes only");
    constexpr int LP = NT * 16;
    constexpr int KC = 64;      // two 32-deep steps per chunk; 41 KB of LDS at l <= 48 (three workgroups per CU)
    constexpr int CTS = 80;     // row stride of the staged code tile (64 codes + padding), bytes
    __shared__ __align__(16) int8_t ct[QOUT ? 2 : 1][QOUT ? 64 * CTS : 16];
    constexpr int KS = KC / 16;                             // float4 loads per lane per chunk
    using WS = WStageBf16<NT, KC, PL>;
    constexpr int LDK = WS::LDK;
    __shared__ __align__(16) uint16_t wl[2][PL * LP * LDK];
    __shared__ __align__(16) float sl[2][2 * KC];   // per-column lambda | step of the chunk (AXIS 1)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int row = blockIdx.x * 64 + wave * 16 + r;
    const bool row_ok = row < rows;
    const float* xp = X + (size_t)(row_ok ? row : 0) * ldx;
    const int kb = blockIdx.y * chunk;
    const int ke = min(cols, kb + chunk);
    float lam_r = 0.f, s_r = 0.f;
    if (AXIS == 0 && row_ok) {
        if (QOUT) {
            make_scales(qo.amax[row], q.qmaxf, lam_r, s_r);
            if (blockIdx.y == 0 && g == 0) {
                qo.lam_out[row] = lam_r;
                qo.s_out[row] = s_r;
            }
        } else {
            lam_r = lam[row];
            s_r = sc[row];
        }
    }
    v4f acc[1][NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[0][nt] = (v4f){0.f, 0.f, 0.f, 0.f};

    float4 xr[KS];
    float scale_reg = 0.f;     // this thread's element of the chunk's lambda (t < KC) or step vector
    WS ws;
    if (FULLK) ws.init();
    const float* xq = xp + 4 * g;
    const float* scq = (QOUT ? qo.amax : ((threadIdx.x & KC) == 0 ? lam : sc)) + (threadIdx.x & (KC - 1));
    auto load_x = [&](int k0) {
        if (FULLK) {
#pragma unroll
            for (int j = 0; j < KS; ++j) xr[j] = *reinterpret_cast<const float4*>(xq + k0 + 16 * j);
            if (AXIS == 1) scale_reg = scq[k0];     // (QOUT: the column's maximum, turned into lambda or s below)
            return;
        }
#pragma unroll
        for (int j = 0; j < KS; ++j) xr[j] = load4f<VEC>(xp, k0 + 16 * j + 4 * g, ke, row_ok);
        if (AXIS == 1) {
            const int t = threadIdx.x & (KC - 1);
            const int kc = min(k0 + t, ke - 1);
            const float v = ((threadIdx.x & KC) == 0) ? lam[kc] : sc[kc];
            scale_reg = (k0 + t < ke) ? v : 0.f;
        }
    };
    auto load_w = [&](int k0) {
        if (FULLK) ws.load_full(W, k0);
        else ws.load(W, k0, ke);
    };
    if (kb < ke) {
        load_x(kb);
        load_w(kb);
    }
    // QOUT: the 64 x 64 code tile of a chunk is staged in LDS (two tiles, so the chunk loop keeps its single
    // barrier) and leaves for global memory one chunk later, 16 bytes per thread: rows of 64 contiguous bytes.
    // Tile rows are X rows (AXIS 0, codes row-major) or X columns (AXIS 1, codes transposed).
    auto flush_codes = [&](int tb, int kprev) {
        const int tr = threadIdx.x >> 2, seg = (threadIdx.x & 3) * 16;
        const uint4 v = *reinterpret_cast<const uint4*>(&ct[tb][tr * CTS + seg]);
        int8_t* dst = AXIS == 0 ? qo.codes + (size_t)(blockIdx.x * 64 + tr) * cols + kprev + seg
                                : qo.codes + (size_t)(kprev + tr) * rows + blockIdx.x * 64 + seg;
        *reinterpret_cast<uint4*>(dst) = v;
    };
    int buf = 0;
    for (int k0 = kb; k0 < ke; k0 += KC, buf ^= 1) {
        ws.store(wl[buf]);
        if (AXIS == 1 && threadIdx.x < 2 * KC) {
            if (QOUT) {     // scale_reg holds the column maximum: lambda for the first KC threads, the step for the next
                float l, st;
                make_scales(scale_reg, q.qmaxf, l, st);
                scale_reg = (threadIdx.x & KC) == 0 ? l : st;
                if (blockIdx.x == 0) ((threadIdx.x & KC) == 0 ? qo.lam_out : qo.s_out)[k0 + (threadIdx.x & (KC - 1))] = scale_reg;
            }
            sl[buf][threadIdx.x] = scale_reg;
        }
        __syncthreads();             // wl[buf], sl[buf] complete; the other buffers no longer read
        if (QOUT && k0 > kb) flush_codes(buf ^ 1, k0 - KC);
        Planes3 ap[KC / 32][1];
        auto residuals = [&](auto mode) {       // one uniform branch on the rounding mode per chunk
            constexpr int RM = decltype(mode)::value;
#pragma unroll
            for (int jj = 0; jj < KC / 32; ++jj) {
                float res[8];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int j = 2 * jj + h;
                    float4 l4, s4;
                    if (AXIS == 0) {
                        l4 = make_float4(lam_r, lam_r, lam_r, lam_r);
                        s4 = make_float4(s_r, s_r, s_r, s_r);
                    } else {
                        l4 = *reinterpret_cast<const float4*>(&sl[buf][16 * j + 4 * g]);
                        s4 = *reinterpret_cast<const float4*>(&sl[buf][KC + 16 * j + 4 * g]);
                    }
                    if (QOUT) {
                        float c0, c1, c2, c3;
                        res[4 * h + 0] = quant_code_residual<RM>(xr[j].x, l4.x, s4.x, q, c0);
                        res[4 * h + 1] = quant_code_residual<RM>(xr[j].y, l4.y, s4.y, q, c1);
                        res[4 * h + 2] = quant_code_residual<RM>(xr[j].z, l4.z, s4.z, q, c2);
                        res[4 * h + 3] = quant_code_residual<RM>(xr[j].w, l4.w, s4.w, q, c3);
                        const int i0 = (int)c0, i1 = (int)c1, i2 = (int)c2, i3 = (int)c3;
                        if (AXIS == 0) {    // four codes along the row: one packed word
                            const uint32_t pk = (uint32_t)(i0 & 0xff) | ((uint32_t)(i1 & 0xff) << 8) |
                                                ((uint32_t)(i2 & 0xff) << 16) | ((uint32_t)(i3 & 0xff) << 24);
                            *reinterpret_cast<uint32_t*>(&ct[buf][(wave * 16 + r) * CTS + 16 * j + 4 * g]) = pk;
                        } else {            // four columns of the transposed tile
                            int8_t* cp = &ct[buf][(16 * j + 4 * g) * CTS + wave * 16 + r];
                            cp[0] = (int8_t)i0;
                            cp[CTS] = (int8_t)i1;
                            cp[2 * CTS] = (int8_t)i2;
                            cp[3 * CTS] = (int8_t)i3;
                        }
                    } else {
                        res[4 * h + 0] = quant_residual_m<RM>(xr[j].x, l4.x, s4.x, q);
                        res[4 * h + 1] = quant_residual_m<RM>(xr[j].y, l4.y, s4.y, q);
                        res[4 * h + 2] = quant_residual_m<RM>(xr[j].z, l4.z, s4.z, q);
                        res[4 * h + 3] = quant_residual_m<RM>(xr[j].w, l4.w, s4.w, q);
                    }
                }
                ap[jj][0] = split_planes<PL>(res);
            }
        };
        if (q.round_mode == 0) residuals(std::integral_constant<int, 0>{});
        else residuals(std::integral_constant<int, 1>{});
        if (k0 + KC < ke) {      // next chunk's loads fly during this chunk's MFMAs
            load_x(k0 + KC);
            load_w(k0 + KC);
        }
        const uint16_t* wb = wl[buf];
#pragma unroll
        for (int jj = 0; jj < KC / 32; ++jj) {
            Planes3 bp[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const uint16_t* src = wb + (16 * nt + r) * LDK + 32 * jj + 8 * g;
                bp[nt].p1 = *reinterpret_cast<const v8bf16*>(src);
                if (PL >= 2) bp[nt].p2 = *reinterpret_cast<const v8bf16*>(src + LP * LDK);
                if (PL >= 3) bp[nt].p3 = *reinterpret_cast<const v8bf16*>(src + 2 * LP * LDK);
            }
            mfma_planes<1, NT, PL>(ap[jj], bp, acc);
        }
    }
    if (QOUT && kb < ke) {
        __syncthreads();
        flush_codes(buf ^ 1, ke - KC);
    }
    float* out = partial + (size_t)blockIdx.y * rows * LP;
    const int orow0 = blockIdx.x * 64 + wave * 16 + 4 * g;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (orow0 + v < rows) out[(size_t)(orow0 + v) * LP + 16 * nt + r] = acc[0][nt][v];
}

// Same contraction with an int8 code matrix as the streamed operand (no scales).
// blockIdx.z selects one of two independent jobs (A~ W and (V^T B~)^T share one launch).
struct CodesJob {
    const int8_t* Cq;   // rows x K codes
    const float* W;     // K x LP
    float* partial;     // [splits][rows][LP]
    int rows, chunk, splits;
};

template <int NT, bool VEC>
__global__ __launch_bounds__(256) void codes_mul_n_kernel(CodesJob j0, CodesJob j1, int K) {
    constexpr int LP = NT * 16;
    __shared__ __align__(16) float wl[2][KCHUNK * (LP + 4)];
    const CodesJob job = blockIdx.z == 0 ? j0 : j1;
    if ((int)blockIdx.x * 64 >= job.rows || (int)blockIdx.y >= job.splits) return;
    const int8_t* __restrict__ Cq = job.Cq;
    const float* __restrict__ W = job.W;
    float* __restrict__ partial = job.partial;
    const int rows = job.rows, chunk = job.chunk;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int row = blockIdx.x * 64 + wave * 16 + r;
    const bool row_ok = row < rows;
    const int8_t* cp = Cq + (size_t)(row_ok ? row : 0) * K;
    const int kb = blockIdx.y * chunk;
    const int ke = min(K, kb + chunk);
    v4f acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = (v4f){0.f, 0.f, 0.f, 0.f};
    uint32_t cr[KSUB];
    WStage<NT> ws;
    auto load_c = [&](int k0) {
#pragma unroll
        for (int j = 0; j < KSUB; ++j) {
            const int k = k0 + 16 * j + 4 * g;
            uint32_t p = 0;
            if (VEC) {      // branch free: clamp, then select (K % 4 == 0)
                const uint32_t t = *reinterpret_cast<const uint32_t*>(cp + min(k, ke - 4));
                p = (row_ok && k < ke) ? t : 0u;
            } else if (row_ok) {
                {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (k + t < ke) p |= (uint32_t)(uint8_t)cp[k + t] << (8 * t);
                }
            }
            cr[j] = p;
        }
    };
    if (kb < ke) {
        load_c(kb);
        ws.load(W, kb, ke);
    }
    int buf = 0;
    for (int k0 = kb; k0 < ke; k0 += KCHUNK, buf ^= 1) {
        ws.store(wl[buf]);
        float res[KSUB][4];
#pragma unroll
        for (int j = 0; j < KSUB; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t) res[j][t] = (float)(int8_t)((cr[j] >> (8 * t)) & 0xff);
        if (k0 + KCHUNK < ke) {
            load_c(k0 + KCHUNK);
            ws.load(W, k0 + KCHUNK, ke);
        }
        __syncthreads();
        const float* wb = wl[buf];
#pragma unroll
        for (int j = 0; j < KSUB; ++j) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* wrow = wb + (16 * j + 4 * g + t) * (LP + 4) + r;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma16(res[j][t], wrow[16 * nt], acc[nt]);
            }
        }
    }
    float* out = partial + (size_t)blockIdx.y * rows * LP;
    const int orow0 = blockIdx.x * 64 + wave * 16 + 4 * g;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (orow0 + v < rows) out[(size_t)(orow0 + v) * LP + 16 * nt + r] = acc[nt][v];
}

// The same code-matrix product on the bf16 matrix cores.  An int8 code is exact in bfloat16
// (8 significant bits) and the float32 factor is supplied as three bfloat16 planes
// hi + mid + lo (exact to 2^-27, see split_bf16x3), so
//   code . w = code . hi + code . mid + code . lo
// holds with every product exact and float32 accumulation in the matrix core: float32
// accuracy at a fraction of the float32 MFMA cost (3 x 16 cycles instead of 8 x 32 per 32 k).
// v_mfma_f32_16x16x32_bf16 operand layout (lane l): A[i = l%16][k = 8(l/16) .. +8],
// B[k = 8(l/16) .. +8][j = l%16], D[i = 4(l/16)+v][j = l%16].  The reduction index may be
// visited in any order: in a 64-deep chunk lane group kq = l/16 owns k = 16 kq .. 16 kq + 15
// (one 16-byte load of codes), first half in MFMA step 0, second half in step 1.
// Bp: [3][RP][Kp] bfloat16 planes of the factor, k fastest, zero padded (Kp % 64 == 0).
// Needs K % 16 == 0, K >= 16 and 16-byte aligned codes.
struct CodesJobBf16 {
    const int8_t* Cq;       // rows x K codes
    const uint16_t* Bp;     // [3][RP][Kp]
    float* partial;         // [splits][rows][RP]
    int rows, chunk, splits;
};
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// 8 int8 codes (two dwords) -> 8 bfloat16: float(code) keeps only its upper 16 bits.
__device__ __forceinline__ v8bf codes_to_bf16(uint32_t lo, uint32_t hi) {
    union { uint32_t u[4]; v8bf v; } r;
    const uint32_t w[2] = {lo, hi};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float f0 = (float)(int)(int8_t)(w[h] & 0xff), f1 = (float)(int)(int8_t)((w[h] >> 8) & 0xff);
        const float f2 = (float)(int)(int8_t)((w[h] >> 16) & 0xff), f3 = (float)(int)(int8_t)(w[h] >> 24);
        r.u[2 * h + 0] = (__float_as_uint(f0) >> 16) | (__float_as_uint(f1) & 0xffff0000u);
        r.u[2 * h + 1] = (__float_as_uint(f2) >> 16) | (__float_as_uint(f3) & 0xffff0000u);
    }
    return r.v;
}

// Launch shape: grid (ceil(rows / (64 MT)), splits, 2 jobs).  A wave owns 16 MT rows; for each KB-deep slab of
// its split it issues ALL its code loads at once (KB bytes per row), the four waves copy the slab of Bp into
// LDS meanwhile, and after one barrier the matrix cores run through the slab without further waits: the HBM
// latency is paid once per slab with the whole operand in flight.
template <int NT, int PL = 3>
struct CodesShape {
    static constexpr int RP = NT * 16;
    static constexpr int KB = 256;                      // slab depth: PL RP (KB + 8) bf16 in LDS
    static constexpr int LDK = KB + 8;
    static constexpr int NC = KB / 64;                  // 64-deep chunks per slab
    static constexpr int PIECES = PL * RP * (KB / 8);   // 16-byte pieces of a slab of the first PL planes of Bp
    static constexpr int BATCH = 8;
};

// PL: planes of the factor that enter (3: float32 accuracy; 2: relative error 2^-16; 1: plain bfloat16 factor).
// MT: 16-row tiles per wave (a wave owns 16 MT rows, a workgroup 64 MT).
template <int NT, int PL = 3, int MT = 4>
__global__ __launch_bounds__(256, 1) void codes_mul_bf16_kernel(CodesJobBf16 j0, CodesJobBf16 j1, int K, int Kp) {
    using S = CodesShape<NT, PL>;
    constexpr int RP = S::RP, KB = S::KB, LDK = S::LDK, NC = S::NC;
    __shared__ __align__(16) uint16_t bs[PL * RP * LDK];
    const CodesJobBf16 job = blockIdx.z == 0 ? j0 : j1;
    if ((int)blockIdx.x * 64 * MT >= job.rows || (int)blockIdx.y >= job.splits) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, kq = lane >> 4;
    const int r0 = blockIdx.x * 64 * MT + wave * 16 * MT;
    const int kb = blockIdx.y * job.chunk, ke = min(K, kb + job.chunk);
    const int8_t* ap[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) ap[mt] = job.Cq + (size_t)min(r0 + 16 * mt + li, job.rows - 1) * K;
    v4f acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int ks = kb; ks < ke; ks += KB) {
        // codes of the whole slab; rows past the end re-read the last row (never stored), and
        // codes past K meet zero planes, so clamped addresses need no mask
        uint4 ca[MT][NC];
#pragma unroll
        for (int c = 0; c < NC; ++c)            // issued in the order of use: the first chunk's products can start
#pragma unroll                                  // while the later chunks are still on their way
            for (int mt = 0; mt < MT; ++mt)
                ca[mt][c] = *reinterpret_cast<const uint4*>(ap[mt] + min(ks + 64 * c + 16 * kq, K - 16));
        if (ks > kb) __syncthreads();       // previous slab no longer read
        for (int p0 = threadIdx.x; p0 < S::PIECES; p0 += 256 * S::BATCH) {
            uint4 t[S::BATCH];
#pragma unroll
            for (int u = 0; u < S::BATCH; ++u) {
                const int p = min(p0 + 256 * u, S::PIECES - 1);
                const int rowp = p / (KB / 8), seg = p - rowp * (KB / 8);
                const int k = ks + 8 * seg;
                const uint4 v = *reinterpret_cast<const uint4*>(job.Bp + (size_t)rowp * Kp + min(k, Kp - 8));
                t[u] = (k < Kp) ? v : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < S::BATCH; ++u) {
                const int p = p0 + 256 * u;
                if (p < S::PIECES) {
                    const int rowp = p / (KB / 8), seg = p - rowp * (KB / 8);
                    *reinterpret_cast<uint4*>(&bs[rowp * LDK + 8 * seg]) = t[u];
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (ks + 64 * c < ke) {             // uniform
#pragma unroll
                for (int sidx = 0; sidx < 2; ++sidx) {
                    v8bf af[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        af[mt] = sidx == 0 ? codes_to_bf16(ca[mt][c].x, ca[mt][c].y)
                                           : codes_to_bf16(ca[mt][c].z, ca[mt][c].w);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int pl = 0; pl < PL; ++pl) {
                            union { uint4 u; v8bf v; } b;
                            b.u = *reinterpret_cast<const uint4*>(
                                &bs[(pl * RP + 16 * nt + li) * LDK + 64 * c + 16 * kq + 8 * sidx]);
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[mt], b.v, acc[mt][nt], 0, 0, 0);
                        }
                }
            }
        }
    }
    float* out = job.partial + (size_t)blockIdx.y * job.rows * RP;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = r0 + 16 * mt + 4 * kq + v;
                if (row < job.rows) out[(size_t)row * RP + 16 * nt + li] = acc[mt][nt][v];
            }
}

// The same product for short rows (K <= 640) and factors of at most 16 columns: all of Bp fits in LDS (PL planes
// x 16 rows x (Kp + 8) bfloat16), so workgroups are persistent -- two of eight waves per CU, the planes copied once --
// and after the one barrier behind that copy the waves are on their own: a wave takes the 16-row tiles w, w + W,
// w + 2W, ... (W waves in the grid) and loads a tile's codes at once (NC 16-byte loads per lane, the whole row);
// the sixteen waves of a CU are at different points of that cycle, which keeps loads in flight while others
// compute.  blockIdx.z selects the job as above.
template <int PL, int NC>
__global__ __launch_bounds__(512, 4) void codes_mul_rows_kernel(CodesJobBf16 j0, CodesJobBf16 j1, int K, int Kp) {
    extern __shared__ __align__(16) uint16_t bsr[];       // [PL][16][Kp + 8]
    const CodesJobBf16 job = blockIdx.z == 0 ? j0 : j1;
    const int ntiles = (job.rows + 15) >> 4;
    if ((int)blockIdx.x * 8 >= ntiles) return;            // no tile for any wave of this workgroup
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, kq = lane >> 4;
    const int LDK = Kp + 8, ppr = Kp >> 3;
    for (int p = threadIdx.x; p < PL * 16 * ppr; p += 512) {
        const int rowp = p / ppr, seg = p - rowp * ppr;
        *reinterpret_cast<uint4*>(&bsr[rowp * LDK + 8 * seg]) =
            *reinterpret_cast<const uint4*>(job.Bp + (size_t)rowp * Kp + 8 * seg);
    }
    __syncthreads();
    const int nwaves = gridDim.x * 8;
    // codes past K meet zero planes and rows past the end re-read the last row (never stored): clamped
    // addresses, no masks
    auto load_tile = [&](uint4 (&ca)[NC], int tile) {
        const int8_t* ap = job.Cq + (size_t)min(tile * 16 + li, job.rows - 1) * K;
#pragma unroll
        for (int c = 0; c < NC; ++c) ca[c] = *reinterpret_cast<const uint4*>(ap + min(64 * c + 16 * kq, K - 16));
    };
    auto process = [&](const uint4 (&ca)[NC], int tile) {
        v4f acc = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (64 * c >= Kp) continue;             // the planes end at Kp (uniform)
#pragma unroll
            for (int sidx = 0; sidx < 2; ++sidx) {
                const v8bf af = sidx == 0 ? codes_to_bf16(ca[c].x, ca[c].y) : codes_to_bf16(ca[c].z, ca[c].w);
#pragma unroll
                for (int pl = 0; pl < PL; ++pl) {
                    union { uint4 u; v8bf v; } b;
                    b.u = *reinterpret_cast<const uint4*>(&bsr[(pl * 16 + li) * LDK + 64 * c + 16 * kq + 8 * sidx]);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, b.v, acc, 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = tile * 16 + 4 * kq + v;
            if (row < job.rows) job.partial[(size_t)row * 16 + li] = acc[v];
        }
    };
    uint4 x[NC];
    for (int tile = blockIdx.x * 8 + wave; tile < ntiles; tile += nwaves) {
        load_tile(x, tile);
        process(x, tile);
    }
}

// ---------------------------------------------------------------------------
// T-type: partial[split][cols][LP] = R[i-range, :]^T . W[i-range, :]
// grid (ceil(cols/64), splits); the 4 waves of a block share one 64-column strip,
// interleave rows, and merge their accumulators through LDS.
// A lane's float4 holds columns c0+4c .. c0+4c+3; component t feeds M-tile t, so
// M-tile t covers the columns {c0 + 4 c + t}.  Likewise N-tile nt covers the W columns
// {NT c + nt}, so a lane's B operands are NT consecutive floats (one wide load).
// Loads run TUNR row groups ahead of the matrix cores (register double buffering).
// ---------------------------------------------------------------------------
#define TUNR 4
template <int NT, int AXIS, bool VEC>
__global__ __launch_bounds__(256) void resid_mul_t_kernel(
    const float* __restrict__ X, int ldx, int rows, int cols, const float* __restrict__ lam,
    const float* __restrict__ sc, QuantParams q, const float* __restrict__ W, int chunk,
    float* __restrict__ partial) {
    constexpr int LP = NT * 16;
    __shared__ __align__(16) float red[64 * LP];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int c0 = blockIdx.x * 64;
    const int kc = c0 + 4 * c;
    const int ib = blockIdx.y * chunk;
    const int ie = min(rows, ib + chunk);
    float4 lc = make_float4(0.f, 0.f, 0.f, 0.f), scol = lc;
    if (AXIS == 1 && kc < cols) {   // padded with zeros to a multiple of 4
        lc = *reinterpret_cast<const float4*>(lam + kc);
        scol = *reinterpret_cast<const float4*>(sc + kc);
    }
    v4f acc[4][NT];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[t][nt] = (v4f){0.f, 0.f, 0.f, 0.f};

    struct Frag {
        float4 x;
        float lr, sr;
        float w[NT];
    };
    auto load_frag = [&](int i0, Frag& f) {
        const int i = i0 + g;
        const bool ok = i < ie;
        const size_t ii = ok ? (size_t)i : 0;
        f.x = load4f<VEC>(X + ii * ldx, kc, cols, ok);
        if (AXIS == 0) {            // unconditional loads from a valid row, then selects
            const float l = lam[ii], sv = sc[ii];
            f.lr = ok ? l : 0.f;
            f.sr = ok ? sv : 0.f;
        }
        const float* wp = W + ii * LP + NT * c;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float wv = wp[nt];
            f.w[nt] = ok ? wv : 0.f;
        }
    };
    Frag cur[TUNR], nxt[TUNR];
    const int istart = ib + wave * 4;
#pragma unroll
    for (int u = 0; u < TUNR; ++u) load_frag(istart + 16 * u, cur[u]);
    for (int i0 = istart; i0 < ie; i0 += 16 * TUNR) {
#pragma unroll
        for (int u = 0; u < TUNR; ++u) load_frag(i0 + 16 * (TUNR + u), nxt[u]);
#pragma unroll
        for (int u = 0; u < TUNR; ++u) {
            float4 l4 = lc, s4 = scol;
            if (AXIS == 0) {
                l4 = make_float4(cur[u].lr, cur[u].lr, cur[u].lr, cur[u].lr);
                s4 = make_float4(cur[u].sr, cur[u].sr, cur[u].sr, cur[u].sr);
            }
            float res[4];
            res[0] = quant_residual(cur[u].x.x, l4.x, s4.x, q);
            res[1] = quant_residual(cur[u].x.y, l4.y, s4.y, q);
            res[2] = quant_residual(cur[u].x.z, l4.z, s4.z, q);
            res[3] = quant_residual(cur[u].x.w, l4.w, s4.w, q);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[t][nt] = mfma16(res[t], cur[u].w[nt], acc[t][nt]);
        }
#pragma unroll
        for (int u = 0; u < TUNR; ++u) cur[u] = nxt[u];
    }
    // merge the four waves (fixed order: deterministic)
    for (int wv = 0; wv < 4; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int cl = 16 * g + 4 * v + t;   // local column of D row 4g+v in M-tile t
                        float* p = red + cl * LP + NT * c + nt;
                        *p = (wv == 0) ? acc[t][nt][v] : (*p + acc[t][nt][v]);
                    }
        }
        __syncthreads();
    }
    float* out = partial + (size_t)blockIdx.y * cols * LP;
    for (int idx = threadIdx.x; idx < 64 * LP / 4; idx += 256) {
        const int e = idx * 4;
        const int cl = e / LP, n = e % LP;
        if (c0 + cl < cols)
            *reinterpret_cast<float4*>(out + (size_t)(c0 + cl) * LP + n) =
                *reinterpret_cast<const float4*>(red + cl * LP + n);
    }
}

// The T-type product on the bf16 matrix cores (see resid_mul_n_bf16_kernel for the plane
// arithmetic).  A wave takes 32 rows per step: lane group g loads rows base + 4e + g (e < 8),
// which are its 8 k-slots; both operands come straight from global memory in that order (a
// float4 of X and NT floats of W per row), so no LDS is needed before the final merge.
// (two workgroups per CU up to l = 64: the register cap costs no spills there and hides the loads better)
// FULLT: the vector path with whole column strips and a split length that is a multiple of the
// 128 rows a workgroup takes per step: no load needs a guard, and the row part of every address
// is wave-uniform (scalar registers), the lane part a constant 32-bit offset.
template <int NT, int AXIS, bool VEC, bool FULLT = false, int PL = 3>
__global__ __launch_bounds__(256, (NT <= 4 || FULLT) ? 2 : 1) void resid_mul_t_bf16_kernel(
    const float* __restrict__ X, int ldx, int rows, int cols, const float* __restrict__ lam,
    const float* __restrict__ sc, QuantParams q, const float* __restrict__ W, int chunk,
    float* __restrict__ partial) {
    constexpr int LP = NT * 16;
    __shared__ __align__(16) float red[64 * LP];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int c0 = blockIdx.x * 64;
    const int kc = c0 + 4 * c;
    const int ib = blockIdx.y * chunk;
    const int ie = min(rows, ib + chunk);
    float lcol[4] = {0.f, 0.f, 0.f, 0.f}, scol[4] = {0.f, 0.f, 0.f, 0.f};
    if (AXIS == 1 && kc < cols) {   // padded with zeros to a multiple of 4
        const float4 l4 = *reinterpret_cast<const float4*>(lam + kc);
        const float4 s4 = *reinterpret_cast<const float4*>(sc + kc);
        lcol[0] = l4.x; lcol[1] = l4.y; lcol[2] = l4.z; lcol[3] = l4.w;
        scol[0] = s4.x; scol[1] = s4.y; scol[2] = s4.z; scol[3] = s4.w;
    }
    v4f acc[4][NT];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[t][nt] = (v4f){0.f, 0.f, 0.f, 0.f};

    struct Group {
        float x[8][4];
        float lr[8], sr[8];
        float w[8][NT];
    };
    auto load_group = [&](int i0, Group& f) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int i = i0 + 4 * e + g;
            const bool ok = i < ie;
            const size_t ii = ok ? (size_t)i : 0;      // unconditional loads from a valid row, then selects
            const float4 xv = load4f<VEC>(X + ii * ldx, kc, cols, ok);
            f.x[e][0] = xv.x; f.x[e][1] = xv.y; f.x[e][2] = xv.z; f.x[e][3] = xv.w;
            if (AXIS == 0) {
                const float l = lam[ii], sv = sc[ii];
                f.lr[e] = ok ? l : 0.f;
                f.sr[e] = ok ? sv : 0.f;
            }
            const float* wp = W + ii * LP + NT * c;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float wv = wp[nt];
                f.w[e][nt] = ok ? wv : 0.f;
            }
        }
    };
    const int xoff = g * ldx + kc, woff = g * LP + NT * c;      // lane part of the addresses (FULLT)
    auto load_group_full = [&](int i0, Group& f) {              // i0 wave-uniform
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float* xrow = X + (size_t)(i0 + 4 * e) * ldx;
            const float4 xv = *reinterpret_cast<const float4*>(xrow + xoff);
            f.x[e][0] = xv.x; f.x[e][1] = xv.y; f.x[e][2] = xv.z; f.x[e][3] = xv.w;
            if (AXIS == 0) {
                f.lr[e] = (lam + i0 + 4 * e)[g];
                f.sr[e] = (sc + i0 + 4 * e)[g];
            }
            const float* wrow = W + (size_t)(i0 + 4 * e) * LP;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) f.w[e][nt] = wrow[woff + nt];
        }
    };
    Group cur, nxt;
    const int istart = ib + 32 * (FULLT ? __builtin_amdgcn_readfirstlane(wave) : wave);
    if (FULLT) load_group_full(istart, cur);
    else load_group(istart, cur);
    for (int i0 = istart; i0 < ie; i0 += 128) {
        if (FULLT) load_group_full(i0 + 128 < ie ? i0 + 128 : i0, nxt);     // last step: re-reads its own rows
        else load_group(i0 + 128, nxt);      // past the end: every row masked
        Planes3 bp[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float wv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) wv[e] = cur.w[e][nt];
            bp[nt] = split_planes<PL>(wv);
        }
#pragma unroll
        for (int th = 0; th < 2; ++th) {        // two column components at a time: 2 NT independent chains
            Planes3 ap[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const int t = 2 * th + tt;
                float res[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    res[e] = quant_residual(cur.x[e][t], AXIS == 0 ? cur.lr[e] : lcol[t],
                                            AXIS == 0 ? cur.sr[e] : scol[t], q);
                ap[tt] = split_planes<PL>(res);
            }
            v4f (&a2)[2][NT] = *reinterpret_cast<v4f (*)[2][NT]>(&acc[2 * th]);
            mfma_planes<2, NT, PL>(ap, bp, a2);
        }
        cur = nxt;
    }
    // merge the four waves (fixed order: deterministic)
    for (int wv = 0; wv < 4; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int cl = 16 * g + 4 * v + t;   // local column of D row 4g+v in M-tile t
                        float* p = red + cl * LP + NT * c + nt;
                        *p = (wv == 0) ? acc[t][nt][v] : (*p + acc[t][nt][v]);
                    }
        }
        __syncthreads();
    }
    float* out = partial + (size_t)blockIdx.y * cols * LP;
    for (int idx = threadIdx.x; idx < 64 * LP / 4; idx += 256) {
        const int e = idx * 4;
        const int cl = e / LP, n = e % LP;
        if (c0 + cl < cols)
            *reinterpret_cast<float4*>(out + (size_t)(c0 + cl) * LP + n) =
                *reinterpret_cast<const float4*>(red + cl * LP + n);
    }
}

// ---------------------------------------------------------------------------
// launch plans and dispatch
// ---------------------------------------------------------------------------
static int pick_splits(int blocks_one_split, int reduce_len, int unit, int limit) {
    // aim for ~512 workgroups (2 per CU) but keep >= 4 `unit`-sized steps per split
    int want = ceil_div(512, max(1, blocks_one_split));
    int max_splits = max(1, reduce_len / (4 * unit));
    int s = max(1, min(want, min(max_splits, limit)));
    return s;
}

PassPlan plan_pass_n(int rows, int cols) {
    PassPlan p;
    int s = pick_splits(ceil_div(rows, 64), cols, KCHUNK, MAX_SPLITS);
    p.chunk = ceil_div(ceil_div(cols, s), KCHUNK) * KCHUNK;
    p.splits = ceil_div(cols, p.chunk);
    return p;
}

PassPlan plan_pass_t(int rows, int cols) {
    PassPlan p;
    int s = pick_splits(ceil_div(cols, 64), rows, 16, MAX_SPLITS_T);     // few column strips: many row chunks
    // (a multiple of the 128 rows a workgroup takes per step when there are enough rows: guard-free kernel)
    const int unit = rows >= 512 * s ? 128 : 16;
    p.chunk = ceil_div(ceil_div(rows, s), unit) * unit;
    p.splits = ceil_div(rows, p.chunk);
    return p;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Sketches of up to 16 columns keep the float32 matrix-core kernels (one tile of W columns: the
// matrix cores are nowhere near busy and splitting operands into planes only adds work; the
// conv-shaped workload with l = 8 measures 0.37 ms against 0.39 ms); wider ones use the bf16 kernels.
template <int NT, int AXIS, bool VEC>
struct PassKernels {
    static constexpr auto n = NT == 1 ? resid_mul_n_kernel<NT, AXIS, VEC> : resid_mul_n_bf16_kernel<NT, AXIS, VEC>;
    static constexpr auto t = NT == 1 ? resid_mul_t_kernel<NT, AXIS, VEC> : resid_mul_t_bf16_kernel<NT, AXIS, VEC>;
};
#define LRQ_PASS_ARGS grid, dim3(256), 0, st, X, ldx, rows, cols, lam, s, q, W, chunk, partial
#define LRQ_PASS_ARGS_N LRQ_PASS_ARGS, QOut{}
#define LRQ_PASS_ARGS_TAIL grid, st, X, ldx, rows, cols, lam, s, q, W, chunk, partial
// Reduced precision (planes 2 or 1): the bf16 kernels for every sketch width.
template <int NT, int PL>
static void dispatch_n_reduced(int axis, bool vec, bool fullk, dim3 grid, hipStream_t st, const float* X, int ldx,
                               int rows, int cols, const float* lam, const float* s, QuantParams q, const float* W,
                               int chunk, float* partial) {
    if (fullk) {
        if (axis == 0) hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 0, true, true, PL>), LRQ_PASS_ARGS_N);
        else           hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 1, true, true, PL>), LRQ_PASS_ARGS_N);
    } else if (axis == 0) {
        if (vec) hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 0, true, false, PL>), LRQ_PASS_ARGS_N);
        else     hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 0, false, false, PL>), LRQ_PASS_ARGS_N);
    } else {
        if (vec) hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 1, true, false, PL>), LRQ_PASS_ARGS_N);
        else     hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 1, false, false, PL>), LRQ_PASS_ARGS_N);
    }
}
template <int NT, int PL>
static void dispatch_t_reduced(int axis, bool vec, bool fullt, dim3 grid, hipStream_t st, const float* X, int ldx,
                               int rows, int cols, const float* lam, const float* s, QuantParams q, const float* W,
                               int chunk, float* partial) {
    if (fullt) {
        if (axis == 0) hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 0, true, true, PL>), LRQ_PASS_ARGS);
        else           hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 1, true, true, PL>), LRQ_PASS_ARGS);
    } else if (axis == 0) {
        if (vec) hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 0, true, false, PL>), LRQ_PASS_ARGS);
        else     hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 0, false, false, PL>), LRQ_PASS_ARGS);
    } else {
        if (vec) hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 1, true, false, PL>), LRQ_PASS_ARGS);
        else     hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 1, false, false, PL>), LRQ_PASS_ARGS);
    }
}
template <int NT>
static void dispatch_n(int axis, bool vec, int planes, dim3 grid, hipStream_t st, const float* X, int ldx, int rows,
                       int cols, const float* lam, const float* s, QuantParams q, const float* W, int chunk,
                       float* partial) {
    // every chunk of every split is whole: the guard-free instantiation
    const bool fullk = vec && cols % 64 == 0 && chunk % 64 == 0;
    if (planes == 2) return dispatch_n_reduced<NT, 2>(axis, vec, fullk, LRQ_PASS_ARGS_TAIL);
    if (planes == 1) return dispatch_n_reduced<NT, 1>(axis, vec, fullk, LRQ_PASS_ARGS_TAIL);
    if constexpr (NT > 1) {
        if (fullk) {
            if (axis == 0) hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 0, true, true>), LRQ_PASS_ARGS_N);
            else           hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NT, 1, true, true>), LRQ_PASS_ARGS_N);
            return;
        }
    }
    if (axis == 0) {
        if (vec) hipLaunchKernelGGL((PassKernels<NT, 0, true>::n), LRQ_PASS_ARGS_N);
        else     hipLaunchKernelGGL((PassKernels<NT, 0, false>::n), LRQ_PASS_ARGS_N);
    } else {
        if (vec) hipLaunchKernelGGL((PassKernels<NT, 1, true>::n), LRQ_PASS_ARGS_N);
        else     hipLaunchKernelGGL((PassKernels<NT, 1, false>::n), LRQ_PASS_ARGS_N);
    }
}

template <int NT>
static void dispatch_t(int axis, bool vec, int planes, dim3 grid, hipStream_t st, const float* X, int ldx, int rows,
                       int cols, const float* lam, const float* s, QuantParams q, const float* W, int chunk,
                       float* partial) {
    // whole column strips, whole 128-row steps in every split: the guard-free instantiation
    const bool fullt = vec && cols % 64 == 0 && chunk % 128 == 0 && rows % 128 == 0;
    if (planes == 2) return dispatch_t_reduced<NT, 2>(axis, vec, fullt, LRQ_PASS_ARGS_TAIL);
    if (planes == 1) return dispatch_t_reduced<NT, 1>(axis, vec, fullt, LRQ_PASS_ARGS_TAIL);
    if constexpr (NT > 1) {
        if (fullt) {
            if (axis == 0) hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 0, true, true>), LRQ_PASS_ARGS);
            else           hipLaunchKernelGGL((resid_mul_t_bf16_kernel<NT, 1, true, true>), LRQ_PASS_ARGS);
            return;
        }
    }
    if (axis == 0) {
        if (vec) hipLaunchKernelGGL((PassKernels<NT, 0, true>::t), LRQ_PASS_ARGS);
        else     hipLaunchKernelGGL((PassKernels<NT, 0, false>::t), LRQ_PASS_ARGS);
    } else {
        if (vec) hipLaunchKernelGGL((PassKernels<NT, 1, true>::t), LRQ_PASS_ARGS);
        else     hipLaunchKernelGGL((PassKernels<NT, 1, false>::t), LRQ_PASS_ARGS);
    }
}

template <int NT>
static void dispatch_c(bool vec, dim3 grid, hipStream_t st, CodesJob j0, CodesJob j1, int K) {
    if (vec) hipLaunchKernelGGL((codes_mul_n_kernel<NT, true>), grid, dim3(256), 0, st, j0, j1, K);
    else     hipLaunchKernelGGL((codes_mul_n_kernel<NT, false>), grid, dim3(256), 0, st, j0, j1, K);
}

#define NT_SWITCH(NTV, CALL)            \
    switch (NTV) {                      \
        case 1: { constexpr int NT_ = 1; CALL; } break; \
        case 2: { constexpr int NT_ = 2; CALL; } break; \
        case 3: { constexpr int NT_ = 3; CALL; } break; \
        case 4: { constexpr int NT_ = 4; CALL; } break; \
        case 5: { constexpr int NT_ = 5; CALL; } break; \
        default: return LRQMM_ERR_UNSUPPORTED;          \
    }

int launch_resid_mul_n(const float* X, int ldx, int rows, int cols, int axis, const float* lam, const float* s,
                       QuantParams q, const float* W, int LP, PassPlan plan, float* partial,
                       hipStream_t st, int planes) {
    const bool vec = (cols % 4 == 0) && (ldx % 4 == 0) && aligned16(X);
    dim3 grid(ceil_div(rows, 64), plan.splits);
    NT_SWITCH(LP / 16, (dispatch_n<NT_>(axis, vec, planes, grid, st, X, ldx, rows, cols, lam, s, q, W, plan.chunk, partial)));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

bool quant_sketch_fusable(const float* X, int ldx, int rows, int cols, int LP, PassPlan plan, const int8_t* codes) {
    return LP >= 32 && rows % 64 == 0 && cols % 64 == 0 && plan.chunk % 64 == 0 && ldx % 4 == 0 && aligned16(X) &&
           aligned16(codes);
}

int launch_quant_sketch(const float* X, int ldx, int rows, int cols, int axis, const float* amax, QuantParams q,
                        const float* W, int LP, PassPlan plan, float* partial, float* lam_out, float* s_out,
                        int8_t* codes, hipStream_t st, int planes) {
    if (!quant_sketch_fusable(X, ldx, rows, cols, LP, plan, codes)) return LRQMM_ERR_UNSUPPORTED;
    dim3 grid(rows / 64, plan.splits);
    const QOut qo = {amax, lam_out, s_out, codes};
    const float* lam = nullptr;
    const float* s = nullptr;
    const int chunk = plan.chunk;
#define LRQ_QS(NTV, PLV)                                                                                           \
    do {                                                                                                            \
        if (axis == 0) hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NTV, 0, true, true, PLV, true>), LRQ_PASS_ARGS, qo); \
        else           hipLaunchKernelGGL((resid_mul_n_bf16_kernel<NTV, 1, true, true, PLV, true>), LRQ_PASS_ARGS, qo); \
    } while (0)
#define LRQ_QS_PL(NTV) do { if (planes == 2) LRQ_QS(NTV, 2); else if (planes == 1) LRQ_QS(NTV, 1); else LRQ_QS(NTV, 3); } while (0)
    switch (LP / 16) {
        case 2: LRQ_QS_PL(2); break;
        case 3: LRQ_QS_PL(3); break;
        case 4: LRQ_QS_PL(4); break;
        case 5: LRQ_QS_PL(5); break;
        default: return LRQMM_ERR_UNSUPPORTED;
    }
#undef LRQ_QS_PL
#undef LRQ_QS
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

bool quant_sketch_rows_usable(const float* X, int ldx, int rows, int cols, int LP, const int8_t* codes) {
    // (rows of up to 576 columns: beyond that the two register sets of a tile no longer fit 128 registers)
    return rows > 0 && LP == 16 && cols >= 16 && cols % 16 == 0 && cols <= 576 && ldx % 4 == 0 && aligned16(X) &&
           ((uintptr_t)codes & 3) == 0;
}

int quant_sketch_rows_blocks(int rows) { return min(ceil_div(rows, 16), LRQ_QSR_MAX_BLOCKS); }

int launch_quant_sketch_rows(const float* X, int ldx, int rows, int cols, QuantParams q, const float* W, int LP,
                             float* Y, double* gpart, float* amax, float* lam_out, float* s_out, int8_t* codes,
                             hipStream_t st) {
    if (!quant_sketch_rows_usable(X, ldx, rows, cols, LP, codes)) return LRQMM_ERR_UNSUPPORTED;
    // persistent workgroups, each with a run of 16-row tiles; their number does not depend on the device, so
    // neither does the order in which the Gram matrix is summed (two per compute unit on a 256-CU chip)
    dim3 grid(quant_sketch_rows_blocks(rows));
    const size_t lds = (size_t)16 * (cols + ((68 - (cols & 63)) & 63)) * sizeof(float);
#define LRQ_QSR(NSV) case NSV: hipLaunchKernelGGL((quant_sketch_rows_kernel<NSV>), grid, dim3(512), lds, st, X, ldx, rows, cols, q, W, Y, gpart, amax, lam_out, s_out, codes); break
    switch (ceil_div(cols, 32)) {
        LRQ_QSR(1); LRQ_QSR(2); LRQ_QSR(3); LRQ_QSR(4); LRQ_QSR(5); LRQ_QSR(6); LRQ_QSR(7); LRQ_QSR(8); LRQ_QSR(9); LRQ_QSR(10);
        LRQ_QSR(11); LRQ_QSR(12); LRQ_QSR(13); LRQ_QSR(14); LRQ_QSR(15); LRQ_QSR(16); LRQ_QSR(17); LRQ_QSR(18);
        default: return LRQMM_ERR_UNSUPPORTED;
    }
#undef LRQ_QSR
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_resid_mul_t(const float* X, int ldx, int rows, int cols, int axis, const float* lam, const float* s,
                       QuantParams q, const float* W, int LP, PassPlan plan, float* partial,
                       hipStream_t st, int planes) {
    const bool vec = (cols % 4 == 0) && (ldx % 4 == 0) && aligned16(X);
    dim3 grid(ceil_div(cols, 64), plan.splits);
    NT_SWITCH(LP / 16, (dispatch_t<NT_>(axis, vec, planes, grid, st, X, ldx, rows, cols, lam, s, q, W, plan.chunk, partial)));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_codes_mul_n2(const int8_t* codesA, int rowsA, const float* WA, const uint16_t* WA3, PassPlan planA,
                        float* partialA, const int8_t* codesB, int rowsB, const float* WB, const uint16_t* WB3,
                        PassPlan planB, float* partialB, int K, int Kp, int LP, hipStream_t st, int planes) {
    const bool fast = (K % 16 == 0) && K >= 16 && ((uintptr_t)codesA % 16 == 0) && ((uintptr_t)codesB % 16 == 0);
    if (fast) {
        CodesJobBf16 j0 = {codesA, WA3, partialA, rowsA, planA.chunk, planA.splits};
        CodesJobBf16 j1 = {codesB, WB3, partialB, rowsB, planB.chunk, planB.splits};
        // short rows, one tile of factor columns, no split of the reduction: the persistent kernel
        const size_t lds_rows = (size_t)planes * 16 * (Kp + 8) * sizeof(uint16_t);
        if (LP == 16 && K <= 640 && planA.splits == 1 && planB.splits == 1 && lds_rows <= 64 * 1024) {
            int dev = 0, cus = 0;
            if (hipGetDevice(&dev) != hipSuccess ||
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
                return LRQMM_ERR_HIP;
            dim3 g2(min(ceil_div(ceil_div(max(rowsA, rowsB), 16), 8), 2 * cus), 1, 2);
            const int nc = ceil_div(K, 64);
#define LRQ_CMR(PLV, NCV) hipLaunchKernelGGL((codes_mul_rows_kernel<PLV, NCV>), g2, dim3(512), lds_rows, st, j0, j1, K, Kp)
#define LRQ_CMR_NC(PLV) do { if (nc <= 2) LRQ_CMR(PLV, 2); else if (nc <= 4) LRQ_CMR(PLV, 4); else if (nc <= 6) LRQ_CMR(PLV, 6); \
            else if (nc <= 8) LRQ_CMR(PLV, 8); else LRQ_CMR(PLV, 10); } while (0)
            if (planes == 2) LRQ_CMR_NC(2); else if (planes == 1) LRQ_CMR_NC(1); else LRQ_CMR_NC(3);
#undef LRQ_CMR_NC
#undef LRQ_CMR
            LRQ_CHECK_LAUNCH();
            return LRQMM_OK;
        }
        // Up to 48 factor columns a workgroup takes 128 rows (two 16-row tiles per wave): with the 256-deep slabs
        // two or three workgroups share a CU and cover each other's load and staging phases (4096^2 codes, 32
        // columns: 17.5 -> 16.0 us; 16 columns: 13.8 -> 11.3 us; same bits).  Wider factors keep 256 rows.
#define LRQ_CM(PLV, MTV) NT_SWITCH(LP / 16, hipLaunchKernelGGL((codes_mul_bf16_kernel<NT_, PLV, MTV>), dim3(ceil_div(max(rowsA, rowsB), 64 * MTV), max(planA.splits, planB.splits), 2), dim3(256), 0, st, j0, j1, K, Kp))
#define LRQ_CM_PL(MTV) do { if (planes == 2) { LRQ_CM(2, MTV); } else if (planes == 1) { LRQ_CM(1, MTV); } else { LRQ_CM(3, MTV); } } while (0)
        if (LP <= 48) LRQ_CM_PL(2); else LRQ_CM_PL(4);
#undef LRQ_CM_PL
#undef LRQ_CM
        LRQ_CHECK_LAUNCH();
        return LRQMM_OK;
    }
    const bool vec = (K % 4 == 0) && ((uintptr_t)codesA % 4 == 0) && ((uintptr_t)codesB % 4 == 0);
    CodesJob j0 = {codesA, WA, partialA, rowsA, planA.chunk, planA.splits};
    CodesJob j1 = {codesB, WB, partialB, rowsB, planB.chunk, planB.splits};
    dim3 grid(ceil_div(max(rowsA, rowsB), 64), max(planA.splits, planB.splits), 2);
    NT_SWITCH(LP / 16, (dispatch_c<NT_>(vec, grid, st, j0, j1, K)));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
