// Integer GEMM on the int8 matrix cores with a fused dequantize + low-rank
// compensation epilogue (paper: Eq. (INTGEMM), Eq. (QUANTGEMM); Algorithm 2, integer product,
// dequantization and compensation steps).
//
// The three compensation terms of Algorithm 2 are never formed as M x N matrices:
//   RC1 + RC2 + RC3 = (U Sig)(Vt B~) + (A~ W)(Gam Zt) + (U Sig)(Vt W)(Gam Zt)
//                   = [U Sig | A~ W] . [Vt B~ + (Vt W) Gam Zt ; Gam Zt]
// i.e. a rank-2r update Lp . Rp^T applied to each output tile while its int32
// accumulators are still in registers.
//
// Main loop: 128x128 workgroup tile, 4 waves in 2x2, each wave 64x64 as 2x2
// v_mfma_i32_32x32x32_i8 tiles; both operands are K-major (A codes M x K, B codes
// stored transposed N x K), staged through double-buffered LDS with a padded row
// stride (80 B) that makes the 16-byte operand reads bank-conflict free.
// 32x32 accumulator layout (lane l, register v): row 8*(v/4) + 4*(l/32) + v%4,
// column l%32 -- identical for the i32 and f32 32x32 MFMAs, which lets the
// epilogue continue on the same registers with v_mfma_f32_32x32x2_f32.
#include "kernels.h"

#define TM 128
#define TN 128
#define BK 64
#ifndef LDS_STRIDE
#define LDS_STRIDE 80
#endif

// 16 code bytes of one operand row.  The vector path (K % 16 == 0) is branch free: clamped
// address, then a select; a load under a branch would make the compiler drain every
// outstanding load each iteration and defeat the prefetch ring.
template <bool VEC>
__device__ __forceinline__ uint4 load16b(const int8_t* __restrict__ base, int row, int nrows, int K,
                                         int k) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (VEC) {
        const int rc = min(row, nrows - 1), kc = min(k, K - 16);
        const uint4 t = *reinterpret_cast<const uint4*>(base + (size_t)rc * K + kc);
        const bool ok = row < nrows && k < K;
        v.x = ok ? t.x : 0u;
        v.y = ok ? t.y : 0u;
        v.z = ok ? t.z : 0u;
        v.w = ok ? t.w : 0u;
    } else {
        if (row >= nrows) return v;
        const int8_t* p = base + (size_t)row * K + k;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int b = 0; b < 16; ++b)
            if (k + b < K) w[b >> 2] |= (uint32_t)(uint8_t)p[b] << (8 * (b & 3));
        v = make_uint4(w[0], w[1], w[2], w[3]);
    }
    return v;
}

// Last step of Algorithm 2 on one element: D <- alpha * value + beta * D (D is not read when
// beta == 0, so it may then hold anything).
__device__ __forceinline__ void store_out(const GemmOut& out, int row, int col, float value) {
    float* p = out.C + (size_t)row * out.ldc + col;
    float o = out.alpha * value;
    if (out.beta != 0.f) o = o + out.beta * *p;
    *p = o;
}

// Workgroup ids are dealt round-robin to the 8 XCDs, each with an L2 of its own.  The tile grid
// is cut into gm x gn = 8 rectangles, one per XCD, as square as the tile counts allow, so that an
// XCD fetches tiles_m/gm row panels of A and tiles_n/gn of B instead of whole bands (at 16 x 16
// tiles: 8 + 4 panels per XCD instead of 2 + 16).  Tile counts that are no multiple of 8 keep
// the launch order.
__device__ __forceinline__ int xcd_tile(int id, int tiles_n, int ntiles) {
    if (ntiles & 7) return id;
    const int tiles_m = ntiles / tiles_n;
    int gm = 0, best = 0x7fffffff;
#pragma unroll
    for (int g = 1; g <= 8; g *= 2) {
        const int h = 8 / g;
        if (tiles_m % g == 0 && tiles_n % h == 0) {
            const int cost = tiles_m / g + tiles_n / h;
            if (cost < best) { best = cost; gm = g; }
        }
    }
    // ntiles % 8 == 0 guarantees that one of the four cuts divides both tile counts
    const int gn = 8 / gm, bn = tiles_n / gn, bm = tiles_m / gm;
    const int x = id & 7, j = id >> 3;
    // Inside its rectangle an XCD works through sub-blocks of 32 tiles (one per CU, the tiles that run at the
    // same time), 4 x 8 or 8 x 4 where the rectangle allows: the panels that one round of tiles streams through
    // the L2 are then 12 instead of bn + 32 / bn.
    int r = j / bn, c = j % bn;
    if (bm * bn > 32) {
        const int sm = (bm % 4 == 0 && bn % 8 == 0) ? 4 : ((bm % 8 == 0 && bn % 4 == 0) ? 8 : 0);
        if (sm) {
            const int sn = 32 / sm, sub = j >> 5, in = j & 31, per_row = bn / sn;
            r = (sub / per_row) * sm + in / sn;
            c = (sub % per_row) * sn + in % sn;
        }
    }
    return ((x / gn) * bm + r) * tiles_n + (x % gn) * bn + c;
}

// NTW: 32-column MFMA tiles per wave along N.  2: the 128 x 128 tile (waves 2 x 2, each 64 x 64); 1: a 128 x 64 tile
// (each wave 64 x 32) for outputs of at most 64 columns, e.g. a convolution with 64 output channels as a product --
// on a 128-wide tile half the matrix-core work and half of B's LDS tile would be zeros.
template <bool VEC, bool COMP, bool WCINT, int NTW = 2>
__global__ __launch_bounds__(256) void int8_gemm_kernel(int M, int N, int K,
                                                        const int8_t* __restrict__ Aq,
                                                        const int8_t* __restrict__ BqT,
                                                        const float* __restrict__ sA,
                                                        const float* __restrict__ sB,
                                                        const float* __restrict__ Lp,
                                                        const float* __restrict__ Rp, int R2P,
                                                        GemmOut out,
                                                        int32_t* __restrict__ Cint, int tiles_n,
                                                        int ntiles) {
    __shared__ __align__(16) int8_t As[2][TM * LDS_STRIDE];
    constexpr int TNW = 64 * NTW;       // tile width
    __shared__ __align__(16) int8_t Bs[2][TNW * LDS_STRIDE];
    const int tile = xcd_tile(blockIdx.x, tiles_n, ntiles);
    const int m0 = (tile / tiles_n) * TM, n0 = (tile % tiles_n) * TNW;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    v16i acc[2][NTW];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NTW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // staging: 512 16-byte chunks per operand tile, two per thread.  Global loads run three K-tiles ahead of the
    // matrix cores in a ring of three sets of named registers (as arrays they would go to scratch memory): with
    // one tile of lookahead every iteration waited for a global load, which short reductions (K = 576 for the
    // conv-shaped workload: nine tiles) never amortize.  Tiles past the end load zeros and are never stored.
    const int srow0 = tid >> 2, skc = (tid & 3) * 16;
#define LRQ_DECL(S) uint4 S##a0, S##a1, S##b0, S##b1
#define LRQ_GLOAD(S, k0)                                                   \
    S##a0 = load16b<VEC>(Aq, m0 + srow0, M, K, (k0) + skc);                \
    S##b0 = load16b<VEC>(BqT, n0 + srow0, N, K, (k0) + skc);               \
    S##a1 = load16b<VEC>(Aq, m0 + srow0 + 64, M, K, (k0) + skc);           \
    if (NTW == 2) S##b1 = load16b<VEC>(BqT, n0 + srow0 + 64, N, K, (k0) + skc);
#define LRQ_SSTORE(S, buf)                                                                  \
    *reinterpret_cast<uint4*>(&As[buf][srow0 * LDS_STRIDE + skc]) = S##a0;                  \
    *reinterpret_cast<uint4*>(&Bs[buf][srow0 * LDS_STRIDE + skc]) = S##b0;                  \
    *reinterpret_cast<uint4*>(&As[buf][(srow0 + 64) * LDS_STRIDE + skc]) = S##a1;           \
    if (NTW == 2) *reinterpret_cast<uint4*>(&Bs[buf][(srow0 + 64) * LDS_STRIDE + skc]) = S##b1;
    LRQ_DECL(r0);
    LRQ_DECL(r1);
    LRQ_DECL(r2);
    auto compute = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < BK / 32; ++kk) {
            v4i af[2], bf[NTW];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                af[mt] = *reinterpret_cast<const v4i*>(
                    &As[buf][(wm * 64 + mt * 32 + l32) * LDS_STRIDE + kk * 32 + lh * 16]);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt)
                bf[nt] = *reinterpret_cast<const v4i*>(
                    &Bs[buf][(wn * 32 * NTW + nt * 32 + l32) * LDS_STRIDE + kk * 32 + lh * 16]);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[mt], bf[nt], acc[mt][nt], 0, 0, 0);
        }
    };
    const int nk = (K + BK - 1) / BK;
    LRQ_GLOAD(r0, 0);
    LRQ_GLOAD(r1, BK);
    LRQ_GLOAD(r2, 2 * BK);
    LRQ_SSTORE(r0, 0);
    __syncthreads();
    // iteration i: the set that held tile i is free -> load tile i + 3; compute tile i; publish tile i + 1
#define LRQ_GEMM_STEP(J, SCUR, SNEXT)                       \
    if (kt + J < nk) {                                      \
        const int i = kt + J;                               \
        LRQ_GLOAD(SCUR, (i + 3) * BK);                      \
        compute(i & 1);                                     \
        if (i + 1 < nk) { LRQ_SSTORE(SNEXT, (i + 1) & 1); } \
        __syncthreads();                                    \
    }
    for (int kt = 0; kt < nk; kt += 3) {
        LRQ_GEMM_STEP(0, r0, r1)
        LRQ_GEMM_STEP(1, r1, r2)
        LRQ_GEMM_STEP(2, r2, r0)
    }
#undef LRQ_GEMM_STEP
#undef LRQ_DECL
#undef LRQ_GLOAD
#undef LRQ_SSTORE

    // ---- epilogue: dequantize, rank-2r update, store ----
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int rbase = m0 + wm * 64 + mt * 32;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int col = n0 + wn * 32 * NTW + nt * 32 + l32;
            const bool col_ok = col < N;
            const float sb = col_ok ? sB[col] : 0.f;
            v16f f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rbase + 8 * (v >> 2) + 4 * lh + (v & 3);
                const float sa = (row < M) ? sA[row] : 0.f;
                if (WCINT && row < M && col_ok) Cint[(size_t)row * N + col] = acc[mt][nt][v];
                f[v] = ((float)acc[mt][nt][v] * sa) * sb;
            }
            if (COMP) {
                const int lrow = rbase + l32;
                const float* lp = Lp + (size_t)(lrow < M ? lrow : 0) * R2P + 4 * lh;
                const float* rp = Rp + (size_t)(col_ok ? col : 0) * R2P + 4 * lh;
                const bool lok = lrow < M;
                for (int t0 = 0; t0 < R2P; t0 += 8) {
                    float4 a4 = lok ? *reinterpret_cast<const float4*>(lp + t0) : make_float4(0.f, 0.f, 0.f, 0.f);
                    float4 b4 = col_ok ? *reinterpret_cast<const float4*>(rp + t0) : make_float4(0.f, 0.f, 0.f, 0.f);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4.x, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4.y, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4.z, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4.w, f, 0, 0, 0);
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rbase + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (row < M && col_ok) store_out(out, row, col, f[v]);
            }
        }
    }
}

// Large-tile variant for big problems: 256x256 workgroup tile, one workgroup of 8 waves per
// CU (two waves per SIMD, so one wave's LDS/global waits and barrier stalls are covered by
// the other's MFMAs).  Waves form a 4x2 grid, each 64x128 = 2x4 MFMA tiles (128 accumulator
// registers); per 32-deep MFMA step a wave reads 6 KB of operands from LDS for 8 MFMAs.  A staged
// tile is 128 deep: 144 KB of LDS for the two buffers of both operands.
#define BTM 256
#define BTN 256
#ifndef BBK
#define BBK 128                 // K depth of one staged tile of the large-tile kernel
#endif
#ifndef LRQ_GRING
#define LRQ_GRING 2             // register sets of global loads in flight (tiles ahead of the matrix cores)
#endif
#define BSTRIDE (BBK + 16)      // padded LDS row stride, conflict-free 16-byte reads
#define BCHUNKS (BBK / 16)      // 16-byte chunks per staged row
#define BROWS (512 / BCHUNKS)   // rows covered by one pass of the 512 threads
#define BLOADS (256 / BROWS)    // staged 16-byte chunks per thread and operand
// FULL: M, N multiples of 256 and K a multiple of the tile depth -- operand loads carry no guard at all, so
// nothing consumes a loaded register before it is written to LDS two iterations later.
// SPLITK (raw sums only, FULL shapes): workgroups [0, full_tiles) compute one tile each as usual;
// the remaining ntiles - full_tiles tiles are cut into `slices` ranges of K, one workgroup per
// (tile, range), which leave their int32 partial sums in `part` ([tile][range][256][256]) for
// sum_tile_slices_kernel (integer addition: exact whatever the cut).
template <bool VEC, bool COMP, bool WCINT, bool FULL, bool SPLITK = false>
__global__ __launch_bounds__(512, 1) void int8_gemm256_kernel(int M, int N, int K,
                                                              const int8_t* __restrict__ Aq,
                                                              const int8_t* __restrict__ BqT,
                                                              const float* __restrict__ sA,
                                                              const float* __restrict__ sB,
                                                              const float* __restrict__ Lp,
                                                              const float* __restrict__ Rp, int R2P,
                                                              GemmOut out,
                                                              int32_t* __restrict__ Cint, int tiles_n,
                                                              int ntiles, int full_tiles, int slices,
                                                              int32_t* __restrict__ part) {
    float* __restrict__ C = out.C;
    __shared__ __align__(16) int8_t As[2][BTM * BSTRIDE];
    __shared__ __align__(16) int8_t Bs[2][BTN * BSTRIDE];
    int wg = blockIdx.x, kt0 = 0, nk = (K + BBK - 1) / BBK;
    bool partial = false;
    if constexpr (SPLITK) {
        if (wg >= full_tiles) {
            const int e = wg - full_tiles, lt = e / slices, sl = e - lt * slices;
            wg = full_tiles + lt;
            part += (size_t)e * (BTM * BTN);
            kt0 = (int)((long long)sl * nk / slices);
            nk = (int)((long long)(sl + 1) * nk / slices) - kt0;
            partial = true;
        }
    }
    const int tile = xcd_tile(wg, tiles_n, ntiles);
    const int m0 = (tile / tiles_n) * BTM, n0 = (tile % tiles_n) * BTN;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    v16i acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // staging: 2048 16-byte chunks per operand tile, four per thread.  Global loads run two 128-deep
    // K-tiles ahead of the matrix cores in a ring of two register sets (a tile's MFMA time is below
    // global-load latency, so one tile of lookahead stalls every iteration); LDS holds the current
    // and the next tile.  (Measured against 64-deep tiles with a ring of three -- the same depth in
    // flight, twice the barriers per product: 84 against 91 us at 4096^3, 3.99 against 4.29 ms at 16384^3.)
    const int srow0 = tid / BCHUNKS, skc = (tid % BCHUNKS) * 16;
    // The register sets are individually named scalars (not arrays passed by reference):
    // that keeps them in VGPRs; as arrays they were demoted to scratch memory.
    auto ldA = [&](int u, int k0) -> uint4 {
        if (FULL)   // tiles past the end of K are loaded (clamped) but never stored or used
            return *reinterpret_cast<const uint4*>(Aq + (size_t)(m0 + srow0 + BROWS * u) * K + min(k0, K - BBK) + skc);
        return load16b<VEC>(Aq, m0 + srow0 + BROWS * u, M, K, k0 + skc);
    };
    auto ldB = [&](int u, int k0) -> uint4 {
        if (FULL)
            return *reinterpret_cast<const uint4*>(BqT + (size_t)(n0 + srow0 + BROWS * u) * K + min(k0, K - BBK) + skc);
        return load16b<VEC>(BqT, n0 + srow0 + BROWS * u, N, K, k0 + skc);
    };
    auto stA = [&](int u, int buf, uint4 v) {
        *reinterpret_cast<uint4*>(&As[buf][(srow0 + BROWS * u) * BSTRIDE + skc]) = v;
    };
    auto stB = [&](int u, int buf, uint4 v) {
        *reinterpret_cast<uint4*>(&Bs[buf][(srow0 + BROWS * u) * BSTRIDE + skc]) = v;
    };
#define LRQ_DECL(S) uint4 S##a0, S##a1, S##a2, S##a3, S##b0, S##b1, S##b2, S##b3
#define LRQ_GLOAD(S, k0)                                                   \
    S##a0 = ldA(0, k0); S##b0 = ldB(0, k0); S##a1 = ldA(1, k0); S##b1 = ldB(1, k0); \
    if (BLOADS == 4) { S##a2 = ldA(2, k0); S##b2 = ldB(2, k0); S##a3 = ldA(3, k0); S##b3 = ldB(3, k0); }
#define LRQ_SSTORE(S, buf)                                                         \
    stA(0, buf, S##a0); stB(0, buf, S##b0); stA(1, buf, S##a1); stB(1, buf, S##b1); \
    if (BLOADS == 4) { stA(2, buf, S##a2); stB(2, buf, S##b2); stA(3, buf, S##a3); stB(3, buf, S##b3); }
    LRQ_DECL(r0);
    LRQ_DECL(r1);
#if LRQ_GRING == 3
    LRQ_DECL(r2);
#endif
    auto compute = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < BBK / 32; ++kk) {
            v4i af[2], bf[4];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                af[mt] = *reinterpret_cast<const v4i*>(
                    &As[buf][(wm * 64 + mt * 32 + l32) * BSTRIDE + kk * 32 + lh * 16]);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                bf[nt] = *reinterpret_cast<const v4i*>(
                    &Bs[buf][(wn * 128 + nt * 32 + l32) * BSTRIDE + kk * 32 + lh * 16]);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[mt], bf[nt], acc[mt][nt], 0, 0, 0);
        }
    };
    LRQ_GLOAD(r0, kt0 * BBK);
    LRQ_GLOAD(r1, (kt0 + 1) * BBK);
#if LRQ_GRING == 3
    LRQ_GLOAD(r2, (kt0 + 2) * BBK);
#endif
    LRQ_SSTORE(r0, 0);
    __syncthreads();
    // iteration i: the set that held tile i is free -> load tile i + LRQ_GRING; compute tile i; publish tile i+1
#define LRQ_GEMM_STEP(J, SCUR, SNEXT)                  \
    if (kt + J < nk) {                                 \
        const int i = kt + J;                          \
        LRQ_GLOAD(SCUR, (kt0 + i + LRQ_GRING) * BBK);       \
        compute(i & 1);                                \
        if (i + 1 < nk) { LRQ_SSTORE(SNEXT, (i + 1) & 1); } \
        __syncthreads();                               \
    }
#if LRQ_GRING == 3
    for (int kt = 0; kt < nk; kt += 3) {
        LRQ_GEMM_STEP(0, r0, r1)
        LRQ_GEMM_STEP(1, r1, r2)
        LRQ_GEMM_STEP(2, r2, r0)
    }
#else
    for (int kt = 0; kt < nk; kt += 2) {
        LRQ_GEMM_STEP(0, r0, r1)
        LRQ_GEMM_STEP(1, r1, r0)
    }
#endif
#undef LRQ_GEMM_STEP
#undef LRQ_DECL
#undef LRQ_GLOAD
#undef LRQ_SSTORE

    // ---- epilogue: dequantize, rank-2r update, store ----
    // C == nullptr: only the raw int32 sums are wanted (the dequantization and the update then
    // run later, in rank_update_kernel), and the step vectors are not read.
    const bool want_c = C != nullptr;
    // Panels of up to 64 columns: the tile's 256 rows of Lp and of Rp are staged in the LDS that the operand
    // tiles have left (whole-row loads; rows past the end as zeros; row stride R2P + 4 floats: conflict-free
    // 16-byte reads), instead of 32 cache lines per load instruction from global memory.  Same values, same
    // order of the products.
    const bool staged = COMP && R2P <= 64;
    const int LDP = R2P + 4;
    float* const Ls = reinterpret_cast<float*>(&As[0][0]);
    float* const Rs = reinterpret_cast<float*>(&Bs[0][0]);
    static_assert(2 * BTM * BSTRIDE >= 256 * 68 * 4, "a 64-column panel tile fits an operand's LDS");
    if (staged) {
        __syncthreads();        // every wave has read its last operand fragments
        const int q4 = R2P / 4;
        for (int idx = tid; idx < 256 * q4; idx += 512) {
            const int rr = idx / q4, c4 = idx - rr * q4;
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 lv = m0 + rr < M ? *reinterpret_cast<const float4*>(Lp + (size_t)(m0 + rr) * R2P + 4 * c4) : z;
            const float4 rv = n0 + rr < N ? *reinterpret_cast<const float4*>(Rp + (size_t)(n0 + rr) * R2P + 4 * c4) : z;
            *reinterpret_cast<float4*>(Ls + rr * LDP + 4 * c4) = lv;
            *reinterpret_cast<float4*>(Rs + rr * LDP + 4 * c4) = rv;
        }
        __syncthreads();
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int rbase = m0 + wm * 64 + mt * 32;
        const int lrow = rbase + l32;
        const bool lok = lrow < M;
        const float* lp = COMP ? Lp + (size_t)(lok ? lrow : 0) * R2P + 4 * lh : nullptr;
        const float* lps = Ls + (wm * 64 + mt * 32 + l32) * LDP + 4 * lh;
        float sa[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = rbase + 8 * (v >> 2) + 4 * lh + (v & 3);
            sa[v] = (want_c && row < M) ? sA[row] : 0.f;
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int col = n0 + wn * 128 + nt * 32 + l32;
            const bool col_ok = col < N;
            const float sb = (want_c && col_ok) ? sB[col] : 0.f;
            v16f f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rbase + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (WCINT && row < M && col_ok) {
                    if (SPLITK && partial) part[(row - m0) * BTN + (col - n0)] = acc[mt][nt][v];
                    else Cint[(size_t)row * N + col] = acc[mt][nt][v];
                }
                f[v] = ((float)acc[mt][nt][v] * sa[v]) * sb;
            }
            if (COMP && staged) {
                const float* rps = Rs + (wn * 128 + nt * 32 + l32) * LDP + 4 * lh;
                for (int t0 = 0; t0 < R2P; t0 += 8) {
                    const float4 a4 = *reinterpret_cast<const float4*>(lps + t0);
                    const float4 b4 = *reinterpret_cast<const float4*>(rps + t0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4.x, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4.y, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4.z, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4.w, f, 0, 0, 0);
                }
            } else if (COMP) {
                const float* rp = Rp + (size_t)(col_ok ? col : 0) * R2P + 4 * lh;
                for (int t0 = 0; t0 < R2P; t0 += 8) {
                    float4 a4 = lok ? *reinterpret_cast<const float4*>(lp + t0) : make_float4(0.f, 0.f, 0.f, 0.f);
                    float4 b4 = col_ok ? *reinterpret_cast<const float4*>(rp + t0) : make_float4(0.f, 0.f, 0.f, 0.f);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4.x, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4.y, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4.z, f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4.w, f, 0, 0, 0);
                }
            }
            if (want_c) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = rbase + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < M && col_ok) store_out(out, row, col, f[v]);
                }
            }
        }
    }
}

// The epilogue of the GEMM as a kernel of its own, for the schedule in which the integer
// product runs early (next to the small kernels of the factorizations) and leaves its raw
// int32 sums in C's memory: C <- float(Cint) sA_i sB_j + Lp . Rp^T in place, with the same
// products accumulated in the same order as the fused epilogue (bit-identical results).
// 128x128 tile per workgroup, 4 waves of 64x64 (2x2 MFMA tiles).  The MFMA runs on the
// transposed tile (Rp rows as the A operand, Lp rows as B), so that a lane owns ONE row of C
// and four groups of 4 consecutive columns: C is read and written with 16-byte accesses
// (needs N % 4 == 0).  A wave first issues all its loads -- its four tiles of sums and, per 64
// panel columns, the panel rows of both row tiles and both column tiles -- without branches,
// and then runs the four accumulation chains interleaved, so neither load latency nor the
// latency of dependent MFMAs is exposed.
__global__ __launch_bounds__(256, 2) void rank_update_kernel(int M, int N, float* __restrict__ C,
                                                          const float* __restrict__ sA,
                                                          const float* __restrict__ sB,
                                                          const float* __restrict__ Lp,
                                                          const float* __restrict__ Rp, int R2P, int tiles_n,
                                                          float alpha) {
    __shared__ __align__(16) float pl[2][128][68];      // Lp and Rp rows of the tile, 64 columns, padded
    const int m0 = (blockIdx.x / tiles_n) * 128, n0 = (blockIdx.x % tiles_n) * 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int rb0 = m0 + wm * 64, cb0 = n0 + wn * 64;
    // D[i][j] of tile (mt, nt): j = l32 is the row of C, i = 8 g + 4 lh + e its column (v = 4 g + e)
    int row[2], colb[2][4];         // this lane's C rows and first columns of its groups (clamped)
    bool row_ok[2], col_ok[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        row_ok[t] = rb0 + t * 32 + l32 < M;
        row[t] = min(rb0 + t * 32 + l32, M - 1);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = cb0 + t * 32 + 8 * g + 4 * lh;
            col_ok[t][g] = c < N;
            colb[t][g] = min(c, N - 4);
        }
    }
    v16f f[2][2];
    int4 raw[2][2][4];
    float4 sb[2][4];
    float sa[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        sa[t] = sA[row[t]];
#pragma unroll
        for (int g = 0; g < 4; ++g) sb[t][g] = *reinterpret_cast<const float4*>(sB + colb[t][g]);
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                raw[mt][nt][g] = *reinterpret_cast<const int4*>(C + (size_t)row[mt] * N + colb[nt][g]);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f[mt][nt][4 * g + 0] = ((float)raw[mt][nt][g].x * sa[mt]) * sb[nt][g].x;
                f[mt][nt][4 * g + 1] = ((float)raw[mt][nt][g].y * sa[mt]) * sb[nt][g].y;
                f[mt][nt][4 * g + 2] = ((float)raw[mt][nt][g].z * sa[mt]) * sb[nt][g].z;
                f[mt][nt][4 * g + 3] = ((float)raw[mt][nt][g].w * sa[mt]) * sb[nt][g].w;
            }
    // The panel rows of the tile go through LDS, 64 columns at a time: the workgroup loads each row once,
    // 16 lanes per 256-byte row, instead of every wave fetching its operands with 16-byte loads that touch
    // 32 cache lines per instruction (measured on this access pattern: 36 instead of 41 us).
    for (int t0 = 0; t0 < R2P; t0 += 64) {      // R2P % 8 == 0
        if (t0 > 0) __syncthreads();            // the previous chunk is no longer read
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int idx = threadIdx.x + 256 * i, r = idx >> 4, c = (idx & 15) * 4;
            const int col = t0 + c;
            const bool in = col < R2P;           // panel columns past R2P enter as zeros
            const int cc = min(col, R2P - 4);
            // rows / columns past the end re-read the last one (never stored)
            const float4 x = *reinterpret_cast<const float4*>(Lp + (size_t)min(m0 + r, M - 1) * R2P + cc);
            const float4 y = *reinterpret_cast<const float4*>(Rp + (size_t)min(n0 + r, N - 1) * R2P + cc);
            *reinterpret_cast<float4*>(&pl[0][r][c]) = make_float4(in ? x.x : 0.f, in ? x.y : 0.f, in ? x.z : 0.f, in ? x.w : 0.f);
            *reinterpret_cast<float4*>(&pl[1][r][c]) = make_float4(in ? y.x : 0.f, in ? y.y : 0.f, in ? y.z : 0.f, in ? y.w : 0.f);
        }
        __syncthreads();
        float4 a4[2][8], b4[2][8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                a4[t][u] = *reinterpret_cast<const float4*>(&pl[0][wm * 64 + t * 32 + l32][8 * u + 4 * lh]);
                b4[t][u] = *reinterpret_cast<const float4*>(&pl[1][wn * 64 + t * 32 + l32][8 * u + 4 * lh]);
            }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {    // A operand: panel row of the column, B operand: of the row
                    f[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b4[nt][u].x, a4[mt][u].x, f[mt][nt], 0, 0, 0);
                    f[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b4[nt][u].y, a4[mt][u].y, f[mt][nt], 0, 0, 0);
                    f[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b4[nt][u].z, a4[mt][u].z, f[mt][nt], 0, 0, 0);
                    f[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b4[nt][u].w, a4[mt][u].w, f[mt][nt], 0, 0, 0);
                }
        }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if (row_ok[mt] && col_ok[nt][g])
                    *reinterpret_cast<float4*>(C + (size_t)row[mt] * N + colb[nt][g]) =
                        make_float4(alpha * f[mt][nt][4 * g + 0], alpha * f[mt][nt][4 * g + 1],
                                    alpha * f[mt][nt][4 * g + 2], alpha * f[mt][nt][4 * g + 3]);
}

// The same update for wide panels (2r > 64), where the float32 matrix cores are the limit (4 R2P flops per output:
// 0.87 ms of matrix-core time at 16384^2 and r = 64).  The panel rows are split into three bfloat16 planes while
// they are staged in LDS (exact: a float32 is the sum of its three planes) and the six plane products of weight
// >= 2^-16 run on v_mfma_f32_32x32x16_bf16 with float32 accumulation: 192 instead of 512 matrix-core cycles per
// 16 panel columns.  Float32-equivalent, but a different rounding order than the float32 instructions: results
// are not bit-identical to the fused epilogue.  Operand layout (lane l): A[i = l%32][k = 8(l/32) .. +8],
// B[k = 8(l/32) .. +8][j = l%32]; D as for the 32x32 float32 instruction.
#define RU_KC 32        // panel columns per LDS chunk
#define RU_LD 40        // plane row stride in bfloat16 (80 bytes: conflict-free 16-byte reads)
__global__ __launch_bounds__(256, 2) void rank_update_bf16_kernel(int M, int N, float* __restrict__ C,
                                                                  const float* __restrict__ sA,
                                                                  const float* __restrict__ sB,
                                                                  const float* __restrict__ Lp,
                                                                  const float* __restrict__ Rp, int R2P, int tiles_n,
                                                                  float alpha) {
    __shared__ __align__(16) uint16_t pp[2][3][128 * RU_LD];     // [Lp | Rp][plane][row][column of the chunk]
    const int m0 = (blockIdx.x / tiles_n) * 128, n0 = (blockIdx.x % tiles_n) * 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int rb0 = m0 + wm * 64, cb0 = n0 + wn * 64;
    int row[2], colb[2][4];
    bool row_ok[2], col_ok[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        row_ok[t] = rb0 + t * 32 + l32 < M;
        row[t] = min(rb0 + t * 32 + l32, M - 1);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = cb0 + t * 32 + 8 * g + 4 * lh;
            col_ok[t][g] = c < N;
            colb[t][g] = min(c, N - 4);
        }
    }
    v16f f[2][2];
    {
        int4 raw[2][2][4];
        float4 sb[2][4];
        float sa[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sa[t] = sA[row[t]];
#pragma unroll
            for (int g = 0; g < 4; ++g) sb[t][g] = *reinterpret_cast<const float4*>(sB + colb[t][g]);
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    raw[mt][nt][g] = *reinterpret_cast<const int4*>(C + (size_t)row[mt] * N + colb[nt][g]);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f[mt][nt][4 * g + 0] = ((float)raw[mt][nt][g].x * sa[mt]) * sb[nt][g].x;
                    f[mt][nt][4 * g + 1] = ((float)raw[mt][nt][g].y * sa[mt]) * sb[nt][g].y;
                    f[mt][nt][4 * g + 2] = ((float)raw[mt][nt][g].z * sa[mt]) * sb[nt][g].z;
                    f[mt][nt][4 * g + 3] = ((float)raw[mt][nt][g].w * sa[mt]) * sb[nt][g].w;
                }
    }
    for (int t0 = 0; t0 < R2P; t0 += RU_KC) {       // R2P % 8 == 0
        if (t0 > 0) __syncthreads();                // the previous chunk is no longer read
        // 2 panels x 128 rows x 4 groups of 8 columns = 1024 units, four per thread: load, split, store the planes
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int unit = threadIdx.x + 256 * i;
            const int pnl = unit >> 9, r = (unit >> 2) & 127, c8 = (unit & 3) * 8;
            const float* src = pnl == 0 ? Lp + (size_t)min(m0 + r, M - 1) * R2P : Rp + (size_t)min(n0 + r, N - 1) * R2P;
            float v[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {           // rows / columns past the end re-read the last one (never stored)
                const int col = t0 + c8 + 4 * h;
                const bool in = col < R2P;          // panel columns past R2P enter as zeros
                const float4 x = *reinterpret_cast<const float4*>(src + min(col, R2P - 4));
                v[4 * h + 0] = in ? x.x : 0.f; v[4 * h + 1] = in ? x.y : 0.f;
                v[4 * h + 2] = in ? x.z : 0.f; v[4 * h + 3] = in ? x.w : 0.f;
            }
            const Planes3 pl = split_planes<3>(v);
            *reinterpret_cast<v8bf16*>(&pp[pnl][0][r * RU_LD + c8]) = pl.p1;
            *reinterpret_cast<v8bf16*>(&pp[pnl][1][r * RU_LD + c8]) = pl.p2;
            *reinterpret_cast<v8bf16*>(&pp[pnl][2][r * RU_LD + c8]) = pl.p3;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < RU_KC / 16; ++u) {
            Planes3 a[2], b[2];     // a: Lp rows of the two row tiles (B operand), b: Rp rows of the two column tiles (A operand)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int oa = (wm * 64 + t * 32 + l32) * RU_LD + 16 * u + 8 * lh;
                const int ob = (wn * 64 + t * 32 + l32) * RU_LD + 16 * u + 8 * lh;
                a[t].p1 = *reinterpret_cast<const v8bf16*>(&pp[0][0][oa]);
                a[t].p2 = *reinterpret_cast<const v8bf16*>(&pp[0][1][oa]);
                a[t].p3 = *reinterpret_cast<const v8bf16*>(&pp[0][2][oa]);
                b[t].p1 = *reinterpret_cast<const v8bf16*>(&pp[1][0][ob]);
                b[t].p2 = *reinterpret_cast<const v8bf16*>(&pp[1][1][ob]);
                b[t].p3 = *reinterpret_cast<const v8bf16*>(&pp[1][2][ob]);
            }
            // the six plane products, smallest first; the four tiles are independent chains
#define LRQ_RU_PP(PB, PA)                                                                                   \
    _Pragma("unroll") for (int mt = 0; mt < 2; ++mt) _Pragma("unroll") for (int nt = 0; nt < 2; ++nt)        \
        f[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[nt].PB, a[mt].PA, f[mt][nt], 0, 0, 0);
            LRQ_RU_PP(p3, p1)
            LRQ_RU_PP(p2, p2)
            LRQ_RU_PP(p1, p3)
            LRQ_RU_PP(p2, p1)
            LRQ_RU_PP(p1, p2)
            LRQ_RU_PP(p1, p1)
#undef LRQ_RU_PP
        }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if (row_ok[mt] && col_ok[nt][g])
                    *reinterpret_cast<float4*>(C + (size_t)row[mt] * N + colb[nt][g]) =
                        make_float4(alpha * f[mt][nt][4 * g + 0], alpha * f[mt][nt][4 * g + 1],
                                    alpha * f[mt][nt][4 * g + 2], alpha * f[mt][nt][4 * g + 3]);
}

// ---------------------------------------------------------------------------
// Panels of the rank-2r update (compensation terms of Algorithm 2 regrouped):
//   C = C0 + [U Sigma | A~ W] . [V^T B~ + (V^T W) Gamma Z^T ; Gamma Z^T]
// Two small launches surround the two code-matrix products A~ W and (V^T B~)^T:
//   panel_prep:   step vectors of both operands, zero-padded copies of W and V for the
//                 matrix-core kernels, and X = V^T W in k-slices;
//   build_panels: sums the split partials of the code products, applies the steps and
//                 assembles the left (M x R2P) and right (N x R2P) panels.
// ---------------------------------------------------------------------------

// Xp[ks][t][u] = sum over the ks-th slice of k of Vt[t][k] W[k][u] (r x r per slice), float64
// accumulation, for the workgroup (t, ks).  Thread (kg, u) walks k = kg, kg + G, ... so a
// wavefront reads whole rows of W (coalesced) against a broadcast element of Vt, eight loads
// deep; the G partial sums are merged through LDS in fixed order.  The slices are summed
// (fixed order) where X is used.
template <int RU>
__device__ __forceinline__ void vtw_block(const float* __restrict__ Vt, const float* __restrict__ W, int K,
                                          int r, int kslice, int t, int ks, float* __restrict__ Xp,
                                          double* __restrict__ part) {
    constexpr int G = 256 / RU;
    const int u = threadIdx.x % RU, kg = threadIdx.x / RU;
    const int uc = min(u, r - 1);
    const int kb = ks * kslice, ke = min(K, kb + kslice);
    const float* vrow = Vt + (size_t)t * K;
    double acc = 0.0;
    for (int k0 = kb + kg; k0 < ke; k0 += 8 * G) {
        float v[8], w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = min(k0 + j * G, K - 1);
            v[j] = vrow[k];
            w[j] = W[(size_t)k * r + uc];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (k0 + j * G < ke) acc = fma((double)v[j], (double)w[j], acc);
    }
    part[kg * RU + u] = acc;
    __syncthreads();
    if (kg == 0 && u < r) {
        double sum = 0.0;
#pragma unroll
        for (int g = 0; g < G; ++g) sum += part[g * RU + u];
        Xp[((size_t)ks * r + t) * r + u] = (float)sum;
    }
}

// x = hi + mid + lo with each term a bfloat16 (the upper 16 bits of a float32): every term is
// the round-to-nearest-even bfloat16 of what is left and the subtractions are exact, so the
// remainder is below 2^-27 |x| -- the three planes carry x to better than float32 precision.
// (Finite inputs; rounding cannot overflow for |x| < 2^127.)
__device__ __forceinline__ uint32_t bf16_rne_bits(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
}
__device__ __forceinline__ void split_bf16x3(float x, uint16_t (&h)[3]) {
    const uint32_t b0 = bf16_rne_bits(x);
    const float r1 = x - __uint_as_float(b0);
    const uint32_t b1 = bf16_rne_bits(r1);
    const float r2 = r1 - __uint_as_float(b1);
    const uint32_t b2 = bf16_rne_bits(r2);
    h[0] = (uint16_t)(b0 >> 16);
    h[1] = (uint16_t)(b1 >> 16);
    h[2] = (uint16_t)(b2 >> 16);
}

struct PrepArgs {
    const float *amaxA, *amaxB, *W, *Vt;
    float *lamA, *sA, *lamB, *sB, *Wp, *Vp, *Xp;
    uint16_t *Wp3, *Vp3;
    int M, Mp, N, Np, K, Kp, r, RP, kslice, nslices;
    float qmaxf;
    int nbA, nbB, nbP;      // workgroups of the first three sections
};

// Workgroup ranges: [0, nbA) steps of A, [nbA, nbA+nbB) steps of B, then nbP workgroups that
// pad W (K x r) and V = Vt^T to K x RP (float32) and write their bfloat16 planes, then
// r * nslices workgroups of V^T W.
__global__ __launch_bounds__(256) void panel_prep_kernel(PrepArgs a) {
    __shared__ double part[256];
    int b = blockIdx.x;
    if (b < a.nbA + a.nbB) {
        const bool isA = b < a.nbA;
        const int i = (isA ? b : b - a.nbA) * 256 + threadIdx.x;
        const int n = isA ? a.M : a.N, npad = isA ? a.Mp : a.Np;
        if (i >= npad) return;
        float l = 0.0f, st = 0.0f;
        if (i < n) make_scales((isA ? a.amaxA : a.amaxB)[i], a.qmaxf, l, st);
        (isA ? a.lamA : a.lamB)[i] = l;
        (isA ? a.sA : a.sB)[i] = st;
        return;
    }
    b -= a.nbA + a.nbB;
    if (b < a.nbP) {
        const size_t idx = (size_t)b * 256 + threadIdx.x;     // k fastest: coalesced plane writes
        if (idx >= (size_t)a.Kp * a.RP) return;
        const int c = (int)(idx / a.Kp), k = (int)(idx % a.Kp);
        const bool in = c < a.r && k < a.K;
        const float wv = in ? a.W[(size_t)k * a.r + c] : 0.f;
        const float vv = in ? a.Vt[(size_t)c * a.K + k] : 0.f;
        if (k < a.K) {
            a.Wp[(size_t)k * a.RP + c] = wv;
            a.Vp[(size_t)k * a.RP + c] = vv;
        }
        uint16_t h[3];
        const size_t plane = (size_t)a.RP * a.Kp;
        split_bf16x3(wv, h);
        a.Wp3[idx] = h[0]; a.Wp3[plane + idx] = h[1]; a.Wp3[2 * plane + idx] = h[2];
        split_bf16x3(vv, h);
        a.Vp3[idx] = h[0]; a.Vp3[plane + idx] = h[1]; a.Vp3[2 * plane + idx] = h[2];
        return;
    }
    b -= a.nbP;
    const int t = b % a.r, ks = b / a.r;
    if (a.r <= 32)      vtw_block<32>(a.Vt, a.W, a.K, a.r, a.kslice, t, ks, a.Xp, part);
    else if (a.r <= 64) vtw_block<64>(a.Vt, a.W, a.K, a.r, a.kslice, t, ks, a.Xp, part);
    else                vtw_block<128>(a.Vt, a.W, a.K, a.r, a.kslice, t, ks, a.Xp, part);
}

// p[0] + p[stride] + ... (n <= MAXN terms, fixed order).  All loads are issued before the first
// add, without branches: a clamped index re-reads the last term, whose value is then masked.
template <int MAXN>
__device__ __forceinline__ float sum_slices(const float* __restrict__ p, int n, size_t stride) {
    float v[MAXN];
#pragma unroll
    for (int t = 0; t < MAXN; ++t) v[t] = p[(size_t)min(t, n - 1) * stride];
    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < MAXN; ++t) acc += (t < n) ? v[t] : 0.f;
    return acc;
}

struct BuildArgs {
    const float *U, *Sig, *sA, *partialA, *sB, *partialB, *Xp, *Gam, *Zt;
    float *Lp, *Rp;
    int M, N, r, RP, R2P, splitsA, splitsB, nslices, nbR;
};

#define BR_J 16     // columns j of C per workgroup of the right panel: short strips, many workgroups --
                    // a workgroup is a chain of three load latencies, so the strips run side by side
// Workgroups [nbR, ...): left panel, one thread per entry:
//   Lp[i][c] = U[i][c] Sig[c] (c < r),  sA[i] sum_sp partialA[sp][i][c-r] (r <= c < 2r), 0 beyond.
// Workgroups [0, nbR) (the longer ones, dispatched first): BR_J rows j of the right panel each:
//   Rp[j][c] = sB[j] sum_sp partialB[sp][j][c] + sum_u X[c][u] Gam[u] Zt[u][j]   (c < r),
//              Gam[c-r] Zt[c-r][j] (r <= c < 2r), 0 beyond,
// with X Gamma and the Zt strip staged in LDS so that global reads and writes stay coalesced.
__global__ __launch_bounds__(256) void build_panels_kernel(BuildArgs a) {
    extern __shared__ float panel_lds[];        // sized by the launcher from r: xg | zt | pv
    const int r = a.r, RP = a.RP, R2P = a.R2P;
    float* const xg = panel_lds;                 // r x (RP + 1): X Gamma
    float* const zt = xg + r * (RP + 1);         // RP x (BR_J + 1): strip of Zt
    float* const pv = zt + RP * (BR_J + 1);      // BR_J x RP: strip of (Vt B~)^T
    if ((int)blockIdx.x >= a.nbR) {
        const size_t idx = (size_t)(blockIdx.x - a.nbR) * 256 + threadIdx.x;
        if (idx >= (size_t)a.M * R2P) return;
        const int i = (int)(idx / R2P), c = (int)(idx % R2P);
        float v = 0.f;
        if (c < r) {
            v = a.U[(size_t)i * r + c] * a.Sig[c];
        } else if (c < 2 * r) {
            const size_t plane = (size_t)a.M * RP;
            v = sum_slices<MAX_SPLITS>(a.partialA + (size_t)i * RP + (c - r), a.splitsA, plane) * a.sA[i];
        }
        a.Lp[idx] = v;
        return;
    }
    const int j0 = (int)blockIdx.x * BR_J;
    for (int e0 = threadIdx.x; e0 < r * r; e0 += 4 * 256) {      // four entries' slice loads in flight
        float x[4];
#pragma unroll
        for (int m = 0; m < 4; ++m)
            x[m] = sum_slices<LRQ_VTW_MAX_SLICES>(a.Xp + min(e0 + 256 * m, r * r - 1), a.nslices, (size_t)r * r);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int e = e0 + 256 * m;
            if (e < r * r) {
                const int c = e / r, u = e - c * r;
                xg[c * (RP + 1) + u] = x[m] * a.Gam[u];
            }
        }
    }
    for (int e0 = threadIdx.x; e0 < RP * BR_J; e0 += 4 * 256) {
        float z[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int e = e0 + 256 * m;
            const int u = min(e / BR_J, r - 1), j = min(j0 + e % BR_J, a.N - 1);
            z[m] = a.Zt[(size_t)u * a.N + j];
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int e = e0 + 256 * m;
            const int u = e / BR_J, jl = e % BR_J;
            if (e < RP * BR_J) zt[u * (BR_J + 1) + jl] = (u < r && j0 + jl < a.N) ? z[m] : 0.f;
        }
    }
    for (int e = threadIdx.x; e < r * (RP - r); e += 256) {     // zero columns u >= r of X Gamma
        const int c = e / (RP - r), u = r + e - c * (RP - r);
        xg[c * (RP + 1) + u] = 0.f;
    }
    // sB[j] sum_sp partialB[sp][j][c] for the strip, four entries' split loads in flight
    const size_t plane = (size_t)a.N * RP;
    const int jn = min(BR_J, a.N - j0);
    for (int e0 = threadIdx.x; e0 < jn * RP; e0 += 4 * 256) {
        float x[4];
#pragma unroll
        for (int m = 0; m < 4; ++m)
            x[m] = sum_slices<MAX_SPLITS>(a.partialB + (size_t)j0 * RP + min(e0 + 256 * m, jn * RP - 1), a.splitsB, plane);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int e = e0 + 256 * m;
            if (e < jn * RP) pv[e] = x[m] * a.sB[j0 + e / RP];
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < BR_J * R2P; e += 256) {
        const int jl = e / R2P, c = e - jl * R2P;
        const int j = j0 + jl;
        if (j >= a.N) break;
        float v = 0.f;
        if (c < r) {
            float acc = pv[jl * RP + c];
            for (int u0 = 0; u0 < RP; u0 += 8) {       // rows u >= r of zt are zero
                float xv[8], zv[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    xv[t] = xg[c * (RP + 1) + u0 + t];
                    zv[t] = zt[(u0 + t) * (BR_J + 1) + jl];
                }
#pragma unroll
                for (int t = 0; t < 8; ++t) acc = fmaf(xv[t], zv[t], acc);
            }
            v = acc;
        } else if (c < 2 * r) {
            v = a.Gam[c - r] * zt[(c - r) * (BR_J + 1) + jl];
        }
        a.Rp[(size_t)j * R2P + c] = v;
    }
}

int vtw_slices(int K) { return max(1, min(LRQ_VTW_MAX_SLICES, K / 256)); }

int launch_panel_prep(int M, int N, int K, int r, int RP, float qmaxf, const float* amaxA, const float* amaxB,
                      const float* W, const float* Vt, float* lamA, float* sA, float* lamB, float* sB, float* Wp,
                      float* Vp, uint16_t* Wp3, uint16_t* Vp3, float* Xp, hipStream_t st) {
    PrepArgs a;
    a.amaxA = amaxA; a.amaxB = amaxB; a.W = W; a.Vt = Vt;
    a.lamA = lamA; a.sA = sA; a.lamB = lamB; a.sB = sB; a.Wp = Wp; a.Vp = Vp; a.Xp = Xp;
    a.Wp3 = Wp3; a.Vp3 = Vp3; a.Kp = (K + 63) / 64 * 64;
    a.M = M; a.Mp = (M + 3) / 4 * 4; a.N = N; a.Np = (N + 3) / 4 * 4; a.K = K; a.r = r; a.RP = RP;
    a.qmaxf = qmaxf;
    a.nbA = ceil_div(a.Mp, 256);
    a.nbB = ceil_div(a.Np, 256);
    int nbV = 0;
    a.nbP = 0; a.kslice = 1; a.nslices = 0;
    if (r > 0) {
        a.nbP = (int)(((size_t)a.Kp * RP + 255) / 256);
        a.kslice = ceil_div(K, vtw_slices(K));
        a.nslices = ceil_div(K, a.kslice);
        nbV = r * a.nslices;
    }
    const int total = a.nbA + a.nbB + a.nbP + nbV;
    if (total == 0) return LRQMM_OK;
    hipLaunchKernelGGL(panel_prep_kernel, dim3(total), dim3(256), 0, st, a);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_build_panels(int M, int N, int K, int r, int RP, int R2P, const float* U, const float* Sig,
                        const float* sA, const float* partialA, int splitsA, const float* sB,
                        const float* partialB, int splitsB, const float* Xp, const float* Gam, const float* Zt,
                        float* Lp, float* Rp, hipStream_t st) {
    BuildArgs a;
    a.U = U; a.Sig = Sig; a.sA = sA; a.partialA = partialA; a.sB = sB; a.partialB = partialB; a.Xp = Xp;
    a.Gam = Gam; a.Zt = Zt; a.Lp = Lp; a.Rp = Rp;
    a.M = M; a.N = N; a.r = r; a.RP = RP; a.R2P = R2P; a.splitsA = splitsA; a.splitsB = splitsB;
    a.nslices = ceil_div(K, ceil_div(K, vtw_slices(K)));
    a.nbR = ceil_div(N, BR_J);
    const int total = a.nbR + (int)(((size_t)M * R2P + 255) / 256);
    const size_t lds = sizeof(float) * ((size_t)r * (RP + 1) + (size_t)RP * (BR_J + 1) + (size_t)BR_J * RP);
    hipLaunchKernelGGL(build_panels_kernel, dim3(total), dim3(256), lds, st, a);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

template <bool VEC>
static void dispatch_gemm256(bool comp, bool wcint, dim3 grid, hipStream_t st, int M, int N, int K,
                             const int8_t* Aq, const int8_t* BqT, const float* sA, const float* sB,
                             const float* Lp, const float* Rp, int R2P, GemmOut C, int32_t* Cint, int tiles_n,
                             int ntiles) {
    const bool full = VEC && (M % BTM == 0) && (N % BTN == 0) && (K % BBK == 0) && K >= BBK;
#define LRQ_GEMM(COMP, WC)                                                                                   \
    do {                                                                                                     \
        if (full)                                                                                            \
            hipLaunchKernelGGL((int8_gemm256_kernel<VEC, COMP, WC, VEC>), grid, dim3(512), 0, st, M, N, K, Aq, \
                               BqT, sA, sB, Lp, Rp, R2P, C, Cint, tiles_n, ntiles, ntiles, 1, nullptr);       \
        else                                                                                                 \
            hipLaunchKernelGGL((int8_gemm256_kernel<VEC, COMP, WC, false>), grid, dim3(512), 0, st, M, N, K,  \
                               Aq, BqT, sA, sB, Lp, Rp, R2P, C, Cint, tiles_n, ntiles, ntiles, 1, nullptr);   \
    } while (0)
    if (comp) {
        if (wcint) LRQ_GEMM(true, true); else LRQ_GEMM(true, false);
    } else {
        if (wcint) LRQ_GEMM(false, true); else LRQ_GEMM(false, false);
    }
#undef LRQ_GEMM
}

template <bool VEC>
static void dispatch_gemm(bool comp, bool wcint, dim3 grid, hipStream_t st, int M, int N, int K,
                          const int8_t* Aq, const int8_t* BqT, const float* sA, const float* sB,
                          const float* Lp, const float* Rp, int R2P, GemmOut C, int32_t* Cint, int tiles_n,
                          int ntiles) {
#define LRQ_GEMM(COMP, WC)                                                                                        \
    do {                                                                                                           \
        if (N <= 64)                                                                                               \
            hipLaunchKernelGGL((int8_gemm_kernel<VEC, COMP, WC, 1>), grid, dim3(256), 0, st, M, N, K, Aq, BqT, sA, sB, \
                               Lp, Rp, R2P, C, Cint, tiles_n, ntiles);                                             \
        else                                                                                                       \
            hipLaunchKernelGGL((int8_gemm_kernel<VEC, COMP, WC, 2>), grid, dim3(256), 0, st, M, N, K, Aq, BqT, sA, sB, \
                               Lp, Rp, R2P, C, Cint, tiles_n, ntiles);                                             \
    } while (0)
    if (comp) {
        if (wcint) LRQ_GEMM(true, true); else LRQ_GEMM(true, false);
    } else {
        if (wcint) LRQ_GEMM(false, true); else LRQ_GEMM(false, false);
    }
#undef LRQ_GEMM
}

// Tiles [first, ntiles) (in xcd_tile order) of C_int <- sum over the K ranges of their partial sums.
__global__ __launch_bounds__(256) void sum_tile_slices_kernel(int32_t* __restrict__ Cint, int N, int tiles_n, int ntiles,
                                                              int first, const int32_t* __restrict__ part, int slices) {
    const int tile = xcd_tile(first + blockIdx.y, tiles_n, ntiles);
    const int m0 = (tile / tiles_n) * BTM, n0 = (tile % tiles_n) * BTN;
    const int e = blockIdx.x * 256 + threadIdx.x;            // 16-byte group of the tile
    const int row = e / (BTN / 4), c4 = e % (BTN / 4);
    const int4* src = reinterpret_cast<const int4*>(part + (size_t)blockIdx.y * slices * (BTM * BTN)) + e;
    int4 acc = make_int4(0, 0, 0, 0);
    for (int s0 = 0; s0 < slices; s0 += 8) {                 // eight loads in flight
        int4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(size_t)min(s0 + u, slices - 1) * (BTM * BTN / 4)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < slices) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    *reinterpret_cast<int4*>(Cint + (size_t)(m0 + row) * N + n0 + 4 * c4) = acc;
}

namespace {
struct SumsPlan { int tiles_n, ntiles, left, slices; };
// Which tiles of the raw-sum product are cut along K when only `resident` CUs are free.
SumsPlan plan_sums(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, int resident) {
    const bool vec = (K % 16 == 0) && K >= 16 && (((uintptr_t)Aq | (uintptr_t)BqT) & 15) == 0;
    const bool full = vec && int8_gemm_large_tiles(M, N) && M % BTM == 0 && N % BTN == 0 && K % BBK == 0 && K >= BBK;
    SumsPlan p = {N / BTN, (M / BTM) * (N / BTN), 0, 1};
    // (with many rounds the last one matters little, and the free CUs change along the way)
    if (full && resident > 0 && p.ntiles > resident && p.ntiles < 4 * resident) {
        p.left = p.ntiles % resident;
        // as many ranges as fill the chip once, each at least four K-tiles deep
        if (p.left > 0) p.slices = max(1, min(min(K / BBK / 4, resident / p.left), LRQ_SUMS_MAX_PARTS / p.left));
    }
    if (p.slices < 2) p.left = 0;
    return p;
}
}  // namespace

size_t int8_gemm_sums_scratch_bytes(int M, int N, int K) {
    const bool shape = int8_gemm_large_tiles(M, N) && M % BTM == 0 && N % BTN == 0 && K % BBK == 0 && K >= 8 * BBK;
    return shape ? (size_t)LRQ_SUMS_MAX_PARTS * BTM * BTN * sizeof(int32_t) : 0;
}

int launch_int8_gemm_sums(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, int32_t* Cint, int resident,
                          int32_t* part, hipStream_t st) {
    const SumsPlan p = part ? plan_sums(M, N, K, Aq, BqT, resident) : SumsPlan{0, 0, 0, 1};
    if (p.left == 0)
        return launch_int8_gemm(M, N, K, Aq, BqT, nullptr, nullptr, nullptr, nullptr, 0, GemmOut{nullptr, N, 1.0f, 0.0f},
                                Cint, st);
    const int full_tiles = p.ntiles - p.left;
    hipLaunchKernelGGL((int8_gemm256_kernel<true, false, true, true, true>), dim3(full_tiles + p.left * p.slices),
                       dim3(512), 0, st, M, N, K, Aq, BqT, nullptr, nullptr, nullptr, nullptr, 0,
                       GemmOut{nullptr, N, 1.0f, 0.0f}, Cint, p.tiles_n, p.ntiles, full_tiles, p.slices, part);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_int8_gemm_sums_finish(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, int32_t* Cint, int resident,
                                 const int32_t* part, hipStream_t st) {
    const SumsPlan p = part ? plan_sums(M, N, K, Aq, BqT, resident) : SumsPlan{0, 0, 0, 1};
    if (p.left == 0) return LRQMM_OK;
    hipLaunchKernelGGL(sum_tile_slices_kernel, dim3(BTM * BTN / 4 / 256, p.left), dim3(256), 0, st, Cint, N, p.tiles_n,
                       p.ntiles, p.ntiles - p.left, part, p.slices);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

// (Measured on both sides of the limit: at 121 tiles of 256 x 256 the 128-tile kernel is as fast, 59 us at
// 2816^3; at 144 tiles it needs 103 us against 63 us at 3072^3.)
bool int8_gemm_large_tiles(int M, int N) {
    return M >= BTM && N >= BTN && (long long)ceil_div(M, BTM) * ceil_div(N, BTN) >= 128;
}

// The early-GEMM schedule needs the large-tile kernel and 16-byte accesses to the rows of C.
bool rank_update_usable(int M, int N, const float* C) {
    return int8_gemm_large_tiles(M, N) && N % 4 == 0 && ((uintptr_t)C & 15) == 0;
}

int launch_rank_update(int M, int N, float* C, const float* sA, const float* sB, const float* Lp, const float* Rp,
                       int R2P, float alpha, hipStream_t st) {
    const int tiles_n = ceil_div(N, 128);
    if (R2P > 64)       // wide panels: bound by the float32 matrix cores, so the plane products on the bf16 ones
        hipLaunchKernelGGL(rank_update_bf16_kernel, dim3(ceil_div(M, 128) * tiles_n), dim3(256), 0, st, M, N, C, sA, sB,
                           Lp, Rp, R2P, tiles_n, alpha);
    else
        hipLaunchKernelGGL(rank_update_kernel, dim3(ceil_div(M, 128) * tiles_n), dim3(256), 0, st, M, N, C, sA, sB, Lp,
                           Rp, R2P, tiles_n, alpha);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

// K == 0: every sum is empty.  One thread per output element.
__global__ __launch_bounds__(256) void empty_product_kernel(int M, int N, GemmOut out, int32_t* __restrict__ Cint) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)M * N) return;
    const int row = (int)(idx / N), col = (int)(idx % N);
    if (Cint) Cint[idx] = 0;
    if (out.C) store_out(out, row, col, 0.0f);
}

int launch_empty_product(int M, int N, GemmOut C, int32_t* Cint, hipStream_t st) {
    const size_t total = (size_t)M * N;
    if (total == 0) return LRQMM_OK;
    hipLaunchKernelGGL(empty_product_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, M, N, C, Cint);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_int8_gemm(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, const float* sA,
                     const float* sB, const float* Lp, const float* Rp, int R2P, GemmOut C, int32_t* Cint,
                     hipStream_t st) {
    // the GEMM kernels issue their first operand loads unconditionally: an empty reduction never reaches them
    if (K <= 0) return launch_empty_product(M, N, C, Cint, st);
    // (the 16-byte load path clamps its address to K - 16, so it needs at least one whole group)
    const bool vec = (K % 16 == 0) && K >= 16 && (((uintptr_t)Aq | (uintptr_t)BqT) & 15) == 0;
    const bool comp = Lp != nullptr;
    // big problems: 256x256 tiles, one workgroup per CU
    const int btiles = ceil_div(M, BTM) * ceil_div(N, BTN);
    if (int8_gemm_large_tiles(M, N)) {
        const int btn = ceil_div(N, BTN);
        dim3 bgrid(btiles);
        if (vec) dispatch_gemm256<true>(comp, Cint != nullptr, bgrid, st, M, N, K, Aq, BqT, sA, sB, Lp, Rp, R2P, C, Cint, btn, btiles);
        else     dispatch_gemm256<false>(comp, Cint != nullptr, bgrid, st, M, N, K, Aq, BqT, sA, sB, Lp, Rp, R2P, C, Cint, btn, btiles);
        LRQ_CHECK_LAUNCH();
        return LRQMM_OK;
    }
    const int tiles_m = ceil_div(M, TM), tiles_n = N <= 64 ? 1 : ceil_div(N, TN);     // (one 64-wide tile column)
    const int ntiles = tiles_m * tiles_n;
    dim3 grid(ntiles);
    if (vec) dispatch_gemm<true>(comp, Cint != nullptr, grid, st, M, N, K, Aq, BqT, sA, sB, Lp, Rp, R2P, C, Cint, tiles_n, ntiles);
    else     dispatch_gemm<false>(comp, Cint != nullptr, grid, st, M, N, K, Aq, BqT, sA, sB, Lp, Rp, R2P, C, Cint, tiles_n, ntiles);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
