// Orthonormalization and the small SVD of the randomized range finder (paper:
// Background 2.1 stage 1 "Q with orthogonal columns", Algorithm 1 (range basis and small SVD),
// truncation Eq. (k-svd)).
//
// The tall factors are l <= 80 columns wide, so all O(l^3) work happens on an
// l x l Gram matrix held in LDS by a single workgroup, in float64 (full-rate on
// this chip).  Orthonormalization is Cholesky-QR with the Gram matrix, the
// Cholesky factor, its inverse and the application Q = Y T all in float64; the
// small SVD is a cyclic Jacobi eigen-solve of B B^T.  Accumulating the Gram in
// float64 keeps the squared condition number harmless (residual sketches have
// cond ~ 1e2..1e4).  Columns whose pivot vanishes (rank-deficient sketch, e.g. a
// zero residual) are dropped: the corresponding columns of Q are zero.
#include "kernels.h"

// The kernels of this file are short links of a dependent chain and share the chip with the other operand's
// streaming passes or with the integer product, whose waves keep every SIMD busy.  Their waves ask for the
// highest issue priority on their SIMD (a property of the wave, set by an instruction of the kernel itself: the
// streams all stay at the default priority).  Measured: 4096^3, l = 40: 0.509 -> 0.494 ms per step; 16384^3,
// l = 80: 10.04 -> 9.97 ms.
__device__ __forceinline__ void raise_wave_priority() { __builtin_amdgcn_s_setprio(3); }

#define GB_TILE 64        // rows of Y staged per LDS tile in the Gram kernel
#define GRAM_BATCH 64         // Gram partials per batch of loads when there are more than 64 of them
#define GRAM_MIN_ROWS 64
#define MAXL LRQMM_MAX_SKETCH

// Workgroups of the Gram kernel: 64 for wide sketches (each leaves an LP x LP float64 partial that a later
// kernel has to add up: ~1 MB in all at LP = 48), more for narrow sketches, whose partials are small -- a tall
// operand (10^5 rows at LP = 16) would otherwise keep 64 compute units busy for 25 tiles each.
static int gram_max_blocks(int LP) { return LP <= 16 ? 512 : (LP <= 32 ? 128 : 64); }

static int gram_rows_per_block(int n, int LP) {
    int nblk = min(gram_max_blocks(LP), max(1, ceil_div(n, GRAM_MIN_ROWS)));
    return ceil_div(ceil_div(n, nblk), GB_TILE) * GB_TILE;
}

int gram_blocks(int n, int LP) { return max(1, ceil_div(n, gram_rows_per_block(n, LP))); }

// Y = sum of the pass partials (fixed order, optional row scale); gpart[block] = float64
// Gram matrix of the block's rows.  Threads form a 16 x 16 grid; thread (ta, tb) keeps the
// NT x NT Gram entries (ta + 16x, tb + 16y) in registers, so a staged row costs 2 NT LDS
// reads for NT^2 float64 FMAs.
template <int NT>
__global__ __launch_bounds__(256) void reduce_gram_kernel(const float* __restrict__ partial, int splits,
                                                          int n, int rows_per_block,
                                                          const float* __restrict__ rowscale,
                                                          float* __restrict__ Y,
                                                          double* __restrict__ gpart) {
    constexpr int LP = NT * 16;
    raise_wave_priority();
    constexpr int ld = LP + 1;
    constexpr int Q4 = LP / 4;      // float4 groups per row
    __shared__ float tile[GB_TILE * ld];
    const int rb = blockIdx.x * rows_per_block;
    const int re = min(n, rb + rows_per_block);
    const int ta = threadIdx.x >> 4, tb = threadIdx.x & 15;
    double acc[NT][NT];
#pragma unroll
    for (int x = 0; x < NT; ++x)
#pragma unroll
        for (int y = 0; y < NT; ++y) acc[x][y] = 0.0;
    const size_t plane = (size_t)n * LP;
    for (int r0 = rb; r0 < re; r0 += GB_TILE) {
        __syncthreads();
        if (splits <= MAX_SPLITS) {
            // One batch of splits: every load of the tile is issued before the first add (branch free:
            // clamped row and split indices, masked afterwards), so the tile costs one memory latency
            // instead of one per group of 256 float4.
            constexpr int ITER = (GB_TILE * Q4 + 255) / 256;
            float4 p[ITER][MAX_SPLITS];
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int idx = min((int)threadIdx.x + 256 * it, GB_TILE * Q4 - 1);
                const int rr = idx / Q4, c = (idx % Q4) * 4;
                const size_t off = (size_t)min(r0 + rr, re - 1) * LP + c;
#pragma unroll
                for (int sp = 0; sp < MAX_SPLITS; ++sp)
                    p[it][sp] = *reinterpret_cast<const float4*>(partial + (size_t)min(sp, splits - 1) * plane + off);
            }
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int idx = (int)threadIdx.x + 256 * it;
                if (idx < GB_TILE * Q4) {
                    const int rr = idx / Q4, c = (idx % Q4) * 4;
                    const int row = r0 + rr;
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (row < re) {
#pragma unroll
                        for (int sp = 0; sp < MAX_SPLITS; ++sp)
                            if (sp < splits) { v.x += p[it][sp].x; v.y += p[it][sp].y; v.z += p[it][sp].z; v.w += p[it][sp].w; }
                        if (rowscale) {
                            const float rs = rowscale[row];
                            v.x *= rs; v.y *= rs; v.z *= rs; v.w *= rs;
                        }
                        *reinterpret_cast<float4*>(Y + (size_t)row * LP + c) = v;
                    }
                    float* t = tile + rr * ld + c;
                    t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
                }
            }
        } else
        for (int idx = threadIdx.x; idx < GB_TILE * Q4; idx += 256) {
            const int rr = idx / Q4, c = (idx % Q4) * 4;
            const int row = r0 + rr;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < re) {
                const size_t off = (size_t)row * LP + c;
                // splits are summed in order, MAX_SPLITS at a time: the loads of a batch are all
                // issued before its first add (tall operands use more than one batch)
                for (int s0 = 0; s0 < splits; s0 += MAX_SPLITS) {
                    float4 p[MAX_SPLITS];
#pragma unroll
                    for (int sp = 0; sp < MAX_SPLITS; ++sp)
                        p[sp] = (s0 + sp < splits)
                                    ? *reinterpret_cast<const float4*>(partial + (size_t)(s0 + sp) * plane + off)
                                    : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int sp = 0; sp < MAX_SPLITS; ++sp) {
                        v.x += p[sp].x; v.y += p[sp].y; v.z += p[sp].z; v.w += p[sp].w;
                    }
                }
                if (rowscale) {
                    const float rs = rowscale[row];
                    v.x *= rs; v.y *= rs; v.z *= rs; v.w *= rs;
                }
                *reinterpret_cast<float4*>(Y + off) = v;
            }
            float* t = tile + rr * ld + c;
            t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
        }
        __syncthreads();
        if (gpart) {
#pragma unroll 4
            for (int rr = 0; rr < GB_TILE; ++rr) {
                double av[NT], bv[NT];
#pragma unroll
                for (int x = 0; x < NT; ++x) {
                    av[x] = (double)tile[rr * ld + ta + 16 * x];
                    bv[x] = (double)tile[rr * ld + tb + 16 * x];
                }
#pragma unroll
                for (int x = 0; x < NT; ++x)
#pragma unroll
                    for (int y = 0; y < NT; ++y) acc[x][y] = fma(av[x], bv[y], acc[x][y]);
            }
        }
    }
    if (gpart) {
        double* gp = gpart + (size_t)blockIdx.x * LP * LP;
#pragma unroll
        for (int x = 0; x < NT; ++x)
#pragma unroll
            for (int y = 0; y < NT; ++y) gp[(ta + 16 * x) * LP + tb + 16 * y] = acc[x][y];
    }
}

// Gram matrix = the nb block partials summed by eight threads per entry: thread (part, e) adds the partials
// [part per, (part + 1) per) in order, per = ceil(nb / 8), BATCH loads in flight at a time, and the eight sums are
// added in the order of the parts.  Lanes 8 part + e of a wave: the loads of a part are 8 adjacent entries.
// BATCH = 8 for up to 64 partials: one batch, and few enough registers (under 64) for the waves to start beside
// two resident workgroups of the other operand's pass kernels, which leave about 80 registers per lane free on
// a SIMD -- a kernel with one thread per entry and 64 partials in 128 registers waited for a pass workgroup to
// drain first (16384^3: 58-121 us on average against 4 us alone; the partials were written by other workgroups on
// other XCDs, so every load is a long-latency miss and all loads of a batch are issued before the first add).  BATCH = 64 beyond that (tall
// operands with narrow sketches: several hundred partials).
template <int BATCH>
__global__ __launch_bounds__(64) void gram_sum_parts_kernel(const double* __restrict__ gpart, int nb, int entries,
                                                            double* __restrict__ gram) {
    raise_wave_priority();
    const int e = threadIdx.x & 7, part = threadIdx.x >> 3;
    const int idx = min((int)blockIdx.x * 8 + e, entries - 1);      // (past the end: the last entry again, not stored)
    const int per = (nb + 7) >> 3;
    const int b_begin = min(nb, part * per), b_end = min(nb, b_begin + per);
    const double* src = gpart + idx;
    double acc = 0.0;
    for (int b0 = b_begin; b0 < b_end; b0 += BATCH) {
        double v[BATCH];
#pragma unroll
        for (int blk = 0; blk < BATCH; ++blk) v[blk] = src[(size_t)min(b0 + blk, nb - 1) * entries];
#pragma unroll
        for (int blk = 0; blk < BATCH; ++blk) acc += (b0 + blk < b_end) ? v[blk] : 0.0;
    }
    double sum = __shfl(acc, e, 64);
#pragma unroll
    for (int p = 1; p < 8; ++p) sum += __shfl(acc, 8 * p + e, 64);
    if (part == 0 && (int)blockIdx.x * 8 + e < entries) gram[idx] = sum;
}

// Cholesky-QR factor T = L^-T (upper triangular, Q = Y T) of the Gram matrix G = L L^T, by
// symmetric elimination of the augmented matrix [G | I]: step j subtracts
// (M[i][j] / d_j) * (row j) from every row i > j, d_j the pivot M[j][j].  The left half is then
// L^T with rows unscaled (row j times sqrt(d_j)), the right half is L^-1 with row j unscaled
// the same way, so T[a][b] = M[b][LP + a] / sqrt(d_b).
//
// The matrix lives in registers as KR x KC tiles with strided ownership: worker (ti, tg)
// owns rows ti + NTI*ir (ir < KR) and columns tg + NTI*kc (kc < KC = 2 KR; NTI = LP / KR
// workers each way), so pivot j = tj + NTI*jr sits in register row jr and register column
// jr: compile-time constants inside the unrolled jr loop.  At most four wavefronts (one per SIMD)
// do the work for l <= 64.  A step publishes pivot rows and pivot columns in LDS (two generations,
// so one workgroup barrier per step is enough).  The serial chain per step is LDS write ->
// barrier -> LDS read -> reciprocal -> FMA; the square roots are taken once at the end.
// A pivot below 1e-10 of its original diagonal (rank-deficient sketch) is dead: it
// eliminates nothing and its row and column of T are zero.  The workgroup holds only the
// workers (rounded up to whole waves) and 4 KB of LDS, and every worker loads its tile
// straight from global memory: a small footprint lets the workgroup start at once on a chip
// that another stream keeps full (with 1024 threads and the matrix staged in LDS it waited
// hundreds of microseconds for a free CU at l = 80).
template <int NT>
struct CholShape {
    static constexpr int LP = 16 * NT;
    static constexpr int KR = 4, KC = 8;            // register tile per worker
    static constexpr int NTI = LP / KR;             // workers per row and per column
    static constexpr int WORKERS = NTI * NTI;
    static constexpr int THREADS = (WORKERS + 63) / 64 * 64;
};

// Two pivots per step: pivots j and j+1 share one publication (rows j, j+1
// and columns j, j+1 as they stand before pivot j), one barrier and one LDS round trip, and every
// worker derives the effect of pivot j on row j+1 and on column j+1 itself (redundantly) before it
// applies both rank-1 updates.  Every matrix element receives exactly the operations of plain
// one-pivot-at-a-time elimination in the same order; the serial chain per pivot
// (LDS write -> barrier -> LDS read -> reciprocal -> FMA) is paid once per pair.  NTI is even, so
// a pair never straddles two register rows; an odd l ends with a dead second pivot (zero row).
// Updates that cannot change a value that is read later are skipped at compile time (rows above the
// pivots; eliminated columns of G; columns of the identity half that are still exactly zero):
// 12.5 instead of 32 FMAs per worker and pivot on average, with the same live values.
template <int NT>
__global__ __launch_bounds__(CholShape<NT>::THREADS) void chol_inverse_kernel(const double* __restrict__ gram, int ell,
                                                                     double* __restrict__ T) {
    using S = CholShape<NT>;
    raise_wave_priority();
    constexpr int LP = S::LP, KR = S::KR, KC = S::KC, NTI = S::NTI;
    static_assert(NTI % 2 == 0, "pairs of pivots stay inside one register row");
    __shared__ double rowb[2][2][2 * LP];
    __shared__ double colb[2][2][LP];
    __shared__ double thrb[2][2];
    const int tid = threadIdx.x;
    const bool worker = tid < S::WORKERS;
    const int ti = worker ? tid / NTI : 0, tg = worker ? tid - ti * NTI : 0;
    double mreg[KR][KC];
    double thr[KR];             // 1e-10 * original diagonal of the thread's rows
#pragma unroll
    for (int ir = 0; ir < KR; ++ir) {
        const int i = ti + NTI * ir;        // < LP; rows and columns >= ell enter as zeros
        const double gd = gram[i * LP + i];
        thr[ir] = i < ell ? 1e-10 * gd : 0.0;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const int c = tg + NTI * kc;        // < 2 LP
            const double g = gram[i * LP + (c < LP ? c : c - LP)];     // always inside the LP x LP array
            mreg[ir][kc] = (c < LP) ? ((i < ell && c < ell) ? g : 0.0) : ((c - LP == i && i < ell) ? 1.0 : 0.0);
        }
    }
    double pivot[KR];           // pivots of the thread's rows, 0 when dead
#pragma unroll
    for (int ir = 0; ir < KR; ++ir) pivot[ir] = 0.0;
    int par = 0;
    // Register columns that can still change in register row jr (pivots NTI jr .. NTI jr + NTI - 1).  In the
    // left half [G] the columns of earlier register rows are eliminated and never read again; in the right
    // half [I] the pivot rows are exactly zero beyond their own column, so later register rows see no change.
    auto live_col = [](int kc, int jr) { return kc < KR ? kc >= jr : kc - KR <= jr; };
    auto recip = [](double d) {     // 1/d: hardware estimate and two Newton steps
        double q = __builtin_amdgcn_rcp(d);
        q = fma(fma(-d, q, 1.0), q, q);
        return fma(fma(-d, q, 1.0), q, q);
    };
#pragma unroll
    for (int jr = 0; jr < KR; ++jr) {
        for (int tj = 0; tj < NTI; tj += 2) {
            const int j = tj + NTI * jr;
            if (j >= ell) break;
            if (worker) {
                if (tg == tj || tg == tj + 1) {
#pragma unroll
                    for (int ir = 0; ir < KR; ++ir)
                        if (ir >= jr) colb[par][tg - tj][ti + NTI * ir] = mreg[ir][jr];
                }
                if (ti == tj || ti == tj + 1) {
#pragma unroll
                    for (int kc = 0; kc < KC; ++kc)
                        if (live_col(kc, jr)) rowb[par][ti - tj][tg + NTI * kc] = mreg[jr][kc];
                    if (tg == ti) thrb[par][ti - tj] = thr[jr];
                }
            }
            __syncthreads();
            double l[KR], x[KR], r0[KC], r1[KC];
#pragma unroll
            for (int ir = 0; ir < KR; ++ir) {
                l[ir] = ir >= jr ? colb[par][0][ti + NTI * ir] : 0.0;
                x[ir] = ir >= jr ? colb[par][1][ti + NTI * ir] : 0.0;
            }
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                r0[kc] = live_col(kc, jr) ? rowb[par][0][tg + NTI * kc] : 0.0;
                r1[kc] = live_col(kc, jr) ? rowb[par][1][tg + NTI * kc] : 0.0;
            }
            const double a = rowb[par][0][j], brow = rowb[par][0][j + 1], c11 = rowb[par][1][j + 1];
            const double lnext = colb[par][0][j + 1];
            const double thr0 = thrb[par][0], thr1 = thrb[par][1];
            // pivot j
            const bool live0 = a > thr0 && a > 0.0;
            const double qa = live0 ? recip(a) : 0.0;
            // its effect on row j+1 (every worker, for its own columns) and on the next pivot
            const double f = -(lnext * qa);
            double r1p[KC];
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) r1p[kc] = live_col(kc, jr) ? fma(f, r0[kc], r1[kc]) : 0.0;
            const double d1 = fma(f, brow, c11);
            const bool live1 = d1 > thr1 && d1 > 0.0;
            const double qd = live1 ? recip(d1) : 0.0;
            if (ti == tj) pivot[jr] = live0 ? a : 0.0;
            if (ti == tj + 1) pivot[jr] = live1 ? d1 : 0.0;
#pragma unroll
            for (int ir = 0; ir < KR; ++ir) {
                if (ir < jr) continue;          // rows above the pivots: nothing to eliminate
                const int i = ti + NTI * ir;
                const double lq = (i > j) ? -(l[ir] * qa) : 0.0;
                const double xi = fma(lq, brow, x[ir]);             // column j+1 after pivot j
                const double mq = (i > j + 1) ? -(xi * qd) : 0.0;
#pragma unroll
                for (int kc = 0; kc < KC; ++kc)
                    if (live_col(kc, jr)) mreg[ir][kc] = fma(mq, r1p[kc], fma(lq, r0[kc], mreg[ir][kc]));
            }
            par ^= 1;
        }
    }
    if (!worker) return;
#pragma unroll
    for (int ir = 0; ir < KR; ++ir) {
        const double pv = pivot[ir];
        double inv = 0.0;
        if (pv > 0.0) {      // 1/sqrt by the hardware estimate and three Newton steps
            inv = __builtin_amdgcn_rsq(pv);
            inv = inv * fma(-0.5 * pv, inv * inv, 1.5);
            inv = inv * fma(-0.5 * pv, inv * inv, 1.5);
            inv = inv * fma(-0.5 * pv, inv * inv, 1.5);
        }
        const int i = ti + NTI * ir;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const int c = tg + NTI * kc;
            if (c >= LP) T[(c - LP) * LP + i] = mreg[ir][kc] * inv;
        }
    }
}

// out = In . Mat with float64 accumulation on the float64 matrix cores, one wavefront per 16
// rows.  v_mfma_f64_16x16x4 operand layout (lane l): A[i = l%16][k = l/16], B[k = l/16][j = l%16],
// D[i = 4v + l/16][j = l%16] for v = 0..3.  The reduction index may be visited in any order, so
// lane group l/16 takes the contiguous quarter [kq KQ, (kq+1) KQ) of the LP columns: a lane
// loads KQ consecutive floats of its row (the wavefront's 16 rows form one contiguous block)
// and, per step, one element of Mat.  Every wavefront reads all its rows before it writes any,
// so `out` may alias `In` (same leading dimension).
struct ApplyJob {
    const float* In;
    const double* Mat;
    float* out;
    int n, cm, ldm, ldo, transposed;
};

// Workgroups [0, nb0) work on job j0, the rest on j1.
template <int NT>
__global__ __launch_bounds__(64) void apply_kernel(ApplyJob j0, ApplyJob j1, int nb0) {
    constexpr int LP = NT * 16;
    raise_wave_priority();
    constexpr int KQ = LP / 4;
    const bool first = (int)blockIdx.x < nb0;
    const ApplyJob job = first ? j0 : j1;
    const float* __restrict__ In = job.In;
    const double* __restrict__ Mat = job.Mat;
    float* __restrict__ out = job.out;
    const int n = job.n, cm = job.cm, ldm = job.ldm, ldo = job.ldo, transposed = job.transposed;
    const int l = threadIdx.x, li = l & 15, kq = l >> 4;
    const int r0 = (first ? blockIdx.x : blockIdx.x - nb0) * 16;
    const int row = min(r0 + li, n - 1);
    const bool row_ok = r0 + li < n;
    float a[KQ];
    const float4* ip = reinterpret_cast<const float4*>(In + (size_t)row * LP + kq * KQ);
#pragma unroll
    for (int u = 0; u < KQ / 4; ++u) {
        const float4 t = ip[u];
        a[4 * u + 0] = row_ok ? t.x : 0.f;
        a[4 * u + 1] = row_ok ? t.y : 0.f;
        a[4 * u + 2] = row_ok ? t.z : 0.f;
        a[4 * u + 3] = row_ok ? t.w : 0.f;
    }
    typedef double v4d __attribute__((ext_vector_type(4)));
    v4d acc[NT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) acc[ct] = (v4d){0.0, 0.0, 0.0, 0.0};
    const int nct = (cm + 15) >> 4;         // column tiles that hold output
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        if (ct < nct) {                     // uniform
            const int c = 16 * ct + li;
            const bool c_ok = c < cm;
            const double* mp = Mat + (size_t)(kq * KQ) * ldm + (c_ok ? c : 0);
            double b[KQ];
#pragma unroll
            for (int sidx = 0; sidx < KQ; ++sidx) {
                const double t = mp[(size_t)sidx * ldm];
                b[sidx] = c_ok ? t : 0.0;
            }
#pragma unroll
            for (int sidx = 0; sidx < KQ; ++sidx)
                acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a[sidx], b[sidx], acc[ct], 0, 0, 0);
        }
    }
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const int c = 16 * ct + li;
        if (ct < nct && c < cm) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int orow = r0 + 4 * v + kq;
                if (orow < n) {
                    if (transposed) out[(size_t)c * ldo + orow] = (float)acc[ct][v];
                    else            out[(size_t)orow * ldo + c] = (float)acc[ct][v];
                }
            }
        }
    }
}

// Jacobi rotation that annihilates the off-diagonal entry of [[gpp, gpq], [gpq, gqq]]
// under G <- J^T G J with J = [[c, s], [-s, c]].  The angle is formed in float (an inexact
// angle still converges); c and s are then made orthonormal to float64 accuracy.
// Returns true when the entry was still "large" (|gpq| > 3e-4 sqrt(gpp gqq)) before the
// rotation: Jacobi converges quadratically, so a sweep that saw no large entry leaves
// off-diagonals of relative size ~1e-7 -- the resolution of the float32 factors that leave
// this kernel -- and is the last one (one sweep fewer than with a float64-level criterion,
// with the same distance to the float64 oracle).
__device__ __forceinline__ bool jacobi_rotation(double gpp, double gqq, double gpq, double gsc, double& c,
                                                double& s) {
    c = 1.0;
    s = 0.0;
    const float bf = (float)(2.0 * gpq * gsc);
    const double g2 = gpq * gpq, dd = fabs(gpp * gqq);
    if (!(g2 > 1e-24 * dd) || bf == 0.0f) return false;
    const bool large = g2 > 1e-7 * dd;
    const float th = (float)((gqq - gpp) * gsc) * __builtin_amdgcn_rcpf(bf);
    const float tf = copysignf(1.0f, th) * __builtin_amdgcn_rcpf(fabsf(th) + __builtin_amdgcn_sqrtf(th * th + 1.0f));
    const double t = (double)tf;
    const double x = fma(t, t, 1.0);
    double r = __builtin_amdgcn_rsq(x);
    r = r * fma(-0.5 * x, r * r, 1.5);
    r = r * fma(-0.5 * x, r * r, 1.5);
    c = r;
    s = t * r;
    return large;
}

// Cyclic Jacobi eigen-solve of the l x l matrix G = B B^T (B = Q^T R) with round-robin
// pairing, so l/2 disjoint rotations run per step.
//
// Tournament on m (even) players, circle method: positions 0..m-2 rotate, position m-1 is
// fixed, and slot i pairs positions (i, m-1-i); after a step the player at position c moves
// to c-1 (mod m-1), and position c holds player (step + c) mod (m-1).  G is stored BY SLOT
// (index i = first member of slot i, index half+i = its second member) and moved as part of
// the update (read from one LDS copy, written permuted to the other), so every read and
// write address of a thread is the same in every step: the loop carries no index
// arithmetic, and with a row stride = half (mod 32) consecutive threads hit consecutive
// LDS banks.  The eigenvector matrix is kept transposed and by player (Vt[player][component])
// and is updated in place with 16-byte accesses.  After a whole sweep the arrangement is
// the identity again.
//
// A step has one workgroup barrier:
//  * the update waves apply the step's rotations: thread (P, Q) updates the 2x2 block
//    (slot P rows, slot Q columns) of G <- J^T G J and two components of the column pair
//    of slot P of V <- V J;
//  * meanwhile the rotation wave (wave 0, one lane per pair of the NEXT step) forms the
//    three entries its next pair will have after this step's rotations, in registers, from
//    the copy being read, and derives the next rotation from them.
// Eigenvalues are the squared singular values of B, eigenvectors its left singular vectors.
#define SVD_UPDATE_THREADS 448
#define SVD_THREADS (64 + SVD_UPDATE_THREADS)
#define SVD_POOL 19600     // float64 words of LDS for the two copies of G and for Vt

// Loop-invariant addresses of one 2x2 block task of an update thread.
struct SvdTask {
    int active;
    int P, Q;
    int o11, o12, o21, o22;     // read offsets in G (words)
    int w11, w12, w21, w22;     // write offsets in the other copy
    int v1, v2;                 // word offsets in Vt of the slot's two eigenvector columns
    int v1_wrap, v2_wrap, dv2;  // both run up one player (ldv words) per step and wrap after player m-2
};

template <int NB>
__global__ __launch_bounds__(SVD_THREADS) void small_svd_kernel(const double* __restrict__ gram, int ell,
                                                                int LP, int rank,
                                                                float* __restrict__ Sigma,
                                                                double* __restrict__ Ur,
                                                                double* __restrict__ Mv) {
    __shared__ __align__(16) double pool[SVD_POOL];
    raise_wave_priority();
    __shared__ __align__(16) double2 rot[2][MAXL / 2];      // (c, s) per slot, two generations
    __shared__ int order[MAXL];
    __shared__ int finished;
    const int tid = threadIdx.x;
    const int m = (ell + 1) & ~1;   // even number of players; a zero dummy row/column when ell is odd
    const int half = m / 2;
    int ldg = m + ((half - m) & 31);                      // >= m, = half (mod 32)
    if (2 * m * ldg + m * m > SVD_POOL) ldg = m + 1;       // largest sketches: accept bank conflicts
    const int ldv = m;
    double* const G0 = pool;
    double* const G1 = pool + m * ldg;
    double* const Vt = pool + 2 * m * ldg;
    // slot index of a player when the arrangement is the identity (start of a sweep)
    auto home = [&](int e) { return e < half ? e : half + (m - 1 - e); };
    // slot index after one step of the tournament
    auto moved = [&](int x) {
        if (m == 2) return x;
        if (x < half) return x == 0 ? half + 1 : x - 1;
        const int y = x - half;
        return y == 0 ? half : (y == half - 1 ? half - 1 : x + 1);
    };
    for (int idx = tid; idx < m * ldg; idx += SVD_THREADS) G0[idx] = 0.0;
    for (int idx = tid; idx < m * m; idx += SVD_THREADS) Vt[idx] = (idx / m == idx % m) ? 1.0 : 0.0;
    if (tid == 0) finished = 0;
    __syncthreads();
    for (int base = 0; base < ell * ell; base += 4 * SVD_THREADS) {     // stored by slot; four loads in flight
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = min(base + u * SVD_THREADS + tid, ell * ell - 1);
            v[u] = gram[(idx / ell) * LP + idx % ell];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * SVD_THREADS + tid;
            if (idx < ell * ell) G0[home(idx / ell) * ldg + home(idx % ell)] = v[u];
        }
    }
    __syncthreads();

    // rotation wave: addresses of the ten entries behind the lane's next pair (loop invariant)
    double gsc = 0.0;
    bool seen_large = false;
    int iaa = 0, iab = 0, ibb = 0, jaa = 0, jab = 0, jbb = 0, x11i = 0, x12i = 0, x21i = 0, x22i = 0, sa = 0, sb = 0;
    bool xfirst = true, yfirst = true;
    SvdTask task[NB];
    if (tid < half) {
        double gmax = 0.0;
        for (int a = 0; a < m; ++a) gmax = fmax(gmax, fabs(G0[a * ldg + a]));
        gsc = gmax > 0.0 ? 1.0 / gmax : 0.0;
        const int p = tid, q = half + tid;
        double c, s;
        seen_large = jacobi_rotation(G0[p * ldg + p], G0[q * ldg + q], G0[p * ldg + q], gsc, c, s);
        rot[0][tid] = make_double2(c, s);
        int cx = p, cy = q;                                // where the next pair sits now
        for (int x = 0; x < m; ++x) {
            const int y = moved(x);
            if (y == p) cx = x;
            if (y == q) cy = x;
        }
        xfirst = cx < half;
        yfirst = cy < half;
        sa = xfirst ? cx : cx - half;
        sb = yfirst ? cy : cy - half;
        const int pa = sa, qa = half + sa, pb = sb, qb = half + sb;
        iaa = pa * ldg + pa; iab = pa * ldg + qa; ibb = qa * ldg + qa;
        jaa = pb * ldg + pb; jab = pb * ldg + qb; jbb = qb * ldg + qb;
        x11i = pa * ldg + pb; x12i = pa * ldg + qb; x21i = qa * ldg + pb; x22i = qa * ldg + qb;
    }
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        SvdTask& k = task[t];
        const int blk = tid - 64 + t * SVD_UPDATE_THREADS;
        k.active = tid >= 64 && blk < half * half;
        const int P = k.active ? blk / half : 0, Q = k.active ? blk - P * half : 0;
        k.P = P; k.Q = Q;
        k.o11 = P * ldg + Q; k.o12 = k.o11 + half; k.o21 = (half + P) * ldg + Q; k.o22 = k.o21 + half;
        const int n1 = moved(P) * ldg, n2 = moved(half + P) * ldg, k1 = moved(Q), k2 = moved(half + Q);
        k.w11 = n1 + k1; k.w12 = n1 + k2; k.w21 = n2 + k1; k.w22 = n2 + k2;
        // eigenvector columns of slot P at step 0: players P and (m - 1 - P) (slot 0: m - 1, fixed)
        k.v1 = P * ldv + 2 * Q;
        k.v2 = (m - 1 - P) * ldv + 2 * Q;
        k.dv2 = (P == 0) ? 0 : ldv;
        k.v1_wrap = (m - 1) * ldv + 2 * Q;     // first offset past player m - 2
        k.v2_wrap = (P == 0) ? 0x7fffffff : k.v1_wrap;   // player m - 1 never moves
    }
    __syncthreads();
    // one tournament step: reads G/rr, writes Gn/rn
    auto do_step = [&](const double* __restrict__ G, double* __restrict__ Gn, const double2* __restrict__ rr,
                       double2* __restrict__ rn, bool last_of_sweep) {
        if (tid < 64) {
            if (tid < half) {
                const double2 ra = rr[sa], rb = rr[sb];
                const double ca = ra.x, sna = ra.y, cb = rb.x, snb = rb.y;
                const double a11 = G[iaa], a12 = G[iab], a22 = G[ibb];
                const double b11 = G[jaa], b12 = G[jab], b22 = G[jbb];
                const double x11 = G[x11i], x12 = G[x12i], x21 = G[x21i], x22 = G[x22i];
                // diagonal entry of J^T D J for a symmetric 2x2 block D:
                //   first : c^2 d11 - 2 c s d12 + s^2 d22     second: s^2 d11 + 2 c s d12 + c^2 d22
                const double wa = 2.0 * ca * sna * a12, wb = 2.0 * cb * snb * b12;
                const double ca2 = ca * ca, sa2 = sna * sna, cb2 = cb * cb, sb2 = snb * snb;
                const double gxx = xfirst ? fma(ca2, a11, fma(sa2, a22, -wa)) : fma(sa2, a11, fma(ca2, a22, wa));
                const double gyy = yfirst ? fma(cb2, b11, fma(sb2, b22, -wb)) : fma(sb2, b11, fma(cb2, b22, wb));
                // entry (x, y) of J_a^T X J_b: column of J_a for x, column of J_b for y
                const double al0 = xfirst ? ca : sna, al1 = xfirst ? -sna : ca;
                const double be0 = yfirst ? cb : snb, be1 = yfirst ? -snb : cb;
                const double gxy = fma(al0, fma(x11, be0, x12 * be1), al1 * fma(x21, be0, x22 * be1));
                double c, s;
                const bool large = jacobi_rotation(gxx, gyy, gxy, gsc, c, s);
                rn[tid] = make_double2(c, s);
                // the flags of a sweep cover the rotations applied in it; the one just
                // formed at the last step opens the next sweep
                if (last_of_sweep) {
                    const bool any = __any(seen_large);
                    if (tid == 0) finished = any ? 0 : 1;
                    seen_large = large;
                } else {
                    seen_large = seen_large || large;
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < NB; ++t) {
                SvdTask& k = task[t];
                if (k.active) {
                    const double2 r1 = rr[k.P], r2 = rr[k.Q];
                    const double c1 = r1.x, s1 = r1.y, c2 = r2.x, s2 = r2.y;
                    const double a11 = G[k.o11], a12 = G[k.o12], a21 = G[k.o21], a22 = G[k.o22];
                    double2* e1p = reinterpret_cast<double2*>(Vt + k.v1);
                    double2* e2p = reinterpret_cast<double2*>(Vt + k.v2);
                    const double2 e1 = *e1p, e2 = *e2p;
                    // rows: J^T G, then columns: (.) J
                    const double t11 = fma(c1, a11, -(s1 * a21)), t12 = fma(c1, a12, -(s1 * a22));
                    const double t21 = fma(s1, a11, c1 * a21), t22 = fma(s1, a12, c1 * a22);
                    Gn[k.w11] = fma(c2, t11, -(s2 * t12));
                    Gn[k.w12] = fma(s2, t11, c2 * t12);
                    Gn[k.w21] = fma(c2, t21, -(s2 * t22));
                    Gn[k.w22] = fma(s2, t21, c2 * t22);
                    *e1p = make_double2(fma(c1, e1.x, -(s1 * e2.x)), fma(c1, e1.y, -(s1 * e2.y)));
                    *e2p = make_double2(fma(s1, e1.x, c1 * e2.x), fma(s1, e1.y, c1 * e2.y));
                    // next step: both columns of the slot are one player further
                    k.v1 += ldv;
                    if (k.v1 >= k.v1_wrap) k.v1 -= (m - 1) * ldv;
                    k.v2 += k.dv2;
                    if (k.v2 >= k.v2_wrap) k.v2 -= (m - 1) * ldv;
                }
            }
        }
        __syncthreads();
    };
    int cur = 0, step = 0, sweeps = 0;
    for (;;) {
        const bool last = (step + 1 == m - 1);
        if (cur == 0) do_step(G0, G1, rot[0], rot[1], last);
        else          do_step(G1, G0, rot[1], rot[0], last);
        cur ^= 1;
        if (last) {
            step = 0;
            if (++sweeps == 16 || finished) break;
        } else {
            ++step;
        }
    }
    const double* G = cur ? G1 : G0;
    // rank eigenvalues: order[pos] = index of the pos-th largest (ties by index)
    if (tid < ell) {
        const double mine = G[home(tid) * ldg + home(tid)];
        int pos = 0;
#pragma unroll 8
        for (int o = 0; o < ell; ++o) {
            const double other = G[home(o) * ldg + home(o)];
            if (other > mine || (other == mine && o < tid)) ++pos;
        }
        order[pos] = tid;
    }
    __syncthreads();
    if (tid < rank) Sigma[tid] = (float)sqrt(fmax(G[home(order[tid]) * ldg + home(order[tid])], 0.0));
    const double top = sqrt(fmax(G[home(order[0]) * ldg + home(order[0])], 0.0));
    for (int idx = tid; idx < LP * rank; idx += SVD_THREADS) {
        const int a = idx / rank, t = idx % rank;
        double u = 0.0, mv = 0.0;
        if (a < ell) {
            const int e = order[t];
            u = Vt[e * ldv + a];
            const double sg = sqrt(fmax(G[home(e) * ldg + home(e)], 0.0));
            mv = (sg > 1e-14 * top && sg > 0.0) ? u / sg : 0.0;
        }
        Ur[idx] = u;
        Mv[idx] = mv;
    }
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

int launch_reduce_gram(const float* partial, int splits, int n, int LP, const float* rowscale, float* Y,
                       double* gpart, hipStream_t st) {
    const int rpb = gram_rows_per_block(n, LP);
    dim3 grid(gram_blocks(n, LP));
    NT_SWITCH(LP / 16, hipLaunchKernelGGL((reduce_gram_kernel<NT_>), grid, dim3(256), 0, st, partial, splits, n,
                                          rpb, rowscale, Y, gpart));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_gram_sum(const double* gpart, int nb, int LP, double* gram, hipStream_t st) {
    if (nb > GRAM_BATCH)
        hipLaunchKernelGGL(gram_sum_parts_kernel<GRAM_BATCH>, dim3(ceil_div(LP * LP, 8)), dim3(64), 0, st, gpart, nb, LP * LP, gram);
    else
        hipLaunchKernelGGL(gram_sum_parts_kernel<8>, dim3(ceil_div(LP * LP, 8)), dim3(64), 0, st, gpart, nb, LP * LP, gram);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_chol_inverse(const double* gram, int ell, int LP, double* T, hipStream_t st) {
    NT_SWITCH(LP / 16, hipLaunchKernelGGL((chol_inverse_kernel<NT_>), dim3(1), dim3(CholShape<NT_>::THREADS), 0, st, gram, ell,
                                          T));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_apply2(const float* In0, int n0, const double* Mat0, int cm0, int ldm0, float* out0, int ldo0,
                  int transposed0, const float* In1, int n1, const double* Mat1, int cm1, int ldm1, float* out1,
                  int ldo1, int transposed1, int LP, hipStream_t st) {
    const ApplyJob j0 = {In0, Mat0, out0, n0, cm0, ldm0, ldo0, transposed0};
    const ApplyJob j1 = {In1, Mat1, out1, n1, cm1, ldm1, ldo1, transposed1};
    const int nb0 = n0 > 0 ? ceil_div(n0, 16) : 0, nb1 = n1 > 0 ? ceil_div(n1, 16) : 0;
    if (nb0 + nb1 == 0) return LRQMM_OK;
    NT_SWITCH(LP / 16, hipLaunchKernelGGL((apply_kernel<NT_>), dim3(nb0 + nb1), dim3(64), 0, st, j0, j1, nb0));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_apply(const float* In, int n, int LP, const double* Mat, int cm, int ldm, float* out, int ldo,
                 int transposed, hipStream_t st) {
    return launch_apply2(In, n, Mat, cm, ldm, out, ldo, transposed, nullptr, 0, nullptr, 0, 0, nullptr, 0, 0, LP,
                         st);
}

int launch_small_svd(const double* gram, int ell, int LP, int rank, float* Sigma, double* Ur, double* Mv,
                     hipStream_t st) {
    const int m = (ell + 1) & ~1, blocks = (m / 2) * (m / 2);
    switch (ceil_div(blocks, SVD_UPDATE_THREADS)) {      // 2x2 blocks per update thread
        case 1: hipLaunchKernelGGL(small_svd_kernel<1>, dim3(1), dim3(SVD_THREADS), 0, st, gram, ell, LP, rank, Sigma, Ur, Mv); break;
        case 2: hipLaunchKernelGGL(small_svd_kernel<2>, dim3(1), dim3(SVD_THREADS), 0, st, gram, ell, LP, rank, Sigma, Ur, Mv); break;
        case 3: hipLaunchKernelGGL(small_svd_kernel<3>, dim3(1), dim3(SVD_THREADS), 0, st, gram, ell, LP, rank, Sigma, Ur, Mv); break;
        case 4: hipLaunchKernelGGL(small_svd_kernel<4>, dim3(1), dim3(SVD_THREADS), 0, st, gram, ell, LP, rank, Sigma, Ur, Mv); break;
        default: return LRQMM_ERR_UNSUPPORTED;
    }
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
