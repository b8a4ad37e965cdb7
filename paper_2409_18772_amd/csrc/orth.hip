// Orthonormalization and the small SVD of the randomized range finder (paper:
// Background 2.1 stage 1 "Q with orthogonal columns", Algorithm 1 lines 2-3,
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

#define GB_TILE 64        // rows of Y staged per LDS tile in the Gram kernel
#define GRAM_MAX_BLOCKS 64
#define GRAM_MIN_ROWS 64
#define MAXL LRQMM_MAX_SKETCH

static int gram_rows_per_block(int n) {
    int nblk = min(GRAM_MAX_BLOCKS, max(1, ceil_div(n, GRAM_MIN_ROWS)));
    return ceil_div(ceil_div(n, nblk), GB_TILE) * GB_TILE;
}

int gram_blocks(int n) { return max(1, ceil_div(n, gram_rows_per_block(n))); }

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
        for (int idx = threadIdx.x; idx < GB_TILE * Q4; idx += 256) {
            const int rr = idx / Q4, c = (idx % Q4) * 4;
            const int row = r0 + rr;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < re) {
                const size_t off = (size_t)row * LP + c;
                // every split's load is issued before the first add (splits <= MAX_SPLITS)
                float4 p[MAX_SPLITS];
#pragma unroll
                for (int sp = 0; sp < MAX_SPLITS; ++sp)
                    p[sp] = (sp < splits) ? *reinterpret_cast<const float4*>(partial + sp * plane + off)
                                          : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int sp = 0; sp < MAX_SPLITS; ++sp) {
                    v.x += p[sp].x; v.y += p[sp].y; v.z += p[sp].z; v.w += p[sp].w;
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

// Sum the Gram partials (fixed order) into LDS, G[a][b] for a, b < ell.  The partials were
// written by other workgroups (other XCDs), so every load is a long-latency miss: a thread
// issues all (up to GRAM_MAX_BLOCKS) loads of an entry before summing them.
__device__ static void load_gram(const double* __restrict__ gpart, int nb, int ell, int LP,
                                 double* __restrict__ G, int ldg) {
    const size_t st = (size_t)LP * LP;
    const int total = ell * ell;
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int a = idx / ell, b = idx % ell;
        const double* src = gpart + a * LP + b;
        double v[GRAM_MAX_BLOCKS];
#pragma unroll
        for (int blk = 0; blk < GRAM_MAX_BLOCKS; ++blk) v[blk] = (blk < nb) ? src[blk * st] : 0.0;
        double acc = 0.0;
#pragma unroll
        for (int blk = 0; blk < GRAM_MAX_BLOCKS; ++blk) acc += v[blk];
        G[a * ldg + b] = acc;
    }
}

// Order LDS traffic inside one wavefront: all earlier LDS reads/writes of every lane of
// this wave are complete and the compiler moves no memory access across.
__device__ __forceinline__ void wave_lds_fence() { __asm__ volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// sum_{k in [lo, hi)} row[k] * other[k] over two LDS rows.  The trip count depends on hi
// only (uniform across the wave); lo is applied as a per-lane mask, so lanes with different
// ranges never diverge.  Eight loads of each row are in flight per batch.
__device__ __forceinline__ double lds_dot(const double* __restrict__ row, const double* __restrict__ other,
                                          int lo, int hi) {
    double s = 0.0;
    for (int k = 0; k < hi; k += 8) {
        double a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {      // rows are MAXL+1 long: k+u stays inside the row
            a[u] = row[k + u];
            b[u] = other[k + u];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool in = (k + u >= lo) && (k + u < hi);
            s = fma(in ? a[u] : 0.0, b[u], s);
        }
    }
    return s;
}

// Cholesky G = L L^T and T = L^-T (upper triangular, Q = Y T) in one left-looking sweep on
// a single wavefront.  Lane t owns row t of the LDS matrix: its lower part becomes row t
// of L, its upper part column t of X = L^-1 (G[t][k] = X[k][t], k > t).  At column j every
// lane forms one dot product with the shared row j of L:
//   t >= j:  L[t][j] = (G[t][j] - sum_{k<j} L[t][k] L[j][k]) / L[j][j]
//   t <  j:  X[j][t] = -(sum_{t<=k<j} L[j][k] X[k][t]) / L[j][j]
// so the inverse comes out of the same loop with no workgroup barrier inside it.
#define CHOL_THREADS 1024
__global__ __launch_bounds__(CHOL_THREADS) void chol_inverse_kernel(const double* __restrict__ gpart, int nb,
                                                           int ell, int LP, double* __restrict__ T) {
    __shared__ double G[MAXL * (MAXL + 1)];
    __shared__ double dinv[MAXL];
    __shared__ int dead[MAXL];
    const int ldg = MAXL + 1;
    const int tid = threadIdx.x;
    load_gram(gpart, nb, ell, LP, G, ldg);
    __syncthreads();
    if (tid < 64) {
        double dorig[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = tid + 64 * h;
            dorig[h] = (t < ell) ? G[t * ldg + t] : 0.0;
        }
        for (int j = 0; j < ell; ++j) {
            const double* rowj = G + j * ldg;
            double val[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int t = tid + 64 * h;
                val[h] = 0.0;
                if (h == 1 && ell <= 64) continue;          // uniform: second row set unused
                const int tt = min(t, ell - 1);             // lanes beyond ell shadow the last row
                const bool lower = tt >= j;
                const double dot = lds_dot(G + tt * ldg, rowj, lower ? 0 : tt + 1, j);
                // t < j: the k = t term uses X[t][t] = 1 / L[t][t]
                const double head = lower ? G[tt * ldg + j] : rowj[tt] * dinv[tt];
                val[h] = lower ? head - dot : -(head + dot);
            }
            const double dj = __shfl(val[j >> 6], j & 63, 64);
            const double d0 = __shfl(dorig[j >> 6], j & 63, 64);
            const bool live = dj > 1e-10 * d0 && dj > 0.0;
            double inv = 0.0;
            if (live) {   // 1/sqrt by the hardware estimate and three Newton steps
                inv = __builtin_amdgcn_rsq(dj);
                inv = inv * fma(-0.5 * dj, inv * inv, 1.5);
                inv = inv * fma(-0.5 * dj, inv * inv, 1.5);
                inv = inv * fma(-0.5 * dj, inv * inv, 1.5);
            }
            if (tid == 0) {
                dead[j] = live ? 0 : 1;
                dinv[j] = live ? inv : 1.0;
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int t = tid + 64 * h;
                if (t >= ell) continue;
                G[t * ldg + j] = (t == j) ? (live ? dj * inv : 1.0) : val[h] * inv;
            }
            wave_lds_fence();
        }
    }
    __syncthreads();
    for (int idx = tid; idx < LP * LP; idx += CHOL_THREADS) {
        const int a = idx / LP, b = idx % LP;
        double v = 0.0;
        if (a < ell && b < ell && !dead[b] && !dead[a]) {
            if (a == b) v = dinv[a];
            else if (b > a) v = G[a * ldg + b];
        }
        T[idx] = v;
    }
}

// out = In . Mat for 32 rows per workgroup, float64 accumulation.  Thread (row, g) computes
// the outputs of its row in columns g, g+8, g+16, ...
template <int NT>
__global__ __launch_bounds__(256) void apply_kernel(const float* __restrict__ In, int n,
                                                    const double* __restrict__ Mat, int cm, int ldm,
                                                    float* __restrict__ out, int ldo, int transposed) {
    constexpr int LP = NT * 16;
    constexpr int E = LP / 8;
    constexpr int ld = LP + 1;
    __shared__ double mat[LP * LP];
    __shared__ float tile[32 * ld];
    const int r0 = blockIdx.x * 32;
    for (int idx = threadIdx.x; idx < LP * LP; idx += 256) {
        const int a = idx / LP, c = idx % LP;
        mat[idx] = (c < cm) ? Mat[a * ldm + c] : 0.0;
    }
    for (int idx = threadIdx.x; idx < 32 * LP; idx += 256) {
        const int rr = idx / LP, c = idx % LP;
        tile[rr * ld + c] = (r0 + rr < n) ? In[(size_t)(r0 + rr) * LP + c] : 0.f;
    }
    __syncthreads();
    const int rr = threadIdx.x & 31, g = threadIdx.x >> 5;
    double acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.0;
#pragma unroll 4
    for (int a = 0; a < LP; ++a) {
        const double x = (double)tile[rr * ld + a];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = fma(x, mat[a * LP + g + 8 * e], acc[e]);
    }
    if (r0 + rr >= n) return;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int c = g + 8 * e;
        if (c < cm) {
            if (transposed) out[(size_t)c * ldo + r0 + rr] = (float)acc[e];
            else            out[(size_t)(r0 + rr) * ldo + c] = (float)acc[e];
        }
    }
}

// Jacobi rotation that annihilates the off-diagonal entry of [[gpp, gpq], [gpq, gqq]]
// under G <- J^T G J with J = [[c, s], [-s, c]].  The angle is formed in float (an inexact
// angle still converges); c and s are then made orthonormal to float64 accuracy.
// Returns true when the entry was still "large" (|gpq| > 1e-5 sqrt(gpp gqq)) before the
// rotation: Jacobi converges quadratically, so a sweep that saw no large entry leaves
// off-diagonals of relative size ~1e-10 and is the last one.
__device__ __forceinline__ bool jacobi_rotation(double gpp, double gqq, double gpq, double gsc, double& c,
                                                double& s) {
    c = 1.0;
    s = 0.0;
    const float bf = (float)(2.0 * gpq * gsc);
    const double g2 = gpq * gpq, dd = fabs(gpp * gqq);
    if (!(g2 > 1e-24 * dd) || bf == 0.0f) return false;
    const bool large = g2 > 1e-10 * dd;
    const float th = (float)((gqq - gpp) * gsc) * __builtin_amdgcn_rcpf(bf);
    const float tf = copysignf(1.0f, th) * __builtin_amdgcn_rcpf(fabsf(th) + __builtin_amdgcn_sqrtf(th * th + 1.0f));
    const double t = (double)tf;
    const double x = fma(t, t, 1.0);
    double r = __builtin_amdgcn_rsq(x);
    r = r * fma(-0.5 * x, r * r, 1.5);
    r = r * fma(-0.5 * x, r * r, 1.5);
    r = r * fma(-0.5 * x, r * r, 1.5);
    c = r;
    s = t * r;
    return large;
}

// Cyclic Jacobi eigen-solve of the l x l matrix G = B B^T (B = Q^T R), round-robin pairing
// so l/2 disjoint rotations run per step.  A step is two phases: (1) one thread per pair
// derives its rotation from the pair's 2x2 diagonal block; (2) one thread per (row pair,
// column pair) updates that 2x2 block of G = J^T G J and of V = V J in place (every
// element belongs to exactly one block, so no double buffering is needed).  The kernel is
// bound by instruction issue, so phase 2 is kept to index arithmetic plus 24 multiply/FMA.
// Eigenvalues are the squared singular values of B, eigenvectors its left singular vectors.
#define SVD_THREADS 512
__global__ __launch_bounds__(SVD_THREADS) void small_svd_kernel(const double* __restrict__ gpart, int nb,
                                                                int ell, int LP, int rank,
                                                                float* __restrict__ Sigma,
                                                                double* __restrict__ Ur,
                                                                double* __restrict__ Mv) {
    __shared__ double G[MAXL * (MAXL + 1)];
    __shared__ double V[MAXL * (MAXL + 1)];
    __shared__ double cs[MAXL / 2], sn[MAXL / 2];
    __shared__ int order[MAXL];
    __shared__ int rotated;
    const int ldg = MAXL + 1;
    const int tid = threadIdx.x;
    const int m = (ell + 1) & ~1;   // even number of players; a zero dummy row/column when ell is odd
    for (int idx = tid; idx < m * m; idx += SVD_THREADS) {
        const int a = idx / m, b = idx % m;
        G[a * ldg + b] = 0.0;
        V[a * ldg + b] = (a == b) ? 1.0 : 0.0;
    }
    if (tid == 0) rotated = 0;
    __syncthreads();
    load_gram(gpart, nb, ell, LP, G, ldg);
    __syncthreads();
    const int half = m / 2;
    // round-robin tournament: player m-1 stays, the others rotate (no integer division)
    auto pair_of = [&](int slot, int step, int& p, int& q) {
        int a = step + slot;
        if (a >= m - 1) a -= m - 1;
        if (slot == 0) a = m - 1;
        int b = step - slot;
        if (b < 0) b += m - 1;
        p = min(a, b);
        q = max(a, b);
    };
    double gsc = 0.0;
    if (tid < half) {
        double gmax = 0.0;
        for (int a = 0; a < ell; ++a) gmax = fmax(gmax, fabs(G[a * ldg + a]));
        gsc = gmax > 0.0 ? 1.0 / gmax : 0.0;
    }
    // a thread's blocks are fixed for the whole run: (P, Q) = (blk / half, blk % half)
    for (int sweep = 0; sweep < 16; ++sweep) {
        for (int step = 0; step < m - 1; ++step) {
            if (tid < half) {
                int p, q;
                pair_of(tid, step, p, q);
                double c, s;
                if (jacobi_rotation(G[p * ldg + p], G[q * ldg + q], G[p * ldg + q], gsc, c, s)) rotated = 1;
                cs[tid] = c;
                sn[tid] = s;
            }
            __syncthreads();
            for (int blk = tid; blk < half * half; blk += SVD_THREADS) {
                const int P = blk / half, Q = blk - P * half;
                int p1, q1, p2, q2;
                pair_of(P, step, p1, q1);
                pair_of(Q, step, p2, q2);
                const double c1 = cs[P], s1 = sn[P], c2 = cs[Q], s2 = sn[Q];
                const int r1 = p1 * ldg, r2 = q1 * ldg;
                const double a11 = G[r1 + p2], a12 = G[r1 + q2], a21 = G[r2 + p2], a22 = G[r2 + q2];
                const double b11 = V[r1 + p2], b12 = V[r1 + q2], b21 = V[r2 + p2], b22 = V[r2 + q2];
                // rows: J^T G, then columns: (.) J
                const double t11 = fma(c1, a11, -(s1 * a21)), t12 = fma(c1, a12, -(s1 * a22));
                const double t21 = fma(s1, a11, c1 * a21), t22 = fma(s1, a12, c1 * a22);
                G[r1 + p2] = fma(c2, t11, -(s2 * t12));
                G[r1 + q2] = fma(s2, t11, c2 * t12);
                G[r2 + p2] = fma(c2, t21, -(s2 * t22));
                G[r2 + q2] = fma(s2, t21, c2 * t22);
                V[r1 + p2] = fma(c2, b11, -(s2 * b12));
                V[r1 + q2] = fma(s2, b11, c2 * b12);
                V[r2 + p2] = fma(c2, b21, -(s2 * b22));
                V[r2 + q2] = fma(s2, b21, c2 * b22);
            }
            __syncthreads();
        }
        const int any = rotated;
        __syncthreads();
        if (tid == 0) rotated = 0;
        __syncthreads();
        if (!any) break;
    }
    // rank eigenvalues: order[pos] = index of the pos-th largest (ties by index)
    if (tid < ell) {
        const double mine = G[tid * ldg + tid];
        int pos = 0;
        for (int o = 0; o < ell; ++o) {
            const double other = G[o * ldg + o];
            if (other > mine || (other == mine && o < tid)) ++pos;
        }
        order[pos] = tid;
    }
    __syncthreads();
    if (tid < rank) Sigma[tid] = (float)sqrt(fmax(G[order[tid] * ldg + order[tid]], 0.0));
    const double top = sqrt(fmax(G[order[0] * ldg + order[0]], 0.0));
    for (int idx = tid; idx < LP * rank; idx += SVD_THREADS) {
        const int a = idx / rank, t = idx % rank;
        double u = 0.0, mv = 0.0;
        if (a < ell) {
            const int e = order[t];
            u = V[a * ldg + e];
            const double sg = sqrt(fmax(G[e * ldg + e], 0.0));
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
    const int rpb = gram_rows_per_block(n);
    dim3 grid(gram_blocks(n));
    NT_SWITCH(LP / 16, hipLaunchKernelGGL((reduce_gram_kernel<NT_>), grid, dim3(256), 0, st, partial, splits, n,
                                          rpb, rowscale, Y, gpart));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_chol_inverse(const double* gpart, int nb, int ell, int LP, double* T, hipStream_t st) {
    hipLaunchKernelGGL(chol_inverse_kernel, dim3(1), dim3(CHOL_THREADS), 0, st, gpart, nb, ell, LP, T);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_apply(const float* In, int n, int LP, const double* Mat, int cm, int ldm, float* out, int ldo,
                 int transposed, hipStream_t st) {
    dim3 grid(ceil_div(n, 32));
    NT_SWITCH(LP / 16, hipLaunchKernelGGL((apply_kernel<NT_>), grid, dim3(256), 0, st, In, n, Mat, cm, ldm, out,
                                          ldo, transposed));
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_small_svd(const double* gpart, int nb, int ell, int LP, int rank, float* Sigma, double* Ur,
                     double* Mv, hipStream_t st) {
    hipLaunchKernelGGL(small_svd_kernel, dim3(1), dim3(SVD_THREADS), 0, st, gpart, nb, ell, LP, rank, Sigma, Ur,
                       Mv);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
