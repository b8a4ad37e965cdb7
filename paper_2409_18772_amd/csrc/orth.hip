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

#define GB_ROWS 64   // rows of Y per Gram partial

int gram_blocks(int n) { return ceil_div(n, GB_ROWS); }

__global__ __launch_bounds__(256) void reduce_gram_kernel(const float* __restrict__ partial, int splits,
                                                          int n, int LP,
                                                          const float* __restrict__ rowscale,
                                                          float* __restrict__ Y,
                                                          double* __restrict__ gpart) {
    extern __shared__ float tile[];   // [GB_ROWS][LP+1]
    const int r0 = blockIdx.x * GB_ROWS;
    const int ld = LP + 1;
    for (int idx = threadIdx.x; idx < GB_ROWS * LP; idx += 256) {
        const int rr = idx / LP, c = idx % LP;
        const int row = r0 + rr;
        float v = 0.f;
        if (row < n) {
            const size_t off = (size_t)row * LP + c;
            for (int s = 0; s < splits; ++s) v += partial[(size_t)s * n * LP + off];
            if (rowscale) v *= rowscale[row];
            Y[off] = v;
        }
        tile[rr * ld + c] = v;
    }
    __syncthreads();
    if (!gpart) return;
    double* gp = gpart + (size_t)blockIdx.x * LP * LP;
    for (int idx = threadIdx.x; idx < LP * LP; idx += 256) {
        const int a = idx / LP, b = idx % LP;
        double acc = 0.0;
#pragma unroll 8
        for (int rr = 0; rr < GB_ROWS; ++rr)
            acc = fma((double)tile[rr * ld + a], (double)tile[rr * ld + b], acc);
        gp[idx] = acc;
    }
}

// Sum the Gram partials (fixed order) into LDS, G[a][b] for a, b < ell.
__device__ static void load_gram(const double* __restrict__ gpart, int nb, int ell, int LP,
                                 double* __restrict__ G, int ldg) {
    for (int idx = threadIdx.x; idx < ell * ell; idx += blockDim.x) {
        const int a = idx / ell, b = idx % ell;
        double acc = 0.0;
        for (int blk = 0; blk < nb; ++blk) acc += gpart[(size_t)blk * LP * LP + a * LP + b];
        G[a * ldg + b] = acc;
    }
}

#define MAXL LRQMM_MAX_SKETCH

// Cholesky G = L L^T, then T = L^-T (upper triangular) so that Q = Y T.
__global__ __launch_bounds__(256) void chol_inverse_kernel(const double* __restrict__ gpart, int nb,
                                                           int ell, int LP, double* __restrict__ T) {
    __shared__ double G[MAXL * (MAXL + 1)];
    __shared__ double diag0[MAXL];
    __shared__ double dinv[MAXL];
    __shared__ int dead[MAXL];
    const int ldg = MAXL + 1;
    const int tid = threadIdx.x;
    load_gram(gpart, nb, ell, LP, G, ldg);
    __syncthreads();
    if (tid < ell) diag0[tid] = G[tid * ldg + tid];
    __syncthreads();
    for (int j = 0; j < ell; ++j) {
        if (tid == 0) {
            const double d = G[j * ldg + j];
            const bool live = d > 1e-10 * diag0[j] && d > 0.0;
            dead[j] = live ? 0 : 1;
            G[j * ldg + j] = live ? sqrt(d) : 1.0;
        }
        __syncthreads();
        const double piv = G[j * ldg + j];
        const int dj = dead[j];
        for (int i = j + 1 + tid; i < ell; i += 256) G[i * ldg + j] = dj ? 0.0 : G[i * ldg + j] / piv;
        __syncthreads();
        const int nrem = ell - j - 1;
        for (int idx = tid; idx < nrem * nrem; idx += 256) {
            const int i = j + 1 + idx / nrem, k = j + 1 + idx % nrem;
            if (k <= i) G[i * ldg + k] = fma(-G[i * ldg + j], G[k * ldg + j], G[i * ldg + k]);
        }
        __syncthreads();
    }
    // Inverse of L by forward substitution; column c of L^-1 is kept in row c of the
    // (unused) strict upper triangle of G: G[c][i] = Linv[i][c], i > c.
    if (tid < ell) {
        const int c = tid;
        const double xc = 1.0 / G[c * ldg + c];
        dinv[c] = xc;
        for (int i = c + 1; i < ell; ++i) {
            double sum = G[i * ldg + c] * xc;
            for (int k = c + 1; k < i; ++k) sum = fma(G[i * ldg + k], G[c * ldg + k], sum);
            G[c * ldg + i] = -sum / G[i * ldg + i];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < LP * LP; idx += 256) {
        const int a = idx / LP, b = idx % LP;
        double v = 0.0;
        if (a < ell && b < ell && !dead[b] && !dead[a]) {
            if (a == b) v = dinv[a];
            else if (b > a) v = G[a * ldg + b];
        }
        T[idx] = v;
    }
}

// out = In . Mat for 32 rows per workgroup, float64 accumulation.
__global__ __launch_bounds__(256) void apply_kernel(const float* __restrict__ In, int n, int LP,
                                                    const double* __restrict__ Mat, int cm, int ldm,
                                                    float* __restrict__ out, int ldo, int transposed) {
    extern __shared__ double smem[];
    double* mat = smem;                                        // [LP][cm]
    float* tile = reinterpret_cast<float*>(smem + LP * cm);    // [32][LP+1]
    const int ld = LP + 1;
    const int r0 = blockIdx.x * 32;
    for (int idx = threadIdx.x; idx < LP * cm; idx += 256) mat[idx] = Mat[(idx / cm) * ldm + idx % cm];
    for (int idx = threadIdx.x; idx < 32 * LP; idx += 256) {
        const int rr = idx / LP, c = idx % LP;
        tile[rr * ld + c] = (r0 + rr < n) ? In[(size_t)(r0 + rr) * LP + c] : 0.f;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * cm; idx += 256) {
        int rr, c;
        if (transposed) { rr = idx % 32; c = idx / 32; }
        else            { rr = idx / cm; c = idx % cm; }
        if (r0 + rr >= n) continue;
        double acc = 0.0;
        for (int a = 0; a < LP; ++a) acc = fma((double)tile[rr * ld + a], mat[a * cm + c], acc);
        if (transposed) out[(size_t)c * ldo + r0 + rr] = (float)acc;
        else            out[(size_t)(r0 + rr) * ldo + c] = (float)acc;
    }
}

// Cyclic Jacobi eigen-solve of the l x l matrix G = B B^T (B = Q^T R), round-robin
// pairing so l/2 disjoint rotations run per step.  Eigenvalues are the squared
// singular values of B, eigenvectors its left singular vectors U'.
__global__ __launch_bounds__(256) void small_svd_kernel(const double* __restrict__ gpart, int nb, int ell,
                                                        int LP, int rank, float* __restrict__ Sigma,
                                                        double* __restrict__ Ur, double* __restrict__ Mv) {
    __shared__ double G[MAXL * (MAXL + 1)];
    __shared__ double V[MAXL * (MAXL + 1)];
    __shared__ double cs[MAXL / 2], sn[MAXL / 2];
    __shared__ int pp[MAXL / 2], qq[MAXL / 2];
    __shared__ int order[MAXL];
    __shared__ int rotated;
    __shared__ double gscale;
    const int ldg = MAXL + 1;
    const int tid = threadIdx.x;
    load_gram(gpart, nb, ell, LP, G, ldg);
    for (int idx = tid; idx < ell * ell; idx += 256) {
        const int a = idx / ell, b = idx % ell;
        V[a * ldg + b] = (a == b) ? 1.0 : 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        double mx = 0.0;
        for (int a = 0; a < ell; ++a) mx = fmax(mx, fabs(G[a * ldg + a]));
        gscale = mx;
    }
    __syncthreads();
    const double off_tol = 1e-15 * gscale;   // off-diagonals below this are left alone
    const int m = (ell + 1) & ~1;   // even number of players (a bye when ell is odd)
    const int half = m / 2;
    for (int sweep = 0; sweep < 30; ++sweep) {
        if (tid == 0) rotated = 0;
        __syncthreads();
        for (int step = 0; step < m - 1; ++step) {
            // round-robin: player m-1 fixed, the others rotate
            if (tid < half) {
                int a = (tid == 0) ? m - 1 : (step + tid) % (m - 1);
                int b = (step + m - 1 - tid) % (m - 1);
                int p = min(a, b), q2 = max(a, b);
                double c = 1.0, s = 0.0;
                if (q2 < ell) {
                    const double gpq = G[p * ldg + q2];
                    const double gpp = G[p * ldg + p], gqq = G[q2 * ldg + q2];
                    if (fabs(gpq) > off_tol) {
                        const double theta = (gqq - gpp) / (2.0 * gpq);
                        const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                        c = 1.0 / sqrt(t * t + 1.0);
                        s = t * c;
                        rotated = 1;
                    }
                } else {
                    q2 = -1;
                }
                pp[tid] = p; qq[tid] = q2; cs[tid] = c; sn[tid] = s;
            }
            __syncthreads();
            // rows: G <- J^T G
            for (int idx = tid; idx < half * ell; idx += 256) {
                const int pr = idx / ell, k = idx % ell;
                const int p = pp[pr], q2 = qq[pr];
                if (q2 < 0) continue;
                const double c = cs[pr], s = sn[pr];
                const double gp = G[p * ldg + k], gq = G[q2 * ldg + k];
                G[p * ldg + k] = c * gp - s * gq;
                G[q2 * ldg + k] = s * gp + c * gq;
            }
            __syncthreads();
            // columns: G <- G J, V <- V J
            for (int idx = tid; idx < half * ell; idx += 256) {
                const int pr = idx / ell, k = idx % ell;
                const int p = pp[pr], q2 = qq[pr];
                if (q2 < 0) continue;
                const double c = cs[pr], s = sn[pr];
                const double gp = G[k * ldg + p], gq = G[k * ldg + q2];
                G[k * ldg + p] = c * gp - s * gq;
                G[k * ldg + q2] = s * gp + c * gq;
                const double vp = V[k * ldg + p], vq = V[k * ldg + q2];
                V[k * ldg + p] = c * vp - s * vq;
                V[k * ldg + q2] = s * vp + c * vq;
            }
            __syncthreads();
        }
        if (!rotated) break;
        __syncthreads();
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
    for (int idx = tid; idx < LP * rank; idx += 256) {
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

int launch_reduce_gram(const float* partial, int splits, int n, int LP, const float* rowscale, float* Y,
                       double* gpart, hipStream_t st) {
    const size_t lds = (size_t)GB_ROWS * (LP + 1) * sizeof(float);
    hipLaunchKernelGGL(reduce_gram_kernel, dim3(gram_blocks(n)), dim3(256), lds, st, partial, splits, n, LP,
                       rowscale, Y, gpart);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_chol_inverse(const double* gpart, int nb, int ell, int LP, double* T, hipStream_t st) {
    hipLaunchKernelGGL(chol_inverse_kernel, dim3(1), dim3(256), 0, st, gpart, nb, ell, LP, T);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_apply(const float* In, int n, int LP, const double* Mat, int cm, int ldm, float* out, int ldo,
                 int transposed, hipStream_t st) {
    const size_t lds = (size_t)LP * cm * sizeof(double) + (size_t)32 * (LP + 1) * sizeof(float);
    hipLaunchKernelGGL(apply_kernel, dim3(ceil_div(n, 32)), dim3(256), lds, st, In, n, LP, Mat, cm, ldm, out,
                       ldo, transposed);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}

int launch_small_svd(const double* gpart, int nb, int ell, int LP, int rank, float* Sigma, double* Ur,
                     double* Mv, hipStream_t st) {
    hipLaunchKernelGGL(small_svd_kernel, dim3(1), dim3(256), 0, st, gpart, nb, ell, LP, rank, Sigma, Ur, Mv);
    LRQ_CHECK_LAUNCH();
    return LRQMM_OK;
}
