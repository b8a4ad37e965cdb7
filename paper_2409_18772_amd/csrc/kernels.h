// Internal launch functions of the LRQMM library (one per step of the hot path).
// All pointers are device pointers; every function only enqueues work on `st`
// and returns LRQMM_OK or LRQMM_ERR_HIP.
#pragma once
#include "common.h"
#include "../../include/lrqmm.h"

// ---- quantize.hip -------------------------------------------------------
// X is rows x cols with row stride ldx (>= cols).  per_tensor: one scale for the whole matrix,
// i.e. every entry of amax holds the global maximum.  amax0 != null: quantize the residual of a
// first quantization whose group maxima are amax0 (second level of Eq. (gemm_r_split)).
int launch_quantize_rows(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor,
                         const float* amax0, int8_t* codes, float* amax, hipStream_t st);
// amax_zeroed: the caller has already cleared amax[0 .. cols) on this stream (the column maxima are merged
// with atomics and must start at zero).  lam_out, s_out (both or neither): also write the step vectors
// lam = qmax/amax, s = amax/qmax of the columns, zero padded to a multiple of 4 entries.
int launch_quantize_cols(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor,
                         const float* amax0, int8_t* codesT, float* amax, hipStream_t st, bool amax_zeroed = false,
                         float* lam_out = nullptr, float* s_out = nullptr);
// The group maxima alone (first half of the two launchers above; for columns amax must be zero at launch when
// amax_zeroed is set, and is cleared by a fill kernel otherwise).
int launch_absmax_rows(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor, float* amax,
                       hipStream_t st);
int launch_absmax_cols(const float* X, int ldx, int rows, int cols, QuantParams q, bool per_tensor, float* amax,
                       hipStream_t st, bool amax_zeroed);
// lam[n], s[n] from amax[n]; entries n..npad-1 are zero-filled.
// A minimal kernel (writes one zero word): used as a few microseconds of delay on a stream.
int launch_tick(uint32_t* word, hipStream_t st);
int launch_scales(const float* amax, int n, int npad, float qmaxf, float* lam, float* s,
                  hipStream_t st);

// ---- sketch.hip ---------------------------------------------------------
// omega[i*ld + j] for i < rows, j < ld; columns j >= cols are zero.
int launch_fill_sketch(uint64_t seed, int stream_id, int rows, int cols, int ld, float* omega,
                       hipStream_t st);
// The same plus, in the same launch, the step vectors of the operand: lam[i] = qmax/amax[i],
// s[i] = amax[i]/qmax for i < n, zero up to npad (skipped when amax is null).
int launch_sketch_and_scales(uint64_t seed, int stream_id, int rows, int cols, int ld, float* omega,
                             const float* amax, int n, int npad, float qmaxf, float* lam, float* s,
                             hipStream_t st);
// The sketch plus, in the same launch, zero_n words cleared at zero_words: the first kernel of a
// column-wise quantization followed by a factorization (the sketch depends on neither).
int launch_sketch_and_zero(uint64_t seed, int stream_id, int rows, int cols, int ld, float* omega,
                           uint32_t* zero_words, int zero_n, hipStream_t st);
// dst[i*ld + j] = (j < cols) ? src[i*cols + j] : 0
int launch_pad_copy(const float* src, int rows, int cols, int ld, float* dst, hipStream_t st);

// ---- passes.hip ---------------------------------------------------------
#define MAX_SPLITS 8      // upper bound on the splits of plan_pass_n (its partials are summed in one batch)
#define MAX_SPLITS_T 64   // upper bound for plan_pass_t (only launch_reduce_gram sums those, in batches)
struct PassPlan {
    int splits;   // number of partial results
    int chunk;    // reduction-index range per split (multiple of 64)
};
PassPlan plan_pass_n(int rows, int cols);
PassPlan plan_pass_t(int rows, int cols);
// X is rows x cols with row stride ldx (>= cols) in both passes.
// planes: bfloat16 planes per float32 operand in the matrix-core products (3: float32 accuracy, the default;
// 2: relative error 2^-16 per product; 1: plain bfloat16 operands) -- the reduced-precision compensation of the
// Methodology (text after Eq. (gemm_r_split)).  With planes == 3 sketches of up to 16 columns use the float32
// matrix-core kernels.
// partial[s][rows][LP] = R[:, chunk s] . W[chunk s, :]      (W is cols x LP)
int launch_resid_mul_n(const float* X, int ldx, int rows, int cols, int axis, const float* lam,
                       const float* s, QuantParams q, const float* W, int LP, PassPlan plan,
                       float* partial, hipStream_t st, int planes = 3);
// The quantization of X fused into its first residual product: with the group maxima amax known (rows for
// axis 0, columns for axis 1), one read of X writes the codes (row-major for axis 0, transposed for axis 1), the
// step vectors lam_out / s_out, and the partials of R.W as launch_resid_mul_n does (same arithmetic, same bits).
// Only for the shapes quant_sketch_fusable accepts (guard-free: rows, cols and the split length multiples of 64,
// sketch width above 16, aligned pointers); otherwise LRQMM_ERR_UNSUPPORTED and nothing is launched.
bool quant_sketch_fusable(const float* X, int ldx, int rows, int cols, int LP, PassPlan plan, const int8_t* codes);
int launch_quant_sketch(const float* X, int ldx, int rows, int cols, int axis, const float* amax, QuantParams q,
                        const float* W, int LP, PassPlan plan, float* partial, float* lam_out, float* s_out,
                        int8_t* codes, hipStream_t st, int planes = 3);
// Row quantization and the sketch product from one read, for operands quantized by rows whose rows are short
// (cols <= 576, a multiple of 16) and sketches padded to 16 columns: writes the row maxima amax[rows], the step
// vectors, the codes (rows x cols), Y = R.W (rows x 16) and gpart[quant_sketch_rows_blocks(rows)][16][16], the
// float64 Gram matrices of the workgroups' rows of Y (to be added by launch_gram_sum).  Maxima, steps and codes
// carry the bits of launch_quantize_rows; Y is the float32 matrix-core product of launch_resid_mul_n with the
// reduction cut into eight parts that are added in a fixed order.  Otherwise LRQMM_ERR_UNSUPPORTED and nothing is
// launched.
#define LRQ_QSR_MAX_BLOCKS 512
bool quant_sketch_rows_usable(const float* X, int ldx, int rows, int cols, int LP, const int8_t* codes);
int quant_sketch_rows_blocks(int rows);
int launch_quant_sketch_rows(const float* X, int ldx, int rows, int cols, QuantParams q, const float* W, int LP,
                             float* Y, double* gpart, float* amax, float* lam_out, float* s_out, int8_t* codes,
                             hipStream_t st);
// partial[s][cols][LP] = R[chunk s, :]^T . W[chunk s, :]    (W is rows x LP)
int launch_resid_mul_t(const float* X, int ldx, int rows, int cols, int axis, const float* lam,
                       const float* s, QuantParams q, const float* W, int LP, PassPlan plan,
                       float* partial, hipStream_t st, int planes = 3);
// Two independent products in one launch:
// partialX[s][rowsX][LP] = scale-free codesX[:, chunk s] . WX[chunk s, :]  (codesX rowsX x K int8)
// WX: K x LP float32; WX3: the same factor as three bfloat16 planes [3][LP][Kp] (k fastest,
// Kp = K rounded up to 64, zero padded), used when K % 16 == 0.
int launch_codes_mul_n2(const int8_t* codesA, int rowsA, const float* WA, const uint16_t* WA3, PassPlan planA,
                        float* partialA, const int8_t* codesB, int rowsB, const float* WB, const uint16_t* WB3,
                        PassPlan planB, float* partialB, int K, int Kp, int LP, hipStream_t st, int planes = 3);

// ---- orth.hip -----------------------------------------------------------
int gram_blocks(int n, int LP);
// Y[n][LP] = sum_s partial[s][n][LP] (optionally times rowscale[i]);
// gpart[b][LP*LP] = Gram of rows 64b..64b+63 of Y in float64.
int launch_reduce_gram(const float* partial, int splits, int n, int LP, const float* rowscale,
                       float* Y, double* gpart, hipStream_t st);
// gram (LP x LP float64) = sum over b < nb of gpart[b], in fixed order.
int launch_gram_sum(const double* gpart, int nb, int LP, double* gram, hipStream_t st);
// T (LP x LP float64, upper triangular) with (Y T)^T (Y T) = I on the live columns, from
// the Gram matrix of Y.
int launch_chol_inverse(const double* gram, int ell, int LP, double* T, hipStream_t st);
// out = In[n x LP] . Mat[LP x cm]; normal: out[i*ldo + c]; transposed: out[c*ldo + i].
int launch_apply(const float* In, int n, int LP, const double* Mat, int cm, int ldm, float* out,
                 int ldo, int transposed, hipStream_t st);
// Two independent products of that kind in one launch.
int launch_apply2(const float* In0, int n0, const double* Mat0, int cm0, int ldm0, float* out0, int ldo0,
                  int transposed0, const float* In1, int n1, const double* Mat1, int cm1, int ldm1, float* out1,
                  int ldo1, int transposed1, int LP, hipStream_t st);
// Eigen-decomposition of the Gram matrix (l x l, leading dimension LP): Sigma[r] = sqrt of
// the r largest eigenvalues, Ur (LP x r) their eigenvectors, Mv = Ur diag(1/Sigma).
int launch_small_svd(const double* gram, int ell, int LP, int rank, float* Sigma, double* Ur,
                     double* Mv, hipStream_t st);

// ---- gemm.hip -----------------------------------------------------------
// X = V^T W is kept as vtw_slices(K) k-slices Xp[ks][t][u] that are summed where X is used.
#define LRQ_VTW_MAX_SLICES 16
int vtw_slices(int K);
// One launch: step vectors lamX/sX (padded to a multiple of 4) of both operands and, when
// r > 0, the zero-padded K x RP copies Wp of W and Vp of Vt^T and the slices Xp of V^T W.
// Wp3 / Vp3: the same two factors as bfloat16 planes [3][RP][Kp] (see launch_codes_mul_n2).
int launch_panel_prep(int M, int N, int K, int r, int RP, float qmaxf, const float* amaxA, const float* amaxB,
                      const float* W, const float* Vt, float* lamA, float* sA, float* lamB, float* sB, float* Wp,
                      float* Vp, uint16_t* Wp3, uint16_t* Vp3, float* Xp, hipStream_t st);
// Left panel  Lp[i][0..r) = U[i][t] Sig[t],  Lp[i][r..2r) = sA[i] sum_s partialA[s][i][u]
// Right panel Rp[j][0..r) = sB[j] sum_s partialB[s][j][t] + sum_u X[t][u] Gam[u] Zt[u][j]
//             Rp[j][r..2r) = Gam[u] Zt[u][j];   both zero padded to R2P columns.
int launch_build_panels(int M, int N, int K, int r, int RP, int R2P, const float* U, const float* Sig,
                        const float* sA, const float* partialA, int splitsA, const float* sB,
                        const float* partialB, int splitsB, const float* Xp, const float* Gam, const float* Zt,
                        float* Lp, float* Rp, hipStream_t st);
// Destination of the GEMM: D (row stride ldc) <- alpha * result + beta * D; D is not read when beta == 0.
struct GemmOut {
    float* C;
    int ldc;
    float alpha, beta;
};
// result = diag(sA) (Aq . BqT^T) diag(sB) [+ Lp . Rp^T when Lp != null]; optional raw int32 output
// (M x N, dense).
int launch_int8_gemm(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, const float* sA,
                     const float* sB, const float* Lp, const float* Rp, int R2P, GemmOut C,
                     int32_t* Cint, hipStream_t st);
// The product with an empty reduction (K == 0): D <- alpha * 0 + beta * D (D not read when beta == 0) and,
// when Cint is given, zeros in Cint.  Reads no operand.
int launch_empty_product(int M, int N, GemmOut C, int32_t* Cint, hipStream_t st);
// The raw int32 sums alone (C_int, row stride N), for a chip on which only `resident` CUs are
// free (0: unknown): with one 256x256 tile per workgroup, the tiles beyond a whole number of
// rounds over those CUs would cost a full extra round; they are cut along K instead, one
// workgroup per range, which leave partial sums in `part` (int8_gemm_sums_scratch_bytes; null:
// no cut), and launch_int8_gemm_sums_finish (same arguments, later on the same stream) adds
// them up into C_int.  Integer sums: the result is bit-identical to the plain kernel's.
#define LRQ_SUMS_MAX_PARTS 64       // (tile, range) pairs at most
size_t int8_gemm_sums_scratch_bytes(int M, int N, int K);
int launch_int8_gemm_sums(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, int32_t* Cint, int resident,
                          int32_t* part, hipStream_t st);
int launch_int8_gemm_sums_finish(int M, int N, int K, const int8_t* Aq, const int8_t* BqT, int32_t* Cint, int resident,
                                 const int32_t* part, hipStream_t st);
// True when launch_int8_gemm uses the large-tile kernel, which accepts C == null together with
// Cint != null (raw int32 sums only; sA, sB are then not read).
bool int8_gemm_large_tiles(int M, int N);
// True when the integer product may run early and launch_rank_update finish the job: the
// large-tile kernel applies, N % 4 == 0 and C is 16-byte aligned.
bool rank_update_usable(int M, int N, const float* C);
// C (dense, holding raw int32 sums in its memory) <- alpha (float(Cint) sA_i sB_j + Lp . Rp^T), in place.
int launch_rank_update(int M, int N, float* C, const float* sA, const float* sB, const float* Lp, const float* Rp,
                       int R2P, float alpha, hipStream_t st);
