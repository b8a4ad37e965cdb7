/*
 * lrqmm.h -- C ABI of the MI355X (gfx950) LRQMM library.
 *
 * LRQMM = low-rank residual quantized matrix multiplication: C ~ A.B with A, B
 * float32, computed as an N-bit integer GEMM plus a rank-r correction obtained
 * from a randomized SVD of the quantization residuals (paper: Methodology,
 * Algorithm 2).
 *
 * Conventions for every entry point
 *  - All matrix/vector pointers are DEVICE pointers owned by the caller (e.g. a
 *    torch tensor's data_ptr()); the library never allocates or frees memory and
 *    writes only the declared outputs and the caller's workspace.
 *  - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *    only enqueue work on that stream; they do not synchronise with the host.
 *  - Matrices are dense row-major float32 unless stated.  Inputs must be finite.
 *  - Return value: LRQMM_OK or a negative LRQMM_ERR_* code (no exceptions, no
 *    errno).  Zero-sized problems return LRQMM_OK and do nothing.
 *  - bits N in [2, 8]; qmax = 2^(N-1)-1; codes are sign-extended int8 in
 *    [-qmax-1, qmax] (int4 codes live in int8 operands).
 *  - A scale group is a row (axis LRQMM_AXIS_ROW, operand A) or a column (axis
 *    LRQMM_AXIS_COL, operand B) -- vector-wise quantization, Background 2.2.  The
 *    `amax` arrays hold the raw absolute maxima; every kernel re-derives
 *    lambda = fl32(qmax/amax) and the step s = fl32(amax/qmax) by one IEEE
 *    division each (Eq. (quantA)); amax < 1e-30 means lambda = s = 0.
 */
#ifndef LRQMM_H
#define LRQMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LRQMM_API __attribute__((visibility("default")))

#define LRQMM_OK                 0
#define LRQMM_ERR_INVALID_ARG   -1   /* null pointer, negative size, rank out of range */
#define LRQMM_ERR_UNSUPPORTED   -2   /* bits outside [2,8], K too large for int32, l > LRQMM_MAX_SKETCH */
#define LRQMM_ERR_WORKSPACE     -3   /* workspace missing, misaligned or too small */
#define LRQMM_ERR_HIP           -4   /* a HIP launch failed */
#define LRQMM_ERR_STATIC_LIMIT  -5   /* lrqmm_gemm_static: the problem needs more than LRQMM_STATIC_SCRATCH_BYTES */

#define LRQMM_AXIS_ROW  0
#define LRQMM_AXIS_COL  1

#define LRQMM_ROUND_FLOOR    0   /* round down: residual entries in [0, s)  (Eq. (get_ra2)) */
#define LRQMM_ROUND_NEAREST  1   /* round to nearest, ties to even          (Eq. (quantAB)) */

/* Largest supported extent of any matrix dimension (M, N, K, rows, cols); an M x N output may further have
 * at most 2^31 - 1 tiles of 128 x 128.  Beyond that the entry points return LRQMM_ERR_UNSUPPORTED (the size
 * functions return 0): host-side block, grid and padding arithmetic is in int. */
#define LRQMM_MAX_DIM (1 << 24)

#define LRQMM_SCALE_VECTOR   0   /* one scale per row of A / per column of B (Background 2.2) */
#define LRQMM_SCALE_TENSOR   1   /* one scale per matrix, as in the paper's own equations (Eq. (quantA)) */

/* Arithmetic of the compensation path (Methodology, text after Eq. (gemm_r_split): the compensation terms
 * may be computed in the original precision or in half precision).  It selects how the float32 operands of
 * the residual products R.Omega, R^T Q, R Z, Q^T R and the factors in A~ W, V^T B~ enter the bfloat16 matrix
 * cores: as three bfloat16 planes each with the six plane products of weight >= 2^-16 (float32 accuracy),
 * as two planes with three products (relative error of a product 2^-16), or as plain bfloat16 values (2^-8).
 * Quantization, the integer product, the Gram/Cholesky/eigen steps (float64) and the rank-2r update of C
 * (float32) are the same in every mode.  Shapes that take the float32 matrix-core kernels (sketches of up to
 * 16 columns in LRQMM_PREC_FP32 only; reduction lengths that are no multiple of 16 in the code products) are
 * computed at full precision.  `bench.py --precision-modes` measures time and error of every mode. */
#define LRQMM_PREC_FP32    0     /* default: float32-equivalent, results match the float64 oracle to 1e-5 */
#define LRQMM_PREC_BF16X2  1     /* two bfloat16 planes per operand */
#define LRQMM_PREC_BF16    2     /* one bfloat16 plane per operand: "half precision" */
#define LRQMM_PREC_SUBSPACE_BF16X2  3   /* two planes in the sketch and power-iteration products, which only shape
                                           the subspace; three planes where values enter C (Q^T R, code products) */

#define LRQMM_MAX_SKETCH  80     /* largest supported sketch width l = rank + oversample */

/* Human-readable text for a status code (static storage). */
LRQMM_API const char* lrqmm_status_string(int status);

/* Bytes of device workspace that lrqmm_rsvd / lrqmm_gemm / lrqmm_matmul need for
 * a problem of this size (the maximum over the three).  The workspace must be
 * 256-byte aligned.  Returns 0 for invalid arguments. */
LRQMM_API size_t lrqmm_workspace_bytes(int M, int N, int K, int rank, int oversample);

/*
 * Symmetric data-free quantization (Background 2.2, Eq. (quantA); floor variant
 * Methodology Eq. (get_ra2); Algorithm 2, quantization step).
 *   X      rows x cols float32, row-major (device, read only)
 *   axis   LRQMM_AXIS_ROW: one scale per row,  amax[rows],
 *                          codes rows x cols row-major;
 *          LRQMM_AXIS_COL: one scale per column, amax[cols],
 *                          codes stored TRANSPOSED, cols x rows row-major
 *                          (so both GEMM operands are contiguous along K).
 *   code = clamp(floor_or_rint(fl32(lambda * x)), -qmax-1, qmax)
 * Outputs: codes (int8), amax (float32).  Bit-exact and order-independent.
 */
LRQMM_API int lrqmm_quantize(const float* X, int rows, int cols, int axis, int bits, int round_mode,
                   int8_t* codes, float* amax, void* stream);

/*
 * The same with a leading dimension and a choice of scale granularity.
 *   ldx         row stride of X in elements, ldx >= cols (X is a window of a larger
 *               row-major array; codes are always stored densely)
 *   scale_mode  LRQMM_SCALE_VECTOR: as lrqmm_quantize;
 *               LRQMM_SCALE_TENSOR: a single lambda = qmax / max|X| for the whole
 *               matrix (Eq. (quantA) as printed); every entry of amax then holds that
 *               global maximum, so all later stages take the array unchanged.
 * Errors: LRQMM_ERR_INVALID_ARG for ldx < cols or an unknown scale_mode.
 */
LRQMM_API int lrqmm_quantize_ex(const float* X, int ldx, int rows, int cols, int axis, int bits,
                      int round_mode, int scale_mode, int8_t* codes, float* amax, void* stream);

/*
 * Gaussian test matrix of the randomized range finder (Background 2.1, stage 1).
 * omega is rows x cols float32 row-major; element (i, j) is a function of
 * (seed, stream_id, i, j) only: splitmix64 counter hash -> two 24-bit uniforms ->
 * Box-Muller, evaluated in float64 with a fixed operation order and rounded to
 * float32.  stream_id 0 is used for R_A, 1 for R_B.
 */
LRQMM_API int lrqmm_fill_sketch(uint64_t seed, int stream_id, int rows, int cols, float* omega,
                      void* stream);

/*
 * Rank-`rank` randomized SVD of the quantization residual
 *     R = X - Dequant(Quant(X))          (Algorithm 2, residual and RSVD steps; Algorithm 1)
 * R is never stored: it is regenerated from X and amax inside every pass.
 *   X, amax, rows, cols, axis, bits, round_mode   as for lrqmm_quantize
 *   rank r >= 1, oversample p >= 0, l = r + p <= min(rows, cols, LRQMM_MAX_SKETCH)
 *   power_iters q >= 0: Y = R.Omega, Q = orth(Y); q times Z = orth(R^T Q),
 *          Q = orth(R Z); B = Q^T R; SVD of B truncated to r (Eq. (k-svd)); U = Q U'.
 *   omega_or_null  optional cols x l sketch (row-major) replacing the internal
 *          generator (which uses lrqmm_fill_sketch(seed, axis, cols, l)).
 * Outputs: U rows x rank, Sigma[rank] (descending), Vt rank x cols, row-major.
 * Singular vectors are defined up to sign; only U.diag(Sigma).Vt is unique.
 */
LRQMM_API int lrqmm_rsvd(const float* X, const float* amax, int rows, int cols, int axis, int bits,
               int round_mode, int rank, int oversample, int power_iters, uint64_t seed,
               const float* omega_or_null, float* U, float* Sigma, float* Vt,
               void* workspace, size_t workspace_bytes, void* stream);

/* lrqmm_rsvd for an X with row stride ldx >= cols (elements) and a choice of arithmetic for the four
 * residual products (precision: LRQMM_PREC_*; anything else is LRQMM_ERR_INVALID_ARG). */
LRQMM_API int lrqmm_rsvd_ex(const float* X, int ldx, const float* amax, int rows, int cols, int axis, int bits,
                  int round_mode, int rank, int oversample, int power_iters, uint64_t seed,
                  const float* omega_or_null, int precision, float* U, float* Sigma, float* Vt,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Quantized GEMM with fused dequantization and rank-2r compensation
 * (Eq. (INTGEMM), Eq. (QUANTGEMM); Algorithm 2, integer product, dequantization and compensation steps):
 *   C[i,j] = sA[i] sB[j] sum_k Aq[i,k] BqT[j,k]
 *            + (U Sig)(Vt B~) + (A~ W)(Gam Zt) + (U Sig)(Vt W)(Gam Zt)
 * with A~ = diag(sA) Aq, B~ = Bq diag(sB).
 *   Aq   M x K int8 row-major;  BqT  N x K int8 row-major (B's codes transposed)
 *   amaxA[M], amaxB[N]          raw absolute maxima (steps are re-derived)
 *   U M x rank, Sig[rank], Vt rank x K     factors of R_A
 *   W K x rank, Gam[rank], Zt rank x N     factors of R_B
 *   rank == 0: factor pointers are ignored; plain direct-quantization product.
 *   C    M x N float32 row-major (output)
 *   Cint_or_null  optional M x N int32 output of the raw integer accumulators.
 * K must satisfy K * (qmax+1)^2 < 2^31.
 */
LRQMM_API int lrqmm_gemm(int M, int N, int K, int bits, int rank,
               const int8_t* Aq, const float* amaxA, const int8_t* BqT, const float* amaxB,
               const float* U, const float* Sig, const float* Vt,
               const float* W, const float* Gam, const float* Zt,
               float* C, int32_t* Cint_or_null,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * lrqmm_gemm followed by the last step of Algorithm 2, fused into the store phase of
 * the GEMM:   D <- alpha * C_F + beta * D,   C_F being what lrqmm_gemm would write.
 *   alpha, beta  float32 scalars, passed by value
 *   D     M x N float32, row stride ldd >= N elements; input and output.  With
 *         beta == 0 the old contents are never read (they may be uninitialised or NaN).
 *   The products alpha * C_F and beta * D are rounded separately and then added
 *   (no fused multiply-add).  Cint_or_null stays dense (row stride N).
 * Errors: LRQMM_ERR_INVALID_ARG for ldd < N, otherwise as lrqmm_gemm.
 */
LRQMM_API int lrqmm_gemm_ex(int M, int N, int K, int bits, int rank,
                  const int8_t* Aq, const float* amaxA, const int8_t* BqT, const float* amaxB,
                  const float* U, const float* Sig, const float* Vt,
                  const float* W, const float* Gam, const float* Zt,
                  float alpha, float beta, float* D, int ldd, int32_t* Cint_or_null,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * lrqmm_gemm_ex for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results; the scratch memory (step vectors, padded factor copies, partial
 * code products and the two panels of the rank-2r update) is a fixed array of
 * LRQMM_STATIC_SCRATCH_BYTES bytes inside the library's device image, one copy per GPU, held until
 * the process ends.  The call allocates and frees nothing.  (Its first call on a device looks the
 * array's address up; make that call outside a capture.)
 * Problems that need more than LRQMM_STATIC_SCRATCH_BYTES return LRQMM_ERR_STATIC_LIMIT and enqueue
 * nothing (the need is what lrqmm_workspace_bytes reports for lrqmm_gemm alone, about
 * 4 (M + N) (3 rank + 4 rank * splits) + 20 K rank bytes; 16 MiB covers M = N = K = 4096 at rank 32).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race on it and must be serialised by the caller; a call does not depend on what an
 * earlier call left there (every word a kernel reads is written earlier in the same call).
 */
#define LRQMM_STATIC_SCRATCH_BYTES (16u << 20)
LRQMM_API int lrqmm_gemm_static(int M, int N, int K, int bits, int rank,
                      const int8_t* Aq, const float* amaxA, const int8_t* BqT, const float* amaxB,
                      const float* U, const float* Sig, const float* Vt,
                      const float* W, const float* Gam, const float* Zt,
                      float alpha, float beta, float* D, int ldd, int32_t* Cint_or_null, void* stream);

/*
 * The whole hot path, all of Algorithm 2 except its final alpha/beta update, from float32 A (M x K) and
 * B (K x N) to float32 C (M x N): quantize both operands, factor both residuals
 * (sketch seeds (seed, 0) and (seed, 1)), integer GEMM, fused compensation.
 * rank == 0 runs the direct-quantization pipeline only.
 * With rank > 0 the work on A (quantization, factorization of R_A) is enqueued on
 * a second stream owned by the library (created on first use, default priority),
 * forked from and joined back into `stream` with events, so the call is still
 * ordered like a single-stream call from the caller's point of view.  For large
 * problems with a sketch of at least 32 columns (a small SVD long enough to hide it)
 * the integer product is enqueued on a third library stream while both
 * factorizations are in their small SVD (the GPU is nearly idle then); it leaves
 * raw int32 sums in C's memory, and the dequantizing rank-2r update runs after the
 * panels as a kernel of its own with the arithmetic of the fused epilogue (same
 * bits for panels of up to 64 columns, 2 rank <= 64; wider panels are accumulated from
 * bfloat16 planes, float32-equivalent but in another rounding order).  C must therefore not be read between the call and its completion on
 * `stream`.  Calls must not be issued concurrently from several host threads.
 * The call enqueues only kernels and event waits (memory is cleared by fill kernels), so it may be
 * recorded into a HIP graph by stream capture on `stream`; the library's own streams join the
 * capture through their fork event.  The call asks hipStreamIsCapturing itself: under capture it creates
 * nothing and returns LRQMM_ERR_UNSUPPORTED (nothing enqueued) if profiling is enabled (timing events do not
 * belong in a graph) or if this device's streams and events do not exist yet -- they are created by the first
 * call with rank > 0 outside a capture, so make one such call first.
 */
LRQMM_API int lrqmm_matmul(int M, int N, int K, int bits, int rank, int oversample, int power_iters,
                 uint64_t seed, int round_mode, const float* A, const float* B, float* C,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * All of Algorithm 2 including its last step, D <- alpha * C_F + beta * D, for operands
 * that are windows of larger row-major arrays:
 *   A  M x K, row stride lda >= K;   B  K x N, row stride ldb >= N;
 *   D  M x N, row stride ldd >= N, input (unless beta == 0) and output
 *   scale_mode  LRQMM_SCALE_VECTOR or LRQMM_SCALE_TENSOR (see lrqmm_quantize_ex)
 *   precision   LRQMM_PREC_*: arithmetic of the residual products of both factorizations and of the
 *               code products A~ W, V^T B~ in the panels
 * lrqmm_matmul is this call with dense operands, alpha = 1, beta = 0, vector
 * scales and LRQMM_PREC_FP32.  Schedule and stream rules are those of lrqmm_matmul; the early integer
 * product is used only when beta == 0 and ldd == N (it needs D's memory for the raw
 * sums), otherwise the update is fused into the GEMM's store phase.  Strides that are
 * not multiples of 4 elements (or bases that are not 16-byte aligned) select the
 * scalar-load variants of the streaming kernels.
 * Errors: LRQMM_ERR_INVALID_ARG for a stride below the row length or an unknown
 * scale_mode or precision, otherwise as lrqmm_matmul.
 */
LRQMM_API int lrqmm_matmul_ex(int M, int N, int K, int bits, int rank, int oversample, int power_iters,
                    uint64_t seed, int round_mode, int scale_mode, int precision,
                    const float* A, int lda, const float* B, int ldb,
                    float alpha, float beta, float* D, int ldd,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Complete residual compensation (Methodology, Eq. (gemm_r_split)) -- the full-size
 * alternative that LRQMM replaces by low-rank terms, kept as a measured baseline:
 * the residual of each operand is quantized a second time with scales of its own and
 *     D <- alpha * (A~ B~ + A~ R~_B + R~_A B~ + R~_A R~_B) + beta * D
 * is evaluated with one integer GEMM per term, taking the first `terms` terms:
 *   terms = 1  direct quantization;  3  the variant the Evaluation calls QT(1,1,0);
 *   terms = 4  all four, QT(1,1,1).
 *
 * lrqmm_quantize_residual: second-level quantization of X (layout, axis, bits, round
 * and scale modes as lrqmm_quantize_ex).  amax0 (device, read only) holds the group
 * maxima that the first quantization of X returned; the value quantized is the
 * float32 residual fl32(x - code0 * s0).  Outputs: codesR (int8, layout as
 * lrqmm_quantize), amaxR (the residual's own group maxima; must not alias amax0).
 *
 * lrqmm_residual_matmul: A (M x K, stride lda), B (K x N, stride ldb), D (M x N, stride
 * ldd) as in lrqmm_matmul_ex; every kernel runs on `stream`.  The workspace (256-byte
 * aligned, lrqmm_residual_workspace_bytes(M, N, K) bytes) holds both levels of codes.
 * Errors: LRQMM_ERR_INVALID_ARG for terms outside {1, 3, 4}, otherwise as lrqmm_matmul_ex.
 */
LRQMM_API int lrqmm_quantize_residual(const float* X, int ldx, const float* amax0, int rows, int cols,
                            int axis, int bits, int round_mode, int scale_mode,
                            int8_t* codesR, float* amaxR, void* stream);
LRQMM_API size_t lrqmm_residual_workspace_bytes(int M, int N, int K);
LRQMM_API int lrqmm_residual_matmul(int M, int N, int K, int bits, int terms, int round_mode, int scale_mode,
                          const float* A, int lda, const float* B, int ldb,
                          float alpha, float beta, float* D, int ldd,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage timing of lrqmm_matmul for measurement (the split of Algorithm 2 into
 * quantization, the two residual factorizations, panel preparation and the
 * integer GEMM with its fused epilogue).  While enabled, each lrqmm_matmul call
 * records HIP events on its stream at the stage boundaries (up to 512 calls
 * between reads).  lrqmm_profile_read waits for the last recorded call (host
 * synchronisation), writes the per-stage mean duration in milliseconds to
 * stage_ms[LRQMM_PROF_STAGES] (host pointer) and the number of calls averaged to
 * *ncalls (host pointer), then resets the call counter.  Not thread safe.
 *   stage 0 quantize A   stage 1 RSVD of R_A     (stages 0-1 and 2-3 run concurrently: the larger
 *   stage 2 quantize B   stage 3 RSVD of R_B      operand's on the caller's stream, the other's on
 *                                                 the library's second stream)
 *   stage 4 compensation panels
 *   stage 5 int8 GEMM kernel with fused epilogue, or -- when the integer product ran early,
 *           see lrqmm_matmul -- the dequantizing rank-2r update kernel alone
 *   stage 6 the early integer product on the library's third stream (0 when fused)
 *
 * lrqmm_profile_enable(LRQMM_PROF_GEMM_ONLY) records only the two events around the integer
 * GEMM kernel, on the stream that kernel is launched on (for the early product that is the
 * library's third stream, off the critical path), so a timed run is not lengthened by the other
 * nine records; lrqmm_profile_read then fills stage 5 or 6 only.  1 = all stages, 0 = off.
 */
#define LRQMM_PROF_STAGES 7
#define LRQMM_PROF_GEMM_ONLY 2
LRQMM_API int lrqmm_profile_enable(int on);
LRQMM_API int lrqmm_profile_read(float* stage_ms, int* ncalls);

#ifdef __cplusplus
}
#endif
#endif /* LRQMM_H */
