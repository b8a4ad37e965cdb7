// Host-side check of the library's argument validation and workspace carving, meant to be linked against a
// build of the library whose host code is compiled with -DLRQMM_CHECK, AddressSanitizer and
// UndefinedBehaviorSanitizer (paper_2409_18772_amd/build.py, build_host_check).  It needs no GPU and touches
// none: every call below either computes a size or is made with an argument error or a workspace that is
// too small, and the entry points return LRQMM_ERR_* for those before their first HIP call.  The operand
// pointers are made-up addresses that host code only forms and compares, never dereferences.
// What a run checks: no signed overflow, no misaligned or overflowing region in the carving arithmetic
// (sanitizers and the LRQMM_CHECK assertions, over shapes up to 2^17 per dimension), the error code of every
// rejected argument, and that the size functions are consistent with what the entry points accept.
#include "lrqmm.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>

static int g_fail = 0;
static long g_checks = 0;
#define EXPECT_EQ(got, want, ...)                                              \
    do {                                                                       \
        ++g_checks;                                                            \
        const long long g_ = (long long)(got), w_ = (long long)(want);        \
        if (g_ != w_) {                                                        \
            ++g_fail;                                                          \
            std::printf("FAIL %s:%d: got %lld, want %lld: ", __FILE__, __LINE__, g_, w_); \
            std::printf(__VA_ARGS__);                                          \
            std::printf("\n");                                                 \
        }                                                                      \
    } while (0)

template <typename T>
static T* fake(uintptr_t where) { return reinterpret_cast<T*>(where); }

int main() {
    // disjoint made-up regions, all 256-byte aligned
    float* A = fake<float>(0x10000000000ull);
    float* B = fake<float>(0x20000000000ull);
    float* D = fake<float>(0x30000000000ull);
    void* ws = fake<void>(0x40000000000ull);
    int8_t* Aq = fake<int8_t>(0x50000000000ull);
    int8_t* Bq = fake<int8_t>(0x60000000000ull);
    float* f1 = fake<float>(0x70000000000ull);
    const int dims[] = {1, 7, 63, 64, 255, 256, 1000, 4096, 4100, 16384, 65536, 100352, 131072, LRQMM_MAX_DIM};
    const int ranks[] = {0, 1, 8, 32, 64, 80};
    const int overs[] = {0, 8, 16};
    const int nd = sizeof(dims) / sizeof(dims[0]);
    for (int im = 0; im < nd; ++im)
        for (int in = 0; in < nd; ++in)
            for (int ik = 0; ik < nd; ++ik) {
                const int M = dims[im], N = dims[in], K = dims[ik];
                const size_t w0 = lrqmm_workspace_bytes(M, N, K, 0, 0);
                if ((long long)((M + 127) / 128) * ((N + 127) / 128) >= (1ll << 31)) {   // more tiles than a grid holds
                    EXPECT_EQ(w0, 0, "output too large M=%d N=%d", M, N);
                    EXPECT_EQ(lrqmm_residual_workspace_bytes(M, N, K), 0, "output too large M=%d N=%d", M, N);
                    continue;
                }
                EXPECT_EQ(w0 > 0, 1, "rank-0 workspace M=%d N=%d K=%d", M, N, K);
                const size_t wr = lrqmm_residual_workspace_bytes(M, N, K);
                EXPECT_EQ(wr >= 2 * ((size_t)M * K + (size_t)N * K), 1, "two levels of codes M=%d N=%d K=%d", M, N, K);
                // a workspace one byte short of what the carving needs is refused (and the carving runs in full)
                EXPECT_EQ(lrqmm_residual_matmul(M, N, K, 4, 4, LRQMM_ROUND_FLOOR, LRQMM_SCALE_VECTOR, A, K, B, N, 1.0f,
                                                0.0f, D, N, ws, wr - 257, nullptr),
                          LRQMM_ERR_WORKSPACE, "residual_matmul short workspace M=%d N=%d K=%d", M, N, K);
                for (int r : ranks)
                    for (int p : overs) {
                        const int ell = r + p;
                        const size_t w = lrqmm_workspace_bytes(M, N, K, r, p);
                        if (ell > LRQMM_MAX_SKETCH) {
                            EXPECT_EQ(w, 0, "sketch too wide r=%d p=%d", r, p);
                            continue;
                        }
                        EXPECT_EQ(w >= w0, 1, "workspace grows with the rank");
                        if (r == 0) continue;
                        const bool fits = ell <= M && ell <= N && ell <= K;
                        const int rc = lrqmm_matmul_ex(M, N, K, 4, r, p, 1, 1, LRQMM_ROUND_FLOOR, LRQMM_SCALE_VECTOR,
                                                       LRQMM_PREC_FP32, A, K, B, N, 1.0f, 0.0f, D, N, ws, w - 257, nullptr);
                        EXPECT_EQ(rc, fits ? LRQMM_ERR_WORKSPACE : LRQMM_ERR_INVALID_ARG,
                                  "matmul_ex short workspace M=%d N=%d K=%d r=%d p=%d", M, N, K, r, p);
                        if (!fits) continue;
                        EXPECT_EQ(lrqmm_rsvd_ex(A, K, f1, M, K, LRQMM_AXIS_ROW, 4, LRQMM_ROUND_FLOOR, r, p, 1, 1, nullptr,
                                                LRQMM_PREC_FP32, f1, f1, f1, ws, 1024, nullptr),
                                  LRQMM_ERR_WORKSPACE, "rsvd_ex short workspace rows=%d cols=%d r=%d p=%d", M, K, r, p);
                        EXPECT_EQ(lrqmm_rsvd_ex(B, N, f1, K, N, LRQMM_AXIS_COL, 4, LRQMM_ROUND_FLOOR, r, p, 2, 1, nullptr,
                                                LRQMM_PREC_BF16X2, f1, f1, f1, ws, 1024, nullptr),
                                  LRQMM_ERR_WORKSPACE, "rsvd_ex short workspace rows=%d cols=%d r=%d p=%d", K, N, r, p);
                        if (p == 0)
                            EXPECT_EQ(lrqmm_gemm_ex(M, N, K, 4, r, Aq, f1, Bq, f1, f1, f1, f1, f1, f1, f1, 1.0f, 0.0f, D, N,
                                                    nullptr, ws, 1024, nullptr),
                                      LRQMM_ERR_WORKSPACE, "gemm_ex short workspace M=%d N=%d K=%d r=%d", M, N, K, r);
                    }
            }

    // rejected arguments, one at a time (nothing is enqueued for any of them)
    const size_t big = (size_t)1 << 40;
    EXPECT_EQ(lrqmm_workspace_bytes(-1, 4, 4, 0, 0), 0, "negative size");
    EXPECT_EQ(lrqmm_residual_workspace_bytes(4, -1, 4), 0, "negative size");
#define MATMUL(M, N, K, bits, r, p, q, rm, sm, pr, lda, ldb, ldd, wsp, wsb) \
    lrqmm_matmul_ex(M, N, K, bits, r, p, q, 1, rm, sm, pr, A, lda, B, ldb, 1.0f, 0.0f, D, ldd, wsp, wsb, nullptr)
    EXPECT_EQ(MATMUL(-1, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 8, 8, ws, big), LRQMM_ERR_INVALID_ARG, "negative M");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 0, 0, 0, 7, 8, 8, ws, big), LRQMM_ERR_INVALID_ARG, "lda < K");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 7, 8, ws, big), LRQMM_ERR_INVALID_ARG, "ldb < N");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 8, 7, ws, big), LRQMM_ERR_INVALID_ARG, "ldd < N");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 2, 0, 0, 8, 8, 8, ws, big), LRQMM_ERR_INVALID_ARG, "round mode");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 0, 2, 0, 8, 8, 8, ws, big), LRQMM_ERR_INVALID_ARG, "scale mode");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 2, 0, 0, 0, 0, 4, 8, 8, 8, ws, big), LRQMM_ERR_INVALID_ARG, "precision");
    const int over = LRQMM_MAX_DIM + 1, imax = 2147483647;
    EXPECT_EQ(lrqmm_workspace_bytes(over, 8, 8, 0, 0), 0, "dimension above the limit");
    EXPECT_EQ(lrqmm_workspace_bytes(imax, imax, imax, 8, 0), 0, "dimension above the limit");
    EXPECT_EQ(lrqmm_workspace_bytes(LRQMM_MAX_DIM, 4096, LRQMM_MAX_DIM, 64, 16) > 0, 1, "largest dimensions");
    EXPECT_EQ(lrqmm_residual_workspace_bytes(8, imax, 8), 0, "dimension above the limit");
    EXPECT_EQ(MATMUL(over, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 8, 8, ws, big), LRQMM_ERR_UNSUPPORTED, "M above the limit");
    EXPECT_EQ(MATMUL(8, 8, imax, 4, 0, 0, 0, 0, 0, 0, imax, 8, 8, ws, big), LRQMM_ERR_UNSUPPORTED, "K above the limit");
    EXPECT_EQ(lrqmm_quantize_ex(A, imax, 8, imax, LRQMM_AXIS_ROW, 4, 0, 0, Aq, f1, nullptr), LRQMM_ERR_UNSUPPORTED,
              "cols above the limit");
    EXPECT_EQ(lrqmm_rsvd_ex(A, over, f1, 8, over, LRQMM_AXIS_ROW, 4, 0, 2, 0, 0, 1, nullptr, 0, f1, f1, f1, ws, big, nullptr),
              LRQMM_ERR_UNSUPPORTED, "cols above the limit");
    EXPECT_EQ(lrqmm_residual_matmul(8, over, 8, 4, 3, 0, 0, A, 8, B, over, 1.0f, 0.0f, D, over, ws, big, nullptr),
              LRQMM_ERR_UNSUPPORTED, "N above the limit");
    EXPECT_EQ(MATMUL(8, 8, 8, 1, 0, 0, 0, 0, 0, 0, 8, 8, 8, ws, big), LRQMM_ERR_UNSUPPORTED, "1 bit");
    EXPECT_EQ(MATMUL(8, 8, 8, 9, 0, 0, 0, 0, 0, 0, 8, 8, 8, ws, big), LRQMM_ERR_UNSUPPORTED, "9 bits");
    EXPECT_EQ(MATMUL(8, 8, 1 << 20, 8, 0, 0, 0, 0, 0, 0, 1 << 20, 8, 8, ws, big), LRQMM_ERR_UNSUPPORTED,
              "K too long for int32 sums at 8 bits");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 6, 4, 0, 0, 0, 0, 8, 8, 8, ws, big), LRQMM_ERR_INVALID_ARG, "sketch wider than the matrix");
    EXPECT_EQ(MATMUL(128, 128, 128, 4, 64, 32, 0, 0, 0, 0, 128, 128, 128, ws, big), LRQMM_ERR_UNSUPPORTED,
              "sketch wider than the library's limit");
    EXPECT_EQ(MATMUL(0, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 8, 8, ws, big), LRQMM_OK, "empty output");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 8, 8, nullptr, big), LRQMM_ERR_WORKSPACE, "no workspace");
    EXPECT_EQ(MATMUL(8, 8, 8, 4, 0, 0, 0, 0, 0, 0, 8, 8, 8, fake<void>(0x40000000010ull), big), LRQMM_ERR_WORKSPACE,
              "misaligned workspace");
    EXPECT_EQ(lrqmm_matmul_ex(8, 8, 8, 4, 0, 0, 0, 1, 0, 0, 0, nullptr, 8, B, 8, 1.0f, 0.0f, D, 8, ws, big, nullptr),
              LRQMM_ERR_INVALID_ARG, "null A");
    EXPECT_EQ(lrqmm_matmul_ex(8, 8, 8, 4, 0, 0, 0, 1, 0, 0, 0, A, 8, B, 8, 1.0f, 0.0f, nullptr, 8, ws, big, nullptr),
              LRQMM_ERR_INVALID_ARG, "null D");
    EXPECT_EQ(lrqmm_residual_matmul(8, 8, 8, 4, 2, 0, 0, A, 8, B, 8, 1.0f, 0.0f, D, 8, ws, big, nullptr),
              LRQMM_ERR_INVALID_ARG, "terms outside {1, 3, 4}");
    EXPECT_EQ(lrqmm_quantize_ex(A, 7, 8, 8, LRQMM_AXIS_ROW, 4, 0, 0, Aq, f1, nullptr), LRQMM_ERR_INVALID_ARG, "ldx < cols");
    EXPECT_EQ(lrqmm_quantize_ex(A, 8, 8, 8, 2, 4, 0, 0, Aq, f1, nullptr), LRQMM_ERR_INVALID_ARG, "axis");
    EXPECT_EQ(lrqmm_gemm_static(4096, 4096, 4096, 4, 64, Aq, f1, Bq, f1, f1, f1, f1, f1, f1, f1, 1.0f, 0.0f, D, 4096,
                                nullptr, nullptr),
              LRQMM_ERR_STATIC_LIMIT, "static scratch limit");
    EXPECT_EQ(lrqmm_gemm_static(64, 64, 64, 4, 0, Aq, f1, Bq, f1, f1, f1, f1, f1, f1, f1, 1.0f, 0.0f, D, 63, nullptr,
                                nullptr),
              LRQMM_ERR_INVALID_ARG, "ldd < N");
    for (int s = 1; s >= -6; --s) EXPECT_EQ(lrqmm_status_string(s) != nullptr && lrqmm_status_string(s)[0] != 0, 1, "text");
    std::printf("host_check: %ld checks, %d failures\n", g_checks, g_fail);
    return g_fail ? 1 : 0;
}
