// C-ABI entry points of the LRQMM library: argument validation, workspace
// carving and the launch sequence of each call (paper: Algorithm 2; Algorithm 1
// for lrqmm_rsvd).  No device memory is allocated here; everything lives in the
// caller's buffers and workspace.
#include "kernels.h"
#include <cstdio>
#include <cstdlib>
#include <functional>
#include <vector>

namespace {

struct Arena {
    char* base;
    size_t off;
    explicit Arena(void* b) : base(static_cast<char*>(b)), off(0) {}
    template <typename T>
    T* take(size_t count) {
        off = align_up(off, 256);
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
#ifdef LRQMM_CHECK      // checked host build: sizes must not wrap, regions must stay aligned and ordered
        size_t bytes = 0, end = 0;
        if (__builtin_mul_overflow(count, sizeof(T), &bytes) || __builtin_add_overflow(off, bytes, &end) ||
            (base && ((uintptr_t)p & 255) != 0) || end < off) {
            std::fprintf(stderr, "LRQMM_CHECK: workspace region overflows (count %zu x %zu bytes at offset %zu)\n", count,
                         sizeof(T), off);
            std::abort();
        }
#endif
        off += count * sizeof(T);
        return p;
    }
};

inline int pad_to(int x, int m) { return (x + m - 1) / m * m; }

struct RsvdWs {
    float *lam, *s, *Wc, *Yr, *partial;
    double *gpart, *gram, *T, *Ur, *Mv;
};

size_t carve_rsvd(Arena& a, int rows, int cols, int axis, int LP, int rank, RsvdWs* w) {
    const int nscale = axis == LRQMM_AXIS_ROW ? rows : cols;
    const int npad = pad_to(nscale, 4);
    const PassPlan pn = plan_pass_n(rows, cols), pt = plan_pass_t(rows, cols);
    const size_t part = (size_t)LP * (size_t)((size_t)pn.splits * rows > (size_t)pt.splits * cols
                                                  ? (size_t)pn.splits * rows
                                                  : (size_t)pt.splits * cols);
    // (the block count is not monotone in the row count -- 4096 rows make 64 blocks of 64, 4100 rows 33 of 128 --
    // so take the larger of the two uses, Gram of a rows x LP and of a cols x LP factor)
    // (and the one-read quantization kernel for row-quantized operands leaves one partial per workgroup)
    int nb = gram_blocks(rows, LP) > gram_blocks(cols, LP) ? gram_blocks(rows, LP) : gram_blocks(cols, LP);
    if (axis == LRQMM_AXIS_ROW && LP == 16 && quant_sketch_rows_blocks(rows) > nb) nb = quant_sketch_rows_blocks(rows);
    RsvdWs t;
    t.lam = a.take<float>(npad);
    t.s = a.take<float>(npad);
    t.Wc = a.take<float>((size_t)cols * LP);
    t.Yr = a.take<float>((size_t)rows * LP);
    t.partial = a.take<float>(part);
    t.gpart = a.take<double>((size_t)nb * LP * LP);
    t.gram = a.take<double>((size_t)LP * LP);
    t.T = a.take<double>((size_t)LP * LP);
    t.Ur = a.take<double>((size_t)LP * rank);
    t.Mv = a.take<double>((size_t)LP * rank);
    if (w) *w = t;
    return a.off;
}

struct GemmWs {
    float *lamA, *sA, *lamB, *sB, *Wp, *Vp, *partialA, *partialB, *X, *Lp, *Rp;
    uint16_t *Wp3, *Vp3;
};

size_t carve_gemm(Arena& a, int M, int N, int K, int rank, GemmWs* w) {
    GemmWs t = {};
    const int Mp = pad_to(M, 4), Np = pad_to(N, 4);
    t.lamA = a.take<float>(Mp);
    t.sA = a.take<float>(Mp);
    t.lamB = a.take<float>(Np);
    t.sB = a.take<float>(Np);
    if (rank > 0) {
        const int RP = pad_to(rank, 16), R2P = pad_to(2 * rank, 8);
        const PassPlan pa = plan_pass_n(M, K), pb = plan_pass_n(N, K);
        t.Wp = a.take<float>((size_t)K * RP);
        t.Vp = a.take<float>((size_t)K * RP);
        t.Wp3 = a.take<uint16_t>((size_t)3 * RP * pad_to(K, 64));
        t.Vp3 = a.take<uint16_t>((size_t)3 * RP * pad_to(K, 64));
        t.partialA = a.take<float>((size_t)RP * pa.splits * M);
        t.partialB = a.take<float>((size_t)RP * pb.splits * N);
        t.X = a.take<float>((size_t)rank * rank * LRQ_VTW_MAX_SLICES);
        t.Lp = a.take<float>((size_t)M * R2P);
        t.Rp = a.take<float>((size_t)N * R2P);
    }
    if (w) *w = t;
    return a.off;
}

struct MatmulWs {
    int8_t *Aq, *BqT;
    float *amaxA, *amaxB, *U, *Sig, *Vt, *W, *Gam, *Zt;
    uint32_t* tick;
    int32_t* parts;                   // partial sums of the early integer product's K ranges
    void *sub, *subA, *subB;          // gemm scratch aliases the two rsvd regions
    size_t sub_bytes, subA_bytes, subB_bytes;
};

size_t carve_matmul(Arena& a, int M, int N, int K, int rank, int oversample, MatmulWs* w) {
    MatmulWs t = {};
    t.Aq = a.take<int8_t>((size_t)M * K);
    t.BqT = a.take<int8_t>((size_t)N * K);
    t.amaxA = a.take<float>(M);
    t.amaxB = a.take<float>(N);
    t.tick = a.take<uint32_t>(64);
    t.parts = nullptr;
    if (rank > 0 && int8_gemm_sums_scratch_bytes(M, N, K) > 0)
        t.parts = a.take<int32_t>(int8_gemm_sums_scratch_bytes(M, N, K) / sizeof(int32_t));
    if (rank > 0) {
        t.U = a.take<float>((size_t)M * rank);
        t.Sig = a.take<float>(rank);
        t.Vt = a.take<float>((size_t)rank * K);
        t.W = a.take<float>((size_t)K * rank);
        t.Gam = a.take<float>(rank);
        t.Zt = a.take<float>((size_t)rank * N);
    }
    a.off = align_up(a.off, 256);
    size_t sub = 0, sa = 0, sb = 0;
    {
        Arena g(nullptr);
        sub = carve_gemm(g, M, N, K, rank, nullptr);
    }
    if (rank > 0) {
        // the two residual factorizations run concurrently: each gets its own region
        const int LP = pad_to(rank + oversample, 16);
        Arena ra(nullptr), rb(nullptr);
        sa = align_up(carve_rsvd(ra, M, K, LRQMM_AXIS_ROW, LP, rank, nullptr), 256);
        sb = align_up(carve_rsvd(rb, K, N, LRQMM_AXIS_COL, LP, rank, nullptr), 256);
        if (sa + sb > sub) sub = sa + sb;
    }
    t.sub = a.base ? a.base + a.off : nullptr;
    t.sub_bytes = sub;
    t.subA = t.sub;
    t.subA_bytes = sa;
    t.subB = a.base ? a.base + a.off + sa : nullptr;
    t.subB_bytes = sb;
    a.off += sub;
    if (w) *w = t;
    return a.off;
}

// Optional stage timing of lrqmm_matmul with HIP events recorded on the caller's stream.
constexpr int kProfStages = LRQMM_PROF_STAGES;
constexpr int kProfEvents = 11;
constexpr int kProfMaxCalls = 512;
// event indices: 0-2 main stream (quantize A, RSVD A), 3-5 side stream (quantize B, RSVD B),
// 6-8 main stream after the join (panels, GEMM or rank update), 9-10 the early integer GEMM on
// the third stream (recorded back to back on the main stream when that schedule is not used)
constexpr int kStageBegin[kProfStages] = {0, 1, 3, 4, 6, 7, 9};
constexpr int kStageEnd[kProfStages] = {1, 2, 4, 5, 7, 8, 10};
constexpr int kLastMainEvent = 8;
struct Prof {
    bool on = false;
    bool gemm_only = false;             // record only the pair of events around the integer GEMM
    bool early[kProfMaxCalls] = {};     // per recorded call: the GEMM ran on the third stream
    int ncalls = 0;
    hipEvent_t ev[kProfMaxCalls][kProfEvents];
    bool created = false;
} g_prof;

// Streams and events that lrqmm_matmul needs beyond the caller's stream, one set per device (created on
// the first call on that device, never destroyed: they live as long as the process).  `stream` carries
// A's quantization and factorization next to B's on the caller's stream; `gemm_stream` the early integer
// product.  All at default priority.
struct Side {
    hipStream_t stream = nullptr;        // A's chain
    hipStream_t gemm_stream = nullptr;   // early integer GEMM
    hipEvent_t fork = nullptr, join = nullptr;
    hipEvent_t gate = nullptr, gate_b = nullptr, gdone = nullptr;
    int cus = 0;                         // compute units of the device
    bool ok = false;
};
constexpr int kMaxDevices = 16;
Side g_side_dev[kMaxDevices];

// The current device's set, or null when it does not exist yet and `create` is false (a call under
// stream capture must not create streams) or when creating it failed.
Side* side_state(bool create) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    Side& s = g_side_dev[dev];
    if (s.ok) return &s;
    if (!create) return nullptr;
    if (hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
    if (hipStreamCreateWithFlags(&s.gemm_stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
    for (hipEvent_t* e : {&s.gate, &s.gate_b, &s.gdone, &s.fork, &s.join})
        if (hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess) return nullptr;
    if (hipDeviceGetAttribute(&s.cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return nullptr;
    s.ok = true;
    return &s;
}

// Scratch memory of lrqmm_gemm_static: a fixed array in the library's device image (every GPU that loads
// the library holds its own copy, at its own address, until the process ends).  In host code the array's
// name is only a handle for hipGetSymbolAddress; the device address is looked up once per device, with
// that device current, and kept.
static __device__ __align__(256) unsigned char scratch[LRQMM_STATIC_SCRATCH_BYTES];
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LRQMM_ERR_HIP;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LRQMM_ERR_HIP;
        if ((uintptr_t)ptr & 255) return LRQMM_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LRQMM_OK;
}

inline void prof_mark(int slot, int i, hipStream_t st) {
    if (slot < 0) return;
    if (g_prof.gemm_only) {     // events 9, 10 bracket the early product, 7, 8 the fused kernel
        const bool early = g_prof.early[slot];
        if (!(early ? (i == 9 || i == 10) : (i == 7 || i == 8))) return;
    }
    (void)hipEventRecord(g_prof.ev[slot][i], st);
}

// arithmetic of the entry points that take no precision argument (lrqmm_rsvd, lrqmm_matmul)
#ifndef LRQMM_DEFAULT_PREC
#define LRQMM_DEFAULT_PREC LRQMM_PREC_FP32
#endif
bool bits_ok(int bits) { return bits >= 2 && bits <= 8; }
// Host-side size arithmetic (padding, block counts) is done in int: dimensions stay well below 2^31.
bool dims_ok(int a, int b, int c = 0) { return a <= LRQMM_MAX_DIM && b <= LRQMM_MAX_DIM && c <= LRQMM_MAX_DIM; }
// ... and an M x N output must leave the number of 128 x 128 tiles (a grid size) below 2^31
bool output_ok(int M, int N) { return (long long)((M + 127) / 128) * ((N + 127) / 128) < (1ll << 31); }
bool precision_ok(int p) {
    return p == LRQMM_PREC_FP32 || p == LRQMM_PREC_BF16X2 || p == LRQMM_PREC_BF16 || p == LRQMM_PREC_SUBSPACE_BF16X2;
}
// bfloat16 planes per operand: in the products that only shape the subspace (sketch and power iterations) and in
// the products whose values enter C directly (the projection Q^T R and the code products of the panels)
int planes_subspace(int p) { return p == LRQMM_PREC_BF16 ? 1 : (p == LRQMM_PREC_FP32 ? 3 : 2); }
int planes_values(int p) { return p == LRQMM_PREC_BF16 ? 1 : (p == LRQMM_PREC_BF16X2 ? 2 : 3); }

// int32 accumulation is safe when K * (qmax+1)^2 < 2^31.
bool k_fits_int32(int K, int bits) {
    const long long lim = 1ll << (2 * (bits - 1));
    return (long long)K * lim < (1ll << 31);
}

// A factorization is first planned as a list of kernel launches and then issued, so that
// lrqmm_matmul can issue the launches of its two factorizations alternately: both streams
// then receive work at the same pace instead of one after the other (the host needs several
// microseconds per launch, and each list holds ~30).
using LaunchList = std::vector<std::function<int()>>;

// Issues a[a0 .. a1) and b[b0 .. b1) alternately.
static int run_interleaved(const LaunchList& a, size_t a0, size_t a1, const LaunchList& b, size_t b0, size_t b1) {
    while (a0 < a1 || b0 < b1) {
        if (a0 < a1) {
            const int rc = a[a0++]();
            if (rc != LRQMM_OK) return rc;
        }
        if (b0 < b1) {
            const int rc = b[b0++]();
            if (rc != LRQMM_OK) return rc;
        }
    }
    return LRQMM_OK;
}
static int run_interleaved(const LaunchList& a, const LaunchList& b) {
    return run_interleaved(a, 0, a.size(), b, 0, b.size());
}

// Validates the arguments of lrqmm_rsvd and appends its launches to `ops`.
static int rsvd_plan(LaunchList& ops, const float* X, int ldx, const float* amax, int rows, int cols, int axis, int bits,
                     int round_mode, int rank, int oversample, int power_iters, uint64_t seed,
                     const float* omega_or_null, float* U, float* Sigma, float* Vt, void* workspace,
                     size_t workspace_bytes, hipStream_t st, int precision, size_t* svd_index = nullptr,
                     bool prepared = false, int8_t* fused_codes = nullptr, float* row_amax_out = nullptr) {
    if (rows < 0 || cols < 0 || rank < 1 || oversample < 0 || power_iters < 0 || ldx < cols) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return LRQMM_ERR_UNSUPPORTED;
    if (!precision_ok(precision)) return LRQMM_ERR_INVALID_ARG;
    const int planes = planes_subspace(precision), planes_last = planes_values(precision);
    if (axis != LRQMM_AXIS_ROW && axis != LRQMM_AXIS_COL) return LRQMM_ERR_INVALID_ARG;
    if (round_mode != LRQMM_ROUND_FLOOR && round_mode != LRQMM_ROUND_NEAREST) return LRQMM_ERR_INVALID_ARG;
    if (!bits_ok(bits)) return LRQMM_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return LRQMM_OK;
    const int ell = rank + oversample;
    if (ell > rows || ell > cols) return LRQMM_ERR_INVALID_ARG;
    if (ell > LRQMM_MAX_SKETCH) return LRQMM_ERR_UNSUPPORTED;
    if (!X || !amax || !U || !Sigma || !Vt) return LRQMM_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return LRQMM_ERR_WORKSPACE;
    const int LP = pad_to(ell, 16);
    RsvdWs w;
    Arena a(workspace);
    if (carve_rsvd(a, rows, cols, axis, LP, rank, &w) > workspace_bytes) return LRQMM_ERR_WORKSPACE;
    const QuantParams q = make_quant_params(bits, round_mode);
    const int nscale = axis == LRQMM_AXIS_ROW ? rows : cols;
    if (prepared) {
        // the caller has already filled the sketch (w.Wc) on this stream, and either the step vectors (w.lam, w.s)
        // too or -- with fused_codes -- only the group maxima: the first pass then quantizes as well; with
        // row_amax_out not even those: the first pass reads the operand once for maxima, codes and Y
    } else if (omega_or_null) {
        ops.push_back([=] { return launch_scales(amax, nscale, pad_to(nscale, 4), q.qmaxf, w.lam, w.s, st); });
        ops.push_back([=] { return launch_pad_copy(omega_or_null, cols, ell, LP, w.Wc, st); });
    } else {
        ops.push_back([=] {
            return launch_sketch_and_scales(seed, axis, cols, ell, LP, w.Wc, amax, nscale, pad_to(nscale, 4), q.qmaxf,
                                            w.lam, w.s, st);
        });
    }
    const PassPlan pn = plan_pass_n(rows, cols), pt = plan_pass_t(rows, cols);
    // Q = orth(partial sums) in place: Gram (float64) -> Cholesky -> Q = Y T
    auto orth = [&](int splits, int n, float* buf) {
        ops.push_back([=] { return launch_reduce_gram(w.partial, splits, n, LP, nullptr, buf, w.gpart, st); });
        ops.push_back([=] { return launch_gram_sum(w.gpart, gram_blocks(n, LP), LP, w.gram, st); });
        ops.push_back([=] { return launch_chol_inverse(w.gram, ell, LP, w.T, st); });
        ops.push_back([=] { return launch_apply(buf, n, LP, w.T, LP, LP, buf, LP, 0, st); });
    };
    auto pass_n = [&] {
        ops.push_back([=] { return launch_resid_mul_n(X, ldx, rows, cols, axis, w.lam, w.s, q, w.Wc, LP, pn, w.partial, st, planes); });
    };
    auto pass_t = [&](int pl) {
        ops.push_back([=] { return launch_resid_mul_t(X, ldx, rows, cols, axis, w.lam, w.s, q, w.Yr, LP, pt, w.partial, st, pl); });
    };
    // Y = R Omega (with fused_codes: the same launch also writes the codes and the step vectors)
    if (fused_codes && row_amax_out) {
        // one read of X: maxima, codes, Y (straight into its place) and the Gram partials of Y
        ops.push_back([=] {
            return launch_quant_sketch_rows(X, ldx, rows, cols, q, w.Wc, LP, w.Yr, w.gpart, row_amax_out, w.lam, w.s,
                                            fused_codes, st);
        });
        ops.push_back([=] { return launch_gram_sum(w.gpart, quant_sketch_rows_blocks(rows), LP, w.gram, st); });
        ops.push_back([=] { return launch_chol_inverse(w.gram, ell, LP, w.T, st); });
        ops.push_back([=] { return launch_apply(w.Yr, rows, LP, w.T, LP, LP, w.Yr, LP, 0, st); });
    } else if (fused_codes)
        ops.push_back([=] {
            return launch_quant_sketch(X, ldx, rows, cols, axis, amax, q, w.Wc, LP, pn, w.partial, w.lam, w.s, fused_codes,
                                       st, planes);
        });
    else
        pass_n();
    if (!(fused_codes && row_amax_out)) orth(pn.splits, rows, w.Yr);
    for (int it = 0; it < power_iters; ++it) {
        // Z = orth(R^T Q); Q = orth(R Z)
        pass_t(planes);
        orth(pt.splits, cols, w.Wc);
        pass_n();
        orth(pn.splits, rows, w.Yr);
    }
    // B^T = R^T Q (cols x l), its Gram B B^T, small SVD, U = Q U', V = B^T U' / sigma
    pass_t(planes_last);
    ops.push_back([=] { return launch_reduce_gram(w.partial, pt.splits, cols, LP, nullptr, w.Wc, w.gpart, st); });
    ops.push_back([=] { return launch_gram_sum(w.gpart, gram_blocks(cols, LP), LP, w.gram, st); });
    if (svd_index) *svd_index = ops.size();         // the GPU is nearly idle from this launch to its end
    ops.push_back([=] { return launch_small_svd(w.gram, ell, LP, rank, Sigma, w.Ur, w.Mv, st); });
    ops.push_back([=] {
        return launch_apply2(w.Yr, rows, w.Ur, rank, rank, U, rank, 0, w.Wc, cols, w.Mv, rank, rank, Vt, cols, 1, LP,
                             st);
    });
    return LRQMM_OK;
}

#define LRQ_TRY(x)                  \
    do {                            \
        rc = (x);                   \
        if (rc != LRQMM_OK) return rc; \
    } while (0)

}  // namespace

extern "C" {

const char* lrqmm_status_string(int status) {
    switch (status) {
        case LRQMM_OK: return "ok";
        case LRQMM_ERR_INVALID_ARG: return "invalid argument";
        case LRQMM_ERR_UNSUPPORTED: return "unsupported configuration";
        case LRQMM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LRQMM_ERR_HIP: return "HIP launch failed";
        case LRQMM_ERR_STATIC_LIMIT: return "problem needs more scratch memory than the library's static buffer holds";
        default: return "unknown status";
    }
}

size_t lrqmm_workspace_bytes(int M, int N, int K, int rank, int oversample) {
    if (M < 0 || N < 0 || K < 0 || rank < 0 || oversample < 0 || !dims_ok(M, N, K) || !output_ok(M, N)) return 0;
    if (rank + oversample > LRQMM_MAX_SKETCH) return 0;
    Arena a(nullptr);
    return carve_matmul(a, M, N, K, rank, oversample, nullptr) + 256;
}

int lrqmm_quantize(const float* X, int rows, int cols, int axis, int bits, int round_mode, int8_t* codes,
                   float* amax, void* stream) {
    return lrqmm_quantize_ex(X, cols, rows, cols, axis, bits, round_mode, LRQMM_SCALE_VECTOR, codes, amax, stream);
}

int lrqmm_quantize_ex(const float* X, int ldx, int rows, int cols, int axis, int bits, int round_mode,
                      int scale_mode, int8_t* codes, float* amax, void* stream) {
    if (rows < 0 || cols < 0 || ldx < cols) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return LRQMM_ERR_UNSUPPORTED;
    if (scale_mode != LRQMM_SCALE_VECTOR && scale_mode != LRQMM_SCALE_TENSOR) return LRQMM_ERR_INVALID_ARG;
    if (axis != LRQMM_AXIS_ROW && axis != LRQMM_AXIS_COL) return LRQMM_ERR_INVALID_ARG;
    if (round_mode != LRQMM_ROUND_FLOOR && round_mode != LRQMM_ROUND_NEAREST) return LRQMM_ERR_INVALID_ARG;
    if (!bits_ok(bits)) return LRQMM_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return LRQMM_OK;
    if (!X || !codes || !amax) return LRQMM_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const QuantParams q = make_quant_params(bits, round_mode);
    const bool per_tensor = scale_mode == LRQMM_SCALE_TENSOR;
    if (axis == LRQMM_AXIS_ROW) return launch_quantize_rows(X, ldx, rows, cols, q, per_tensor, nullptr, codes, amax, st);
    return launch_quantize_cols(X, ldx, rows, cols, q, per_tensor, nullptr, codes, amax, st);
}

int lrqmm_quantize_residual(const float* X, int ldx, const float* amax0, int rows, int cols, int axis, int bits,
                            int round_mode, int scale_mode, int8_t* codesR, float* amaxR, void* stream) {
    if (rows < 0 || cols < 0 || ldx < cols) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return LRQMM_ERR_UNSUPPORTED;
    if (scale_mode != LRQMM_SCALE_VECTOR && scale_mode != LRQMM_SCALE_TENSOR) return LRQMM_ERR_INVALID_ARG;
    if (axis != LRQMM_AXIS_ROW && axis != LRQMM_AXIS_COL) return LRQMM_ERR_INVALID_ARG;
    if (round_mode != LRQMM_ROUND_FLOOR && round_mode != LRQMM_ROUND_NEAREST) return LRQMM_ERR_INVALID_ARG;
    if (!bits_ok(bits)) return LRQMM_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return LRQMM_OK;
    if (!X || !amax0 || !codesR || !amaxR || amax0 == amaxR) return LRQMM_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const QuantParams q = make_quant_params(bits, round_mode);
    const bool per_tensor = scale_mode == LRQMM_SCALE_TENSOR;
    if (axis == LRQMM_AXIS_ROW) return launch_quantize_rows(X, ldx, rows, cols, q, per_tensor, amax0, codesR, amaxR, st);
    return launch_quantize_cols(X, ldx, rows, cols, q, per_tensor, amax0, codesR, amaxR, st);
}

int lrqmm_fill_sketch(uint64_t seed, int stream_id, int rows, int cols, float* omega, void* stream) {
    if (rows < 0 || cols < 0 || stream_id < 0) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return LRQMM_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return LRQMM_OK;
    if (!omega) return LRQMM_ERR_INVALID_ARG;
    return launch_fill_sketch(seed, stream_id, rows, cols, cols, omega, static_cast<hipStream_t>(stream));
}

int lrqmm_rsvd(const float* X, const float* amax, int rows, int cols, int axis, int bits, int round_mode,
               int rank, int oversample, int power_iters, uint64_t seed, const float* omega_or_null, float* U,
               float* Sigma, float* Vt, void* workspace, size_t workspace_bytes, void* stream) {
    return lrqmm_rsvd_ex(X, cols, amax, rows, cols, axis, bits, round_mode, rank, oversample, power_iters, seed,
                         omega_or_null, LRQMM_DEFAULT_PREC, U, Sigma, Vt, workspace, workspace_bytes, stream);
}

int lrqmm_rsvd_ex(const float* X, int ldx, const float* amax, int rows, int cols, int axis, int bits, int round_mode,
                  int rank, int oversample, int power_iters, uint64_t seed, const float* omega_or_null, int precision,
                  float* U, float* Sigma, float* Vt, void* workspace, size_t workspace_bytes, void* stream) {
    LaunchList ops;
    int rc = rsvd_plan(ops, X, ldx, amax, rows, cols, axis, bits, round_mode, rank, oversample, power_iters, seed,
                       omega_or_null, U, Sigma, Vt, workspace, workspace_bytes, static_cast<hipStream_t>(stream),
                       precision);
    if (rc != LRQMM_OK) return rc;
    return run_interleaved(ops, LaunchList());
}

static int gemm_impl(int M, int N, int K, int bits, int rank, const int8_t* Aq, const float* amaxA,
                     const int8_t* BqT, const float* amaxB, const float* U, const float* Sig, const float* Vt,
                     const float* W, const float* Gam, const float* Zt, GemmOut out, int32_t* Cint_or_null,
                     void* workspace, size_t workspace_bytes, void* stream, int prof_slot,
                     hipEvent_t raw_sums_ready = nullptr, int planes = 3) {
    float* const C = out.C;
    if (M < 0 || N < 0 || K < 0 || rank < 0 || out.ldc < N) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || !output_ok(M, N)) return LRQMM_ERR_UNSUPPORTED;
    if (!bits_ok(bits)) return LRQMM_ERR_UNSUPPORTED;
    if (!k_fits_int32(K, bits)) return LRQMM_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return LRQMM_OK;
    if (rank > K || rank > M || rank > N) return LRQMM_ERR_INVALID_ARG;
    if (rank > LRQMM_MAX_SKETCH) return LRQMM_ERR_UNSUPPORTED;
    if (!C || !amaxA || !amaxB || (K > 0 && (!Aq || !BqT))) return LRQMM_ERR_INVALID_ARG;
    if (rank > 0 && (!U || !Sig || !Vt || !W || !Gam || !Zt)) return LRQMM_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return LRQMM_ERR_WORKSPACE;
    GemmWs w;
    Arena a(workspace);
    if (carve_gemm(a, M, N, K, rank, &w) > workspace_bytes) return LRQMM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (K == 0) {
        // An empty reduction: C_F = 0 (rank <= K leaves no compensation either), so only the update
        // D <- alpha * 0 + beta * D remains.  No operand is read and no GEMM kernel is launched.
        prof_mark(prof_slot, 7, st);
        const int r0 = launch_empty_product(M, N, out, Cint_or_null, st);
        for (int e = 8; e <= 10; ++e) prof_mark(prof_slot, e, st);
        return r0;
    }
    const QuantParams q = make_quant_params(bits, 0);
    int rc;
    int R2P = 0;
    const int RP = pad_to(rank, 16);
    LRQ_TRY(launch_panel_prep(M, N, K, rank, RP, q.qmaxf, amaxA, amaxB, W, Vt, w.lamA, w.sA, w.lamB, w.sB, w.Wp,
                              w.Vp, w.Wp3, w.Vp3, w.X, st));
    if (rank > 0) {
        R2P = pad_to(2 * rank, 8);
        // A~ W and (V^T B~)^T without their step vectors, split along K; one launch for both
        const PassPlan pa = plan_pass_n(M, K), pb = plan_pass_n(N, K);
        LRQ_TRY(launch_codes_mul_n2(Aq, M, w.Wp, w.Wp3, pa, w.partialA, BqT, N, w.Vp, w.Vp3, pb, w.partialB, K,
                                    pad_to(K, 64), RP, st, planes));
        LRQ_TRY(launch_build_panels(M, N, K, rank, RP, R2P, U, Sig, w.sA, w.partialA, pa.splits, w.sB,
                                    w.partialB, pb.splits, w.X, Gam, Zt, w.Lp, w.Rp, st));
    }
    if (raw_sums_ready) {
        // the integer product ran early on another stream and left its int32 sums in C
        if (hipStreamWaitEvent(st, raw_sums_ready, 0) != hipSuccess) return LRQMM_ERR_HIP;
        prof_mark(prof_slot, 7, st);
        rc = launch_rank_update(M, N, C, w.sA, w.sB, w.Lp, w.Rp, R2P, out.alpha, st);
        prof_mark(prof_slot, 8, st);
        return rc;
    }
    prof_mark(prof_slot, 7, st);
    rc = launch_int8_gemm(M, N, K, Aq, BqT, w.sA, w.sB, rank > 0 ? w.Lp : nullptr, rank > 0 ? w.Rp : nullptr,
                          R2P, out, Cint_or_null, st);
    prof_mark(prof_slot, 8, st);
    prof_mark(prof_slot, 9, st);
    prof_mark(prof_slot, 10, st);
    return rc;
}

int lrqmm_gemm(int M, int N, int K, int bits, int rank, const int8_t* Aq, const float* amaxA,
               const int8_t* BqT, const float* amaxB, const float* U, const float* Sig, const float* Vt,
               const float* W, const float* Gam, const float* Zt, float* C, int32_t* Cint_or_null,
               void* workspace, size_t workspace_bytes, void* stream) {
    return lrqmm_gemm_ex(M, N, K, bits, rank, Aq, amaxA, BqT, amaxB, U, Sig, Vt, W, Gam, Zt, 1.0f, 0.0f, C, N,
                         Cint_or_null, workspace, workspace_bytes, stream);
}

int lrqmm_gemm_ex(int M, int N, int K, int bits, int rank, const int8_t* Aq, const float* amaxA,
                  const int8_t* BqT, const float* amaxB, const float* U, const float* Sig, const float* Vt,
                  const float* W, const float* Gam, const float* Zt, float alpha, float beta, float* D, int ldd,
                  int32_t* Cint_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    const GemmOut out = {D, ldd, alpha, beta};
    return gemm_impl(M, N, K, bits, rank, Aq, amaxA, BqT, amaxB, U, Sig, Vt, W, Gam, Zt, out, Cint_or_null,
                     workspace, workspace_bytes, stream, -1);
}

int lrqmm_gemm_static(int M, int N, int K, int bits, int rank, const int8_t* Aq, const float* amaxA,
                      const int8_t* BqT, const float* amaxB, const float* U, const float* Sig, const float* Vt,
                      const float* W, const float* Gam, const float* Zt, float alpha, float beta, float* D, int ldd,
                      int32_t* Cint_or_null, void* stream) {
    if (M < 0 || N < 0 || K < 0 || rank < 0 || ldd < N) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || !output_ok(M, N)) return LRQMM_ERR_UNSUPPORTED;
    if (rank > LRQMM_MAX_SKETCH) return LRQMM_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return LRQMM_OK;
    Arena a(nullptr);
    if (carve_gemm(a, M, N, K, rank, nullptr) > (size_t)LRQMM_STATIC_SCRATCH_BYTES) return LRQMM_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != LRQMM_OK) return rc;
    const GemmOut out = {D, ldd, alpha, beta};
    return gemm_impl(M, N, K, bits, rank, Aq, amaxA, BqT, amaxB, U, Sig, Vt, W, Gam, Zt, out, Cint_or_null, ws,
                     LRQMM_STATIC_SCRATCH_BYTES, stream, -1);
}

int lrqmm_matmul(int M, int N, int K, int bits, int rank, int oversample, int power_iters, uint64_t seed,
                 int round_mode, const float* A, const float* B, float* C, void* workspace,
                 size_t workspace_bytes, void* stream) {
    return lrqmm_matmul_ex(M, N, K, bits, rank, oversample, power_iters, seed, round_mode, LRQMM_SCALE_VECTOR,
                           LRQMM_DEFAULT_PREC, A, K, B, N, 1.0f, 0.0f, C, N, workspace, workspace_bytes, stream);
}

int lrqmm_matmul_ex(int M, int N, int K, int bits, int rank, int oversample, int power_iters, uint64_t seed,
                    int round_mode, int scale_mode, int precision, const float* A, int lda, const float* B, int ldb,
                    float alpha, float beta, float* D, int ldd, void* workspace, size_t workspace_bytes, void* stream) {
    float* const C = D;
    if (M < 0 || N < 0 || K < 0 || rank < 0 || oversample < 0 || power_iters < 0) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || !output_ok(M, N)) return LRQMM_ERR_UNSUPPORTED;
    if (!precision_ok(precision)) return LRQMM_ERR_INVALID_ARG;
    if (lda < K || ldb < N || ldd < N) return LRQMM_ERR_INVALID_ARG;
    if (scale_mode != LRQMM_SCALE_VECTOR && scale_mode != LRQMM_SCALE_TENSOR) return LRQMM_ERR_INVALID_ARG;
    if (round_mode != LRQMM_ROUND_FLOOR && round_mode != LRQMM_ROUND_NEAREST) return LRQMM_ERR_INVALID_ARG;
    if (!bits_ok(bits)) return LRQMM_ERR_UNSUPPORTED;
    if (!k_fits_int32(K, bits)) return LRQMM_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return LRQMM_OK;
    if (rank > 0) {
        const int ell = rank + oversample;
        if (ell > M || ell > N || ell > K) return LRQMM_ERR_INVALID_ARG;
        if (ell > LRQMM_MAX_SKETCH) return LRQMM_ERR_UNSUPPORTED;
    }
    if (!C || (K > 0 && (!A || !B))) return LRQMM_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return LRQMM_ERR_WORKSPACE;
    MatmulWs w;
    Arena a(workspace);
    if (carve_matmul(a, M, N, K, rank, oversample, &w) > workspace_bytes) return LRQMM_ERR_WORKSPACE;
    hipStream_t pst = static_cast<hipStream_t>(stream);
    // Under stream capture the call may only enqueue kernels, event records and event waits: it cannot
    // create its streams and events, and timing events do not belong in a graph.
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(pst, &capture) != hipSuccess) return LRQMM_ERR_HIP;
    const bool capturing = capture != hipStreamCaptureStatusNone;
    if (capturing && g_prof.on) return LRQMM_ERR_UNSUPPORTED;
    // the two operands' quantization and factorization run on two streams; rank 0 stays on one stream
    Side* const side = (rank > 0 && K > 0) ? side_state(!capturing) : nullptr;
    if (rank > 0 && K > 0 && !side) return capturing ? LRQMM_ERR_UNSUPPORTED : LRQMM_ERR_HIP;
    const bool overlap = side != nullptr;
    const int slot = (g_prof.on && g_prof.ncalls < kProfMaxCalls) ? g_prof.ncalls++ : -1;
    // The chain of the larger operand (A when M >= N: both share K) stays on the caller's stream and starts at
    // once; the other takes the side stream and absorbs the latency of the fork event.  Measured against the
    // fixed assignment: 3 % of the step at M = 100352, N = 64, 1 % on squares.
    const bool a_on_caller = M >= N;
    hipStream_t sst = overlap ? side->stream : pst;
    hipStream_t ast = a_on_caller ? pst : sst;
    hipStream_t bst = a_on_caller ? sst : pst;
    // Early integer GEMM: with both factorizations in their single-workgroup SVD the GPU is
    // nearly idle, so the int8 product (which needs only the codes) runs there on a third
    // stream, leaves raw int32 sums in C, and the epilogue follows the panels as a kernel of
    // its own.  Used for problems on the large-tile kernel.
    // (the raw sums need D's memory: only when its old contents are not an input and it is dense)
    // Measured on both sides of the rule (4096^3): at l = 24 the SVD takes ~60 us, the product ~85 us -- it outlasts
    // the window, holds the CUs the panel kernels need, and the fused kernel after the panels is 3-5 % faster; at
    // l = 40 (SVD ~115 us) the early product wins by 3-5 %; at 16384^3, l = 80 by 10 % (the SVD and the panel
    // kernels run beside the product, and the update of wide panels has a faster kernel of its own).
    const bool early = overlap && rank_update_usable(M, N, C) && beta == 0.0f && ldd == N && rank + oversample >= 32;
    if (slot >= 0) g_prof.early[slot] = early;
    hipStream_t gst = early ? side->gemm_stream : pst;
    // the two sides are planned first and then issued alternately (see LaunchList)
    LaunchList opsA, opsB;
    size_t svdA = 0, svdB = 0;      // positions of the small-SVD launches in the two lists
    int rc;
    // With a factorization to follow, and for shapes that take the guard-free pass kernels, quantization is
    // split differently: the group maxima come first (one read of the operand), and the operand's second read
    // yields codes, step vectors and the sketch product Y = R.Omega in one launch (one full-size read fewer
    // per operand than quantizing and sketching separately).  The sketch is filled by the chain's first launch
    // (it depends on nothing).  Otherwise: quantize, then factor.
    const QuantParams qp = make_quant_params(bits, round_mode);
    const bool per_tensor = scale_mode == LRQMM_SCALE_TENSOR;
    const int LPm = pad_to(rank + oversample, 16);
    RsvdWs wa = {}, wb = {};
    if (rank > 0 && K > 0) {
        Arena ra(w.subA), rb(w.subB);
        if (carve_rsvd(ra, M, K, LRQMM_AXIS_ROW, LPm, rank, &wa) > w.subA_bytes) return LRQMM_ERR_WORKSPACE;
        if (carve_rsvd(rb, K, N, LRQMM_AXIS_COL, LPm, rank, &wb) > w.subB_bytes) return LRQMM_ERR_WORKSPACE;
    }
    // Short rows of A (an im2col'd convolution: K = 576) stay in registers: maxima, codes and Y from a single read.
    // (in every precision mode: this pass then runs in float32, which the reduced modes allow)
    const bool onepass_a = rank > 0 && K > 0 && !per_tensor && plan_pass_n(M, K).splits == 1 &&
                           quant_sketch_rows_usable(A, lda, M, K, LPm, w.Aq);
    const bool fuse_a = !onepass_a && rank > 0 && K > 0 && quant_sketch_fusable(A, lda, M, K, LPm, plan_pass_n(M, K), w.Aq);
    const bool fuse_b = rank > 0 && K > 0 && quant_sketch_fusable(B, ldb, K, N, LPm, plan_pass_n(K, N), w.BqT);
    opsA.push_back([=] { prof_mark(slot, 0, ast); return LRQMM_OK; });
    if (onepass_a) {
        opsA.push_back([=] { return launch_fill_sketch(seed, LRQMM_AXIS_ROW, K, rank + oversample, LPm, wa.Wc, ast); });
    } else if (fuse_a) {
        opsA.push_back([=] { return launch_fill_sketch(seed, LRQMM_AXIS_ROW, K, rank + oversample, LPm, wa.Wc, ast); });
        opsA.push_back([=] { return launch_absmax_rows(A, lda, M, K, qp, per_tensor, w.amaxA, ast); });
    } else if (K > 0) opsA.push_back([=] { return lrqmm_quantize_ex(A, lda, M, K, LRQMM_AXIS_ROW, bits, round_mode, scale_mode, w.Aq, w.amaxA, ast); });
    else opsA.push_back([=] { return launch_pad_copy(nullptr, M, 0, 1, w.amaxA, ast); });
    opsA.push_back([=] { prof_mark(slot, 1, ast); return LRQMM_OK; });
    if (rank > 0)
        LRQ_TRY(rsvd_plan(opsA, A, lda, w.amaxA, M, K, LRQMM_AXIS_ROW, bits, round_mode, rank, oversample, power_iters,
                          seed, nullptr, w.U, w.Sig, w.Vt, w.subA, w.subA_bytes, ast, precision, &svdA,
                          fuse_a || onepass_a, fuse_a || onepass_a ? w.Aq : nullptr, onepass_a ? w.amaxA : nullptr));
    opsA.push_back([=] { prof_mark(slot, 2, ast); return LRQMM_OK; });
    opsB.push_back([=] { prof_mark(slot, 3, bst); return LRQMM_OK; });
    // B's first kernel fills the sketch and clears the column maxima (they are formed with atomic maxima) in one
    // launch.
    const bool prep_b = rank > 0 && K > 0;
    if (prep_b) {
        opsB.push_back([=] {
            return launch_sketch_and_zero(seed, LRQMM_AXIS_COL, N, rank + oversample, LPm, wb.Wc,
                                          reinterpret_cast<uint32_t*>(w.amaxB), N, bst);
        });
        if (fuse_b)
            opsB.push_back([=] { return launch_absmax_cols(B, ldb, K, N, qp, per_tensor, w.amaxB, bst, true); });
        else    // the quantizing kernel leaves the step vectors: the factorization starts with its first pass at once
            opsB.push_back([=] {
                return launch_quantize_cols(B, ldb, K, N, qp, per_tensor, nullptr, w.BqT, w.amaxB, bst, true, wb.lam, wb.s);
            });
    } else if (K > 0) opsB.push_back([=] { return lrqmm_quantize_ex(B, ldb, K, N, LRQMM_AXIS_COL, bits, round_mode, scale_mode, w.BqT, w.amaxB, bst); });
    else opsB.push_back([=] { return launch_pad_copy(nullptr, N, 0, 1, w.amaxB, bst); });
    opsB.push_back([=] { prof_mark(slot, 4, bst); return LRQMM_OK; });
    if (rank > 0)
        LRQ_TRY(rsvd_plan(opsB, B, ldb, w.amaxB, K, N, LRQMM_AXIS_COL, bits, round_mode, rank, oversample, power_iters,
                          seed, nullptr, w.W, w.Gam, w.Zt, w.subB, w.subB_bytes, bst, precision, &svdB, prep_b,
                          fuse_b ? w.BqT : nullptr));
    opsB.push_back([=] { prof_mark(slot, 5, bst); return LRQMM_OK; });

    // Nothing has been enqueued so far.  From the fork on, every path -- errors included -- joins the
    // library's streams back into the caller's, so that a capture is never left with an open branch
    // and a later call never meets work of a failed one.
    bool forked = false, gemm_forked = false;
    auto issue = [&]() -> int {
        int rc;
        if (overlap) {
            if (hipEventRecord(side->fork, pst) != hipSuccess) return LRQMM_ERR_HIP;
            forked = true;
            if (hipStreamWaitEvent(sst, side->fork, 0) != hipSuccess) return LRQMM_ERR_HIP;
        }
        // the chain on the caller's stream is issued first
        const LaunchList &ops1 = a_on_caller ? opsA : opsB, &ops2 = a_on_caller ? opsB : opsA;
        const size_t svd1 = a_on_caller ? svdA : svdB, svd2 = a_on_caller ? svdB : svdA;
        if (!early) return run_interleaved(ops1, ops2);
        // everything that precedes the two small SVDs
        LRQ_TRY(run_interleaved(ops1, 0, svd1, ops2, 0, svd2));
        // Both gates are recorded here, in this call, before anything waits on them: the integer
        // product needs both operands' codes, and starting it behind the kernels that precede both
        // SVDs keeps it out of the passes' way.
        if (hipEventRecord(side->gate_b, bst) != hipSuccess) return LRQMM_ERR_HIP;
        if (hipEventRecord(side->gate, ast) != hipSuccess) return LRQMM_ERR_HIP;
        LRQ_TRY(ops1[svd1]());
        LRQ_TRY(ops2[svd2]());
        gemm_forked = true;
        for (hipEvent_t e : {side->gate, side->gate_b})
            if (hipStreamWaitEvent(gst, e, 0) != hipSuccess) return LRQMM_ERR_HIP;
        // The product must not take the CUs before the two SVD workgroups have theirs: a few minimal
        // kernels give the SVD launches (one dependent launch behind their events) a head start.  The
        // two SVD workgroups hold a CU each while the product runs.
        const int resident = side->cus - 2;
        for (int t = 0; t < 3; ++t) LRQ_TRY(launch_tick(w.tick, gst));
        prof_mark(slot, 9, gst);
        rc = launch_int8_gemm_sums(M, N, K, w.Aq, w.BqT, reinterpret_cast<int32_t*>(C), resident, w.parts, gst);
        prof_mark(slot, 10, gst);
        if (rc != LRQMM_OK) return rc;
        LRQ_TRY(launch_int8_gemm_sums_finish(M, N, K, w.Aq, w.BqT, reinterpret_cast<int32_t*>(C), resident, w.parts, gst));
        if (hipEventRecord(side->gdone, gst) != hipSuccess) return LRQMM_ERR_HIP;
        return run_interleaved(ops1, svd1 + 1, ops1.size(), ops2, svd2 + 1, ops2.size());
    };
    rc = issue();
    if (forked) {
        if (hipEventRecord(side->join, sst) != hipSuccess || hipStreamWaitEvent(pst, side->join, 0) != hipSuccess)
            rc = rc != LRQMM_OK ? rc : LRQMM_ERR_HIP;
    }
    if (rc == LRQMM_OK) {
        prof_mark(slot, 6, pst);
        rc = gemm_impl(M, N, K, bits, rank, w.Aq, w.amaxA, w.BqT, w.amaxB, w.U, w.Sig, w.Vt, w.W, w.Gam, w.Zt,
                       GemmOut{D, ldd, alpha, beta}, nullptr, w.sub, w.sub_bytes, stream, slot,
                       early ? side->gdone : nullptr, planes_values(precision));
    }
    if (rc != LRQMM_OK && gemm_forked) {
        // failed somewhere behind the fork of the third stream: join it too (a second record of the
        // event after a successful first one is harmless)
        (void)hipEventRecord(side->gdone, gst);
        (void)hipStreamWaitEvent(pst, side->gdone, 0);
    }
    return rc;
}

namespace {
struct ResidualWs {
    int8_t *Aq, *RAq, *BqT, *RBqT;
    float *amaxA, *amaxRA, *amaxB, *amaxRB;
    void* sub;
    size_t sub_bytes;
};
size_t carve_residual(Arena& a, int M, int N, int K, ResidualWs* w) {
    ResidualWs t = {};
    t.Aq = a.take<int8_t>((size_t)M * K);
    t.RAq = a.take<int8_t>((size_t)M * K);
    t.BqT = a.take<int8_t>((size_t)N * K);
    t.RBqT = a.take<int8_t>((size_t)N * K);
    t.amaxA = a.take<float>(M);
    t.amaxRA = a.take<float>(M);
    t.amaxB = a.take<float>(N);
    t.amaxRB = a.take<float>(N);
    a.off = align_up(a.off, 256);
    Arena g(nullptr);
    t.sub_bytes = carve_gemm(g, M, N, K, 0, nullptr);
    t.sub = a.base ? a.base + a.off : nullptr;
    a.off += t.sub_bytes;
    if (w) *w = t;
    return a.off;
}
}  // namespace

size_t lrqmm_residual_workspace_bytes(int M, int N, int K) {
    if (M < 0 || N < 0 || K < 0 || !dims_ok(M, N, K) || !output_ok(M, N)) return 0;
    Arena a(nullptr);
    return carve_residual(a, M, N, K, nullptr) + 256;
}

int lrqmm_residual_matmul(int M, int N, int K, int bits, int terms, int round_mode, int scale_mode, const float* A,
                          int lda, const float* B, int ldb, float alpha, float beta, float* D, int ldd,
                          void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || N < 0 || K < 0 || lda < K || ldb < N || ldd < N) return LRQMM_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || !output_ok(M, N)) return LRQMM_ERR_UNSUPPORTED;
    if (terms != 1 && terms != 3 && terms != 4) return LRQMM_ERR_INVALID_ARG;
    if (round_mode != LRQMM_ROUND_FLOOR && round_mode != LRQMM_ROUND_NEAREST) return LRQMM_ERR_INVALID_ARG;
    if (scale_mode != LRQMM_SCALE_VECTOR && scale_mode != LRQMM_SCALE_TENSOR) return LRQMM_ERR_INVALID_ARG;
    if (!bits_ok(bits)) return LRQMM_ERR_UNSUPPORTED;
    if (!k_fits_int32(K, bits)) return LRQMM_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return LRQMM_OK;
    if (!D || (K > 0 && (!A || !B))) return LRQMM_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return LRQMM_ERR_WORKSPACE;
    ResidualWs w;
    Arena a(workspace);
    if (carve_residual(a, M, N, K, &w) > workspace_bytes) return LRQMM_ERR_WORKSPACE;
    if (K == 0) terms = 1;
    int rc;
    if (K > 0) {
        LRQ_TRY(lrqmm_quantize_ex(A, lda, M, K, LRQMM_AXIS_ROW, bits, round_mode, scale_mode, w.Aq, w.amaxA, stream));
        LRQ_TRY(lrqmm_quantize_ex(B, ldb, K, N, LRQMM_AXIS_COL, bits, round_mode, scale_mode, w.BqT, w.amaxB, stream));
        if (terms >= 3) {
            LRQ_TRY(lrqmm_quantize_residual(A, lda, w.amaxA, M, K, LRQMM_AXIS_ROW, bits, round_mode, scale_mode, w.RAq,
                                            w.amaxRA, stream));
            LRQ_TRY(lrqmm_quantize_residual(B, ldb, w.amaxB, K, N, LRQMM_AXIS_COL, bits, round_mode, scale_mode, w.RBqT,
                                            w.amaxRB, stream));
        }
    } else {
        LRQ_TRY(launch_pad_copy(nullptr, M, 0, 1, w.amaxA, static_cast<hipStream_t>(stream)));
        LRQ_TRY(launch_pad_copy(nullptr, N, 0, 1, w.amaxB, static_cast<hipStream_t>(stream)));
    }
    // one integer GEMM per term of Eq. (gemm_r_split), each dequantized with the scales of its two
    // operands and accumulated into D through the GEMM's own alpha/beta update
    auto term = [&](const int8_t* Lq, const float* amaxL, const int8_t* RqT, const float* amaxR, float b) {
        return gemm_impl(M, N, K, bits, 0, Lq, amaxL, RqT, amaxR, nullptr, nullptr, nullptr, nullptr, nullptr,
                         nullptr, GemmOut{D, ldd, alpha, b}, nullptr, w.sub, w.sub_bytes, stream, -1);
    };
    LRQ_TRY(term(w.Aq, w.amaxA, w.BqT, w.amaxB, beta));
    if (terms >= 3) {
        // alpha * term is added to what D holds now: beta = 1 from here on
        LRQ_TRY(term(w.Aq, w.amaxA, w.RBqT, w.amaxRB, 1.0f));
        LRQ_TRY(term(w.RAq, w.amaxRA, w.BqT, w.amaxB, 1.0f));
    }
    if (terms == 4) LRQ_TRY(term(w.RAq, w.amaxRA, w.RBqT, w.amaxRB, 1.0f));
    return LRQMM_OK;
}

int lrqmm_profile_enable(int on) {
    if (on && !g_prof.created) {
        for (int c = 0; c < kProfMaxCalls; ++c)
            for (int i = 0; i < kProfEvents; ++i)
                if (hipEventCreate(&g_prof.ev[c][i]) != hipSuccess) return LRQMM_ERR_HIP;
        g_prof.created = true;
    }
    g_prof.on = on != 0;
    g_prof.gemm_only = on == LRQMM_PROF_GEMM_ONLY;
    g_prof.ncalls = 0;
    return LRQMM_OK;
}

int lrqmm_profile_read(float* stage_ms, int* ncalls) {
    if (!stage_ms || !ncalls) return LRQMM_ERR_INVALID_ARG;
    const int n = g_prof.ncalls;
    *ncalls = n;
    for (int i = 0; i < kProfStages; ++i) stage_ms[i] = 0.f;
    if (n == 0) return LRQMM_OK;
    if (g_prof.gemm_only) {
        // the caller has synchronized the stream of the calls (see the header); each call
        // contributes its GEMM to stage 6 (early product) or 5 (fused kernel)
        for (int c = 0; c < n; ++c) {
            const int b = g_prof.early[c] ? 9 : 7, stage = g_prof.early[c] ? 6 : 5;
            float ms = 0.f;
            if (hipEventSynchronize(g_prof.ev[c][b + 1]) != hipSuccess) return LRQMM_ERR_HIP;
            if (hipEventElapsedTime(&ms, g_prof.ev[c][b], g_prof.ev[c][b + 1]) != hipSuccess) return LRQMM_ERR_HIP;
            stage_ms[stage] += ms / (float)n;
        }
        g_prof.ncalls = 0;
        return LRQMM_OK;
    }
    if (hipEventSynchronize(g_prof.ev[n - 1][kLastMainEvent]) != hipSuccess) return LRQMM_ERR_HIP;
    for (int c = 0; c < n; ++c)
        for (int i = 0; i < kProfStages; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, g_prof.ev[c][kStageBegin[i]], g_prof.ev[c][kStageEnd[i]]) != hipSuccess)
                return LRQMM_ERR_HIP;
            stage_ms[i] += ms / (float)n;
        }
    g_prof.ncalls = 0;
    return LRQMM_OK;
}

}  // extern "C"
