// Entry points of libqnn: argument validation, engine choice and the multi-launch compositions (Alg. 4 forward).
// Every step of the path runs in the kernels of this library; nothing here computes on the host except the
// BatchNorm fold, which is host-only by definition.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "qnn_internal.h"

// Scratch memory of qnn_binary_mlp_forward_static, the entry point for callers that cannot allocate: every GPU the
// library runs on holds its own copy of this array until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress; kernels receive the looked-up device address as an ordinary argument.
static constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace qnn {

static thread_local char g_err[512] = "";
static thread_local int g_last_engine = 0;
// engines of the multiply launches of the calling thread's last entry-point call, in launch order
static thread_local int g_engines[2 * QNN_MAX_LAYERS];
static thread_local int g_engine_count = 0;

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(QNN_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return QNN_OK;
}

namespace {

bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

int64_t sum_abs(const int32_t *c, int n) {
    int64_t s = 0;
    for (int i = 0; i < n; ++i) s += c[i] < 0 ? -(int64_t)c[i] : (int64_t)c[i];
    return s;
}

int check_planes(const char *who, int P, const int32_t *coef, int mode) {
    if (P < 1 || P > QNN_MAX_PLANES) return fail(QNN_ERR_SHAPE, "%s: plane count %d not in 1..%d", who, P, QNN_MAX_PLANES);
    if (!coef) return fail(QNN_ERR_NULL, "%s: coefficient array is NULL", who);
    if (mode != QNN_PLANE_BIT && mode != QNN_PLANE_SIGN) return fail(QNN_ERR_SHAPE, "%s: unknown plane mode %d", who, mode);
    return QNN_OK;
}

int check_engine(int engine) {
    if (engine < QNN_ENGINE_AUTO || engine > QNN_ENGINE_MFMA_LDS)
        return fail(QNN_ERR_SHAPE, "unknown engine %d", engine);
    return QNN_OK;
}

int check_range(const GemmArgs &g) {
    const int64_t sa = sum_abs(g.pa.coef, g.pa.count), sw = sum_abs(g.pw.coef, g.pw.count);
    // |C| <= sa * sw * K must stay below 2^31
    const long double bound = (long double)sa * (long double)sw * (long double)g.K;
    if (bound >= 2147483648.0L)
        return fail(QNN_ERR_OVERFLOW, "sum|coefA| * sum|coefW| * K = %.0Lf does not fit int32", bound);
    return QNN_OK;
}

// Which engine runs the product: QNN_OK and `chosen`, or QNN_ERR_UNSUPPORTED when the requested engine cannot take it.
int resolve_engine(const GemmArgs &g, int engine, int &chosen) {
    chosen = engine;
    if (engine == QNN_ENGINE_MFMA_FP4 && !mfma_supports(g, true))
        return fail(QNN_ERR_UNSUPPORTED, "FP4 matrix-core engine takes single-plane operands of supported shapes only");
    if (engine == QNN_ENGINE_MFMA && !mfma_supports(g))
        return fail(QNN_ERR_UNSUPPORTED, "matrix-core engine cannot take these arguments");
    if (engine == QNN_ENGINE_MFMA_LDS && !stage_supports(g))
        return fail(QNN_ERR_UNSUPPORTED, "LDS-staged matrix-core kernel cannot take these arguments");
    if (engine == QNN_ENGINE_AUTO) {
        // several planes: merged once per workgroup in LDS (measured 1.3 to 2.5 times faster than per-wave expansion)
        if (mfma_preferred(g) && (g.pa.count > 2 || g.pw.count > 1 || (g.pa.count == 2 && g.A.rows_are_pixels)) &&
            stage_supports(g))
            chosen = QNN_ENGINE_MFMA_LDS;
        else if (mfma_preferred(g) && mfma_supports(g, true))
            chosen = QNN_ENGINE_MFMA_FP4;
        else if (mfma_preferred(g) && mfma_supports(g))
            chosen = QNN_ENGINE_MFMA;
        else
            chosen = QNN_ENGINE_VALU;
    }
    if (chosen == QNN_ENGINE_VALU && !valu_supports(g)) {
        // the vector-ALU engine takes everything except a byte-coded left operand
        if (engine == QNN_ENGINE_AUTO && mfma_supports(g))
            chosen = QNN_ENGINE_MFMA;
        else
            return fail(QNN_ERR_UNSUPPORTED, "vector-ALU engine cannot take these arguments");
    }
    return QNN_OK;
}

int launch_on(const GemmArgs &g, int chosen, hipStream_t s) {
    int rc;
    if (chosen == QNN_ENGINE_VALU)
        rc = launch_gemm_valu(g, s);
    else if (chosen == QNN_ENGINE_MFMA_LDS)
        rc = launch_gemm_stage(g, s);
    else
        rc = launch_gemm_mfma(g, s, chosen == QNN_ENGINE_MFMA_FP4);
    if (rc == QNN_OK) {
        g_last_engine = chosen;
        if (g_engine_count < 2 * QNN_MAX_LAYERS) g_engines[g_engine_count++] = chosen;
    }
    return rc;
}

int dispatch(const GemmArgs &g, int engine, hipStream_t s) {
    int chosen;
    g_engine_count = 0;
    if (int rc = resolve_engine(g, engine, chosen)) return rc;
    return launch_on(g, chosen, s);
}

// Shared validation of the matrix-shaped products; fills `g`.  `empty` = a successful no-op (M == 0 or N == 0).
int gemm_args(const char *who, const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda, int64_t strideA,
              const uint32_t *W, int Pb, const int32_t *coefW, int modeW, int64_t ldw, int64_t strideW,
              const Epilogue &epi, int64_t M, int64_t N, int64_t K, int engine, GemmArgs &g, bool &empty) {
    empty = false;
    if (int rc = check_engine(engine)) return rc;
    if (M < 0 || N < 0) return fail(QNN_ERR_SHAPE, "%s: negative M or N", who);
    if (K < 1 || K > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "%s: K = %lld out of range", who, (long long)K);
    if (int rc = check_planes(who, Pa, coefA, modeA)) return rc;
    if (int rc = check_planes(who, Pb, coefW, modeW)) return rc;
    const int64_t Kw = words_for(K);
    if (lda < Kw || ldw < Kw) return fail(QNN_ERR_SHAPE, "%s: leading dimension below ceil(K/32) = %lld", who, (long long)Kw);
    if (Pa > 1 && strideA < 0) return fail(QNN_ERR_SHAPE, "%s: negative plane stride", who);
    if (Pb > 1 && strideW < 0) return fail(QNN_ERR_SHAPE, "%s: negative plane stride", who);
    if (epi.T || epi.out_bits) {
        if (epi.ldo < words_for(N)) return fail(QNN_ERR_SHAPE, "%s: ldo_words below ceil(N/32)", who);
    } else {
        if (epi.ldc < N) return fail(QNN_ERR_SHAPE, "%s: ldc below N", who);
    }
    if (M == 0 || N == 0) {
        empty = true;
        return QNN_OK;
    }
    if (!A || !W) return fail(QNN_ERR_NULL, "%s: operand pointer is NULL", who);
    if (epi.out_bits && !epi.T) return fail(QNN_ERR_NULL, "%s: threshold pointer is NULL", who);
    if (epi.T ? !epi.out_bits : !epi.C) return fail(QNN_ERR_NULL, "%s: output pointer is NULL", who);
    if (!aligned4(A) || !aligned4(W) || !aligned4(epi.C) || !aligned4(epi.out_bits) || !aligned4(epi.T))
        return fail(QNN_ERR_ALIGN, "%s: pointer not 4-byte aligned", who);
    std::memset(&g, 0, sizeof(g));
    g.A.base = A;
    g.A.ld = lda;
    g.A.plane_stride = strideA;
    g.pa.count = Pa;
    g.pa.mode = modeA;
    for (int i = 0; i < Pa; ++i) g.pa.coef[i] = coefA[i];
    g.W = W;
    g.ldw = ldw;
    g.strideW = strideW;
    g.pw.count = Pb;
    g.pw.mode = modeW;
    for (int i = 0; i < Pb; ++i) g.pw.coef[i] = coefW[i];
    g.epi = epi;
    g.M = M;
    g.N = N;
    g.K = K;
    g.Kw = Kw;
    return check_range(g);
}

int gemm_common(const char *who, const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda,
                int64_t strideA, const uint32_t *W, int Pb, const int32_t *coefW, int modeW, int64_t ldw,
                int64_t strideW, const Epilogue &epi, int64_t M, int64_t N, int64_t K, int engine, void *stream) {
    GemmArgs g;
    bool empty;
    if (int rc = gemm_args(who, A, Pa, coefA, modeA, lda, strideA, W, Pb, coefW, modeW, ldw, strideW, epi, M, N, K, engine,
                           g, empty))
        return rc;
    if (empty) return QNN_OK;
    return dispatch(g, engine, static_cast<hipStream_t>(stream));
}

const int32_t kOne[1] = {1};

}  // namespace
}  // namespace qnn

using namespace qnn;

extern "C" {

int qnn_pack_sign(const float *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *out, int64_t ldo_words,
                  void *stream) {
    if (rows < 0 || K < 1) return fail(QNN_ERR_SHAPE, "pack_sign: rows = %lld, K = %lld", (long long)rows, (long long)K);
    if (ldx < K || ldo_words < words_for(K)) return fail(QNN_ERR_SHAPE, "pack_sign: leading dimension too small");
    if (rows == 0) return QNN_OK;
    if (!x || !out) return fail(QNN_ERR_NULL, "pack_sign: NULL pointer");
    if (!aligned4(x) || !aligned4(out)) return fail(QNN_ERR_ALIGN, "pack_sign: pointer not 4-byte aligned");
    return launch_pack_sign(x, rows, K, ldx, out, ldo_words, static_cast<hipStream_t>(stream));
}

int qnn_pack_bitplanes(const uint8_t *v, int64_t rows, int64_t K, int64_t ldv, int nbits, uint32_t *planes,
                       int64_t ld_words, int64_t plane_stride_words, void *stream) {
    if (rows < 0 || K < 1) return fail(QNN_ERR_SHAPE, "pack_bitplanes: rows = %lld, K = %lld", (long long)rows, (long long)K);
    if (nbits < 1 || nbits > 8) return fail(QNN_ERR_SHAPE, "pack_bitplanes: nbits = %d not in 1..8", nbits);
    if (ldv < K || ld_words < words_for(K)) return fail(QNN_ERR_SHAPE, "pack_bitplanes: leading dimension too small");
    if (nbits > 1 && plane_stride_words < 0) return fail(QNN_ERR_SHAPE, "pack_bitplanes: negative plane stride");
    if (rows == 0) return QNN_OK;
    if (!v || !planes) return fail(QNN_ERR_NULL, "pack_bitplanes: NULL pointer");
    if (!aligned4(planes)) return fail(QNN_ERR_ALIGN, "pack_bitplanes: output not 4-byte aligned");
    return launch_pack_bitplanes(v, rows, K, ldv, nbits, planes, ld_words, plane_stride_words,
                                 static_cast<hipStream_t>(stream));
}

int qnn_binary_gemm_ex(const uint32_t *A, int64_t lda_words, const uint32_t *W, int64_t ldw_words, int32_t *C,
                       int64_t ldc, int64_t M, int64_t N, int64_t K, int engine, void *stream) {
    Epilogue e{C, ldc, nullptr, nullptr, nullptr, 0};
    return gemm_common("binary_gemm", A, 1, kOne, QNN_PLANE_SIGN, lda_words, 0, W, 1, kOne, QNN_PLANE_SIGN, ldw_words,
                       0, e, M, N, K, engine, stream);
}

int qnn_binary_gemm(const uint32_t *A, int64_t lda_words, const uint32_t *W, int64_t ldw_words, int32_t *C,
                    int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream) {
    return qnn_binary_gemm_ex(A, lda_words, W, ldw_words, C, ldc, M, N, K, QNN_ENGINE_AUTO, stream);
}

int qnn_binary_gemm_sign(const uint32_t *A, int64_t lda_words, const uint32_t *W, int64_t ldw_words,
                         const int32_t *T, const uint8_t *flip, uint32_t *out, int64_t ldo_words, int64_t M,
                         int64_t N, int64_t K, int engine, void *stream) {
    if (!T && M > 0 && N > 0) return fail(QNN_ERR_NULL, "binary_gemm_sign: threshold pointer is NULL");
    Epilogue e{nullptr, 0, T, flip, out, ldo_words};
    return gemm_common("binary_gemm_sign", A, 1, kOne, QNN_PLANE_SIGN, lda_words, 0, W, 1, kOne, QNN_PLANE_SIGN,
                       ldw_words, 0, e, M, N, K, engine, stream);
}

int qnn_bitplane_gemm_ex(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda_words,
                         int64_t strideA_words, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
                         int64_t ldw_words, int64_t strideW_words, int32_t *C, int64_t ldc, int64_t M, int64_t N,
                         int64_t K, int engine, void *stream) {
    Epilogue e{C, ldc, nullptr, nullptr, nullptr, 0};
    return gemm_common("bitplane_gemm", A, Pa, coefA, modeA, lda_words, strideA_words, W, Pb, coefW, modeW, ldw_words,
                       strideW_words, e, M, N, K, engine, stream);
}

int qnn_bitplane_gemm(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda_words,
                      int64_t strideA_words, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
                      int64_t ldw_words, int64_t strideW_words, int32_t *C, int64_t ldc, int64_t M, int64_t N,
                      int64_t K, void *stream) {
    return qnn_bitplane_gemm_ex(A, Pa, coefA, modeA, lda_words, strideA_words, W, Pb, coefW, modeW, ldw_words,
                                strideW_words, C, ldc, M, N, K, QNN_ENGINE_AUTO, stream);
}

int qnn_bitplane_gemm_sign(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda_words,
                           int64_t strideA_words, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
                           int64_t ldw_words, int64_t strideW_words, const int32_t *T, const uint8_t *flip,
                           uint32_t *out, int64_t ldo_words, int64_t M, int64_t N, int64_t K, int engine,
                           void *stream) {
    if (!T && M > 0 && N > 0) return fail(QNN_ERR_NULL, "bitplane_gemm_sign: threshold pointer is NULL");
    Epilogue e{nullptr, 0, T, flip, out, ldo_words};
    return gemm_common("bitplane_gemm_sign", A, Pa, coefA, modeA, lda_words, strideA_words, W, Pb, coefW, modeW,
                       ldw_words, strideW_words, e, M, N, K, engine, stream);
}

int qnn_threshold_sign(const int32_t *C, int64_t ldc, int64_t M, int64_t N, const int32_t *T, const uint8_t *flip,
                       uint32_t *out, int64_t ldo_words, void *stream) {
    if (M < 0 || N < 0) return fail(QNN_ERR_SHAPE, "threshold_sign: negative M or N");
    if (ldc < N || ldo_words < words_for(N)) return fail(QNN_ERR_SHAPE, "threshold_sign: leading dimension too small");
    if (M == 0 || N == 0) return QNN_OK;
    if (!C || !T || !out) return fail(QNN_ERR_NULL, "threshold_sign: NULL pointer");
    if (!aligned4(C) || !aligned4(T) || !aligned4(out)) return fail(QNN_ERR_ALIGN, "threshold_sign: pointer not 4-byte aligned");
    return launch_threshold_sign(C, ldc, M, N, T, flip, out, ldo_words, static_cast<hipStream_t>(stream));
}

int qnn_fold_batchnorm(const double *gamma, const double *beta, const double *mean, const double *var, double eps,
                       int64_t n, int32_t *T, uint8_t *flip) {
    if (n < 0) return fail(QNN_ERR_SHAPE, "fold_batchnorm: negative n");
    if (n == 0) return QNN_OK;
    if (!gamma || !beta || !mean || !var || !T || !flip) return fail(QNN_ERR_NULL, "fold_batchnorm: NULL pointer");
    for (int64_t i = 0; i < n; ++i) {
        if (!(var[i] + eps > 0.0)) return fail(QNN_ERR_SHAPE, "fold_batchnorm: var + eps <= 0 at %lld", (long long)i);
        if (gamma[i] == 0.0 || std::isnan(gamma[i])) {
            // y = beta for every s: constant sign
            T[i] = INT32_MIN;
            flip[i] = (beta[i] >= 0.0) ? 0 : 1;
            continue;
        }
        // y >= 0  <=>  gamma * (s - mean) >= -beta * sd  <=>  s >= tau (gamma > 0)  or  s <= tau (gamma < 0)
        const double tau = mean[i] - beta[i] * std::sqrt(var[i] + eps) / gamma[i];
        double t;
        if (gamma[i] > 0.0) {
            t = std::ceil(tau);
            flip[i] = 0;
        } else {
            t = std::floor(tau) + 1.0;  // s <= floor(tau)  <=>  not (s >= floor(tau) + 1)
            flip[i] = 1;
        }
        if (std::isnan(t)) return fail(QNN_ERR_SHAPE, "fold_batchnorm: NaN threshold at %lld", (long long)i);
        // saturate: s >= INT32_MIN is always true; a threshold above INT32_MAX is never reached, and INT32_MAX
        // itself is unreachable for any sum the multiply calls accept (|C| < 2^31 - 1 is not guaranteed, so keep
        // exactness by only clamping values strictly outside the int32 range)
        if (t <= -2147483648.0)
            T[i] = INT32_MIN;
        else if (t > 2147483647.0) {
            // never true: encode as "always true" with the opposite flip
            T[i] = INT32_MIN;
            flip[i] = flip[i] ? 0 : 1;
        } else
            T[i] = (int32_t)t;
    }
    return QNN_OK;
}

size_t qnn_binary_mlp_workspace_bytes(int64_t batch, int in_bits, int n_layers, const int64_t *dims) {
    if (batch < 0 || in_bits < 1 || in_bits > 8 || n_layers < 2 || n_layers > QNN_MAX_LAYERS || !dims) return 0;
    auto round256 = [](size_t b) { return (b + 255) & ~(size_t)255; };
    // rows padded to a multiple of 4 words so that every buffer takes the wide-load path
    auto ldw = [](int64_t d) { return (size_t)((words_for(d) + 3) & ~(int64_t)3); };
    size_t planes = round256((size_t)in_bits * (size_t)batch * ldw(dims[0]) * 4);
    size_t act = 0;
    for (int l = 1; l < n_layers; ++l) {
        size_t b = round256((size_t)batch * ldw(dims[l]) * 4);
        if (b > act) act = b;
    }
    return planes + 2 * act + 256;
}

// Alg. 4 as a list of launches, every one validated (pointers, ranges, engine) before the first is enqueued.
namespace {
struct MlpPlan {
    bool pack_planes;  // the input planes are materialised (otherwise the first layer reads the 8-bit codes)
    bool expand_w;     // the first layer's weights are expanded to bytes first (into the unused plane area)
    int8_t *w_bytes;
    int64_t ld_w_bytes;
    int32_t *rw_scaled;
    const uint8_t *x;
    int64_t batch, in_dim, ldx, ld0, plane_stride;
    int in_bits;
    uint32_t *planes;
    int n;
    GemmArgs g[QNN_MAX_LAYERS];
    int engine[QNN_MAX_LAYERS];
};

int64_t mlp_ldw(int64_t d) { return (words_for(d) + 3) & ~(int64_t)3; }
size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

int plan_mlp(const uint8_t *x, int64_t batch, int64_t ldx, int in_bits, int n_layers, const int64_t *dims,
             const uint32_t *const *W, const int32_t *const *T, const uint8_t *const *flip, int32_t *logits,
             int64_t ld_logits, void *workspace, size_t workspace_bytes, int engine, MlpPlan &plan, bool &empty) {
    empty = false;
    if (int rc = check_engine(engine)) return rc;
    if (batch < 0) return fail(QNN_ERR_SHAPE, "mlp: negative batch");
    if (in_bits < 1 || in_bits > 8) return fail(QNN_ERR_SHAPE, "mlp: in_bits = %d not in 1..8", in_bits);
    if (n_layers < 2 || n_layers > QNN_MAX_LAYERS) return fail(QNN_ERR_SHAPE, "mlp: n_layers = %d not in 2..%d", n_layers, QNN_MAX_LAYERS);
    if (!dims || !W || !T) return fail(QNN_ERR_NULL, "mlp: dims / W / T array is NULL");
    for (int l = 0; l <= n_layers; ++l)
        if (dims[l] < 1 || dims[l] > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "mlp: dims[%d] = %lld", l, (long long)dims[l]);
    if (ldx < dims[0] || ld_logits < dims[n_layers]) return fail(QNN_ERR_SHAPE, "mlp: leading dimension too small");
    if (batch == 0) {
        empty = true;
        return QNN_OK;
    }
    if (!x || !logits) return fail(QNN_ERR_NULL, "mlp: x or logits is NULL");
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l]) return fail(QNN_ERR_NULL, "mlp: W[%d] is NULL", l);
        if (l < n_layers - 1 && !T[l]) return fail(QNN_ERR_NULL, "mlp: T[%d] is NULL", l);
    }
    const size_t need = qnn_binary_mlp_workspace_bytes(batch, in_bits, n_layers, dims);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
        return fail(QNN_ERR_WORKSPACE, "mlp: workspace must be 256-byte aligned and hold %zu bytes", need);

    uint8_t *ws = static_cast<uint8_t *>(workspace);
    plan.x = x, plan.batch = batch, plan.in_dim = dims[0], plan.ldx = ldx, plan.in_bits = in_bits;
    plan.planes = reinterpret_cast<uint32_t *>(ws);
    plan.ld0 = mlp_ldw(dims[0]);
    plan.plane_stride = batch * plan.ld0;
    plan.n = n_layers;
    const size_t off = round256((size_t)in_bits * (size_t)plan.plane_stride * 4);
    size_t act_bytes = 0;
    for (int l = 1; l < n_layers; ++l) {
        const size_t b = round256((size_t)batch * (size_t)mlp_ldw(dims[l]) * 4);
        if (b > act_bytes) act_bytes = b;
    }
    uint32_t *act[2] = {reinterpret_cast<uint32_t *>(ws + off), reinterpret_cast<uint32_t *>(ws + off + act_bytes)};

    // `engine` is a preference: a layer that the requested engine cannot take runs on the library's choice.
    auto choose = [&](const GemmArgs &g, int &chosen) {
        int rc = resolve_engine(g, engine, chosen);
        if (rc == QNN_ERR_UNSUPPORTED && engine != QNN_ENGINE_AUTO) rc = resolve_engine(g, QNN_ENGINE_AUTO, chosen);
        return rc;
    };

    // Step 1 of Alg. 4: s = sum_n 2^(n-1) (x^n . W_1), then Sign(BatchNorm).  By Eq. (FirstLayer) that sum IS x . W_1
    // on the 8-bit codes, and the matrix-core engine can take the codes as they are (x - 128 is an int8 operand): no
    // planes are materialised then.  Otherwise: planes, then the weighted plane products.
    int32_t coef[QNN_MAX_PLANES];
    for (int p = 0; p < in_bits; ++p) coef[p] = 1 << p;
    const Epilogue e0{nullptr, 0, T[0], flip ? flip[0] : nullptr, act[0], mlp_ldw(dims[1])};
    plan.pack_planes = true;
    plan.expand_w = false;
    if (in_bits == 8 && engine != QNN_ENGINE_VALU) {
        GemmArgs &g = plan.g[0];
        std::memset(&g, 0, sizeof(g));
        g.A.base = reinterpret_cast<const uint32_t *>(x);
        g.A.ld = ldx;
        g.A.rows_are_bytes = 1;
        g.pa.count = 8, g.pa.mode = QNN_PLANE_BIT;
        for (int p = 0; p < 8; ++p) g.pa.coef[p] = coef[p];
        g.W = W[0];
        g.ldw = words_for(dims[0]);
        g.pw.count = 1, g.pw.mode = QNN_PLANE_SIGN, g.pw.coef[0] = 1;
        g.epi = e0;
        g.M = batch, g.N = dims[1], g.K = dims[0], g.Kw = words_for(dims[0]);
        if (int rc = check_range(g)) return rc;
        if (mfma_supports(g) && (engine != QNN_ENGINE_AUTO || mfma_preferred(g))) {
            if (!aligned4(W[0]) || !aligned4(T[0])) return fail(QNN_ERR_ALIGN, "mlp: pointer not 4-byte aligned");
            plan.engine[0] = QNN_ENGINE_MFMA;
            plan.pack_planes = false;
            // The plane area of the workspace is free then: if it holds them, the weights go there as bytes (rows of
            // whole 128-element groups) with their row sums, which lets the kernel run without expanding bits per wave.
            const int64_t ldb = (dims[0] + 127) / 128 * 128;
            const size_t wb = round256((size_t)dims[1] * (size_t)ldb), rb = round256((size_t)dims[1] * 4);
            if (wb + rb <= off) {
                plan.expand_w = true;
                plan.w_bytes = reinterpret_cast<int8_t *>(ws);
                plan.ld_w_bytes = ldb;
                plan.rw_scaled = reinterpret_cast<int32_t *>(ws + wb);
                g.w_bytes = plan.w_bytes, g.ld_w_bytes = ldb, g.rw_scaled = plan.rw_scaled;
            }
        }
    }
    bool none;
    if (plan.pack_planes) {
        if (!aligned4(plan.planes)) return fail(QNN_ERR_ALIGN, "mlp: workspace not 4-byte aligned");
        if (int rc = gemm_args("mlp layer 1", plan.planes, in_bits, coef, QNN_PLANE_BIT, plan.ld0, plan.plane_stride, W[0],
                               1, kOne, QNN_PLANE_SIGN, words_for(dims[0]), 0, e0, batch, dims[1], dims[0], engine,
                               plan.g[0], none))
            return rc;
        if (int rc = choose(plan.g[0], plan.engine[0])) return rc;
    }
    // step 2: hidden layers, product + threshold fused; step 3: output layer, integer sums
    int cur = 0;
    for (int l = 1; l < n_layers; ++l) {
        const bool last = l == n_layers - 1;
        const Epilogue e = last ? Epilogue{logits, ld_logits, nullptr, nullptr, nullptr, 0}
                                : Epilogue{nullptr, 0, T[l], flip ? flip[l] : nullptr, act[cur ^ 1], mlp_ldw(dims[l + 1])};
        if (int rc = gemm_args("mlp layer", act[cur], 1, kOne, QNN_PLANE_SIGN, mlp_ldw(dims[l]), 0, W[l], 1, kOne,
                               QNN_PLANE_SIGN, words_for(dims[l]), 0, e, batch, dims[l + 1], dims[l], engine, plan.g[l],
                               none))
            return rc;
        if (int rc = choose(plan.g[l], plan.engine[l])) return rc;
        cur ^= 1;
    }
    return QNN_OK;
}

int run_mlp(const MlpPlan &plan, hipStream_t s) {
    g_engine_count = 0;
    if (plan.pack_planes)
        if (int rc = launch_pack_bitplanes(plan.x, plan.batch, plan.in_dim, plan.ldx, plan.in_bits, plan.planes, plan.ld0,
                                           plan.plane_stride, s))
            return rc;
    if (plan.expand_w)
        if (int rc = bytes_panel::launch_expand_weights(plan.g[0].W, plan.g[0].N, plan.g[0].K, plan.g[0].ldw, plan.w_bytes,
                                                        plan.ld_w_bytes, plan.rw_scaled, s))
            return rc;
    for (int l = 0; l < plan.n; ++l)
        if (int rc = launch_on(plan.g[l], plan.engine[l], s)) return rc;
    return QNN_OK;
}

// Device memory of the entry point that must not allocate: one array per GPU, held until the process ends.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of the calling thread's current device's copy of `scratch` (looked up once per device).
int static_scratch(void *&ptr) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(QNN_ERR_HIP, "static scratch: no current device below %d", kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(QNN_ERR_HIP, "static scratch: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    ptr = g_scratch_ptr[dev];
    return QNN_OK;
}
}  // namespace

int qnn_binary_mlp_forward_ex(const uint8_t *x, int64_t batch, int64_t ldx, int in_bits, int n_layers,
                              const int64_t *dims, const uint32_t *const *W, const int32_t *const *T,
                              const uint8_t *const *flip, int32_t *logits, int64_t ld_logits, void *workspace,
                              size_t workspace_bytes, int engine, void *stream) {
    MlpPlan plan;
    bool empty;
    if (int rc = plan_mlp(x, batch, ldx, in_bits, n_layers, dims, W, T, flip, logits, ld_logits, workspace,
                          workspace_bytes, engine, plan, empty))
        return rc;
    if (empty) return QNN_OK;
    return run_mlp(plan, static_cast<hipStream_t>(stream));
}

int qnn_binary_mlp_forward(const uint8_t *x, int64_t batch, int64_t in_dim, int in_bits, int n_layers,
                           const int64_t *dims, const uint32_t *const *W, const int32_t *const *T,
                           const uint8_t *const *flip, int32_t *logits, int64_t ld_logits, void *workspace,
                           size_t workspace_bytes, void *stream) {
    if (dims && in_dim != dims[0]) return fail(QNN_ERR_SHAPE, "mlp: in_dim = %lld differs from dims[0]", (long long)in_dim);
    return qnn_binary_mlp_forward_ex(x, batch, in_dim, in_bits, n_layers, dims, W, T, flip, logits, ld_logits, workspace,
                                     workspace_bytes, QNN_ENGINE_AUTO, stream);
}

size_t qnn_static_scratch_bytes(void) { return kStaticScratchBytes; }

int qnn_binary_mlp_forward_static(const uint8_t *x, int64_t batch, int64_t in_dim, int in_bits, int n_layers,
                                  const int64_t *dims, const uint32_t *const *W, const int32_t *const *T,
                                  const uint8_t *const *flip, int32_t *logits, int64_t ld_logits, void *stream) {
    if (dims && in_dim != dims[0]) return fail(QNN_ERR_SHAPE, "mlp: in_dim = %lld differs from dims[0]", (long long)in_dim);
    const size_t need = qnn_binary_mlp_workspace_bytes(batch, in_bits, n_layers, dims);
    if (need > kStaticScratchBytes)
        return fail(QNN_ERR_WORKSPACE, "mlp (static scratch): this network and batch need %zu bytes of scratch, the "
                                       "built-in buffer holds %zu", need, kStaticScratchBytes);
    // arguments first (with a stand-in address that is never used), so that an argument error or an empty batch
    // does not depend on the device at all; then the real plan on this device's array
    MlpPlan plan;
    bool empty;
    if (int rc = plan_mlp(x, batch, in_dim, in_bits, n_layers, dims, W, T, flip, logits, ld_logits,
                          reinterpret_cast<void *>(uintptr_t(256)), kStaticScratchBytes, QNN_ENGINE_AUTO, plan, empty))
        return rc;
    if (empty) return QNN_OK;
    void *ws = nullptr;
    if (int rc = static_scratch(ws)) return rc;
    if (int rc = plan_mlp(x, batch, in_dim, in_bits, n_layers, dims, W, T, flip, logits, ld_logits, ws,
                          kStaticScratchBytes, QNN_ENGINE_AUTO, plan, empty))
        return rc;
    return run_mlp(plan, static_cast<hipStream_t>(stream));
}

namespace {
int conv_args(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words, int64_t B, int64_t H,
              int64_t Wd, int64_t Cin, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
              int64_t strideW_words, int64_t Cout, int KH, int KW, int pad, int stride_hw, const Epilogue &epi,
              int engine, GemmArgs &g, bool &empty) {
    empty = false;
    if (int rc = check_engine(engine)) return rc;
    if (B < 0 || Cout < 0) return fail(QNN_ERR_SHAPE, "conv2d: negative batch or Cout");
    if (H < 1 || Wd < 1 || Cin < 1 || KH < 1 || KW < 1 || pad < 0 || stride_hw < 1)
        return fail(QNN_ERR_SHAPE, "conv2d: bad geometry");
    if (H > 32767 || Wd > 32767 || KH > 255 || KW > 255 || Cin > (1 << 24) || pad > 32767 || stride_hw > 32767)
        return fail(QNN_ERR_SHAPE, "conv2d: geometry beyond supported range");
    if (H + 2 * (int64_t)pad < KH || Wd + 2 * (int64_t)pad < KW) return fail(QNN_ERR_SHAPE, "conv2d: kernel larger than padded image");
    if (int rc = check_planes("conv2d", Pa, coefA, modeA)) return rc;
    if (int rc = check_planes("conv2d", Pb, coefW, modeW)) return rc;
    if (modeA == QNN_PLANE_SIGN && pad > 0)
        return fail(QNN_ERR_UNSUPPORTED, "conv2d: zero padding cannot be encoded in a sign-mode activation plane");
    if (B == 0 || Cout == 0) {
        empty = true;
        return QNN_OK;
    }
    if (!A || !W) return fail(QNN_ERR_NULL, "conv2d: NULL pointer");
    if (epi.out_bits && !epi.T) return fail(QNN_ERR_NULL, "conv2d: threshold pointer is NULL");
    if (epi.T ? !epi.out_bits : !epi.C) return fail(QNN_ERR_NULL, "conv2d: output pointer is NULL");
    if (!aligned4(A) || !aligned4(W) || !aligned4(epi.C) || !aligned4(epi.out_bits) || !aligned4(epi.T))
        return fail(QNN_ERR_ALIGN, "conv2d: pointer not 4-byte aligned");
    const int64_t Ho = (H + 2 * (int64_t)pad - KH) / stride_hw + 1, Wo = (Wd + 2 * (int64_t)pad - KW) / stride_hw + 1;
    if (Ho < 1 || Wo < 1 || Ho > 0x7FFFFFFFLL || Wo > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "conv2d: output size out of range");
    const int64_t Cw = words_for(Cin);
    std::memset(&g, 0, sizeof(g));
    g.A.base = A;
    g.A.plane_stride = strideA_words;
    g.A.rows_are_pixels = 1;
    g.A.H = (int)H, g.A.Wd = (int)Wd, g.A.Ho = (int)Ho, g.A.Wo = (int)Wo, g.A.Cw = (int)Cw;
    g.A.KH = KH, g.A.KW = KW, g.A.pad = pad, g.A.stride = stride_hw;
    g.pa.count = Pa, g.pa.mode = modeA;
    for (int i = 0; i < Pa; ++i) g.pa.coef[i] = coefA[i];
    g.W = W;
    g.Kw = (int64_t)KH * KW * Cw;
    g.ldw = g.Kw;
    g.strideW = strideW_words;
    g.pw.count = Pb, g.pw.mode = modeW;
    for (int i = 0; i < Pb; ++i) g.pw.coef[i] = coefW[i];
    g.epi = epi;
    g.M = B * Ho * Wo;
    g.N = Cout;
    g.K = (int64_t)KH * KW * Cin;  // true number of connections per output (channel tail bits are zero)
    if (g.Kw > 0x7FFFFFFFLL / 32) return fail(QNN_ERR_SHAPE, "conv2d: patch too long");
    return check_range(g);
}
}  // namespace

int qnn_bitplane_conv2d_ex(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words,
                           int64_t B, int64_t H, int64_t Wd, int64_t Cin, const uint32_t *W, int Pb,
                           const int32_t *coefW, int modeW, int64_t strideW_words, int64_t Cout, int KH, int KW,
                           int pad, int stride_hw, int32_t *out, int engine, void *stream) {
    GemmArgs g;
    bool empty;
    const Epilogue e{out, Cout, nullptr, nullptr, nullptr, 0};
    if (int rc = conv_args(A, Pa, coefA, modeA, strideA_words, B, H, Wd, Cin, W, Pb, coefW, modeW, strideW_words, Cout,
                           KH, KW, pad, stride_hw, e, engine, g, empty))
        return rc;
    if (empty) return QNN_OK;
    return dispatch(g, engine, static_cast<hipStream_t>(stream));
}

int qnn_bitplane_conv2d_sign(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words,
                             int64_t B, int64_t H, int64_t Wd, int64_t Cin, const uint32_t *W, int Pb,
                             const int32_t *coefW, int modeW, int64_t strideW_words, int64_t Cout, int KH, int KW,
                             int pad, int stride_hw, const int32_t *T, const uint8_t *flip, uint32_t *out_bits,
                             int engine, void *stream) {
    if (!T && B > 0 && Cout > 0) return fail(QNN_ERR_NULL, "conv2d_sign: threshold pointer is NULL");
    GemmArgs g;
    bool empty;
    const Epilogue e{nullptr, 0, T, flip, out_bits, words_for(Cout)};
    if (int rc = conv_args(A, Pa, coefA, modeA, strideA_words, B, H, Wd, Cin, W, Pb, coefW, modeW, strideW_words, Cout,
                           KH, KW, pad, stride_hw, e, engine, g, empty))
        return rc;
    if (empty) return QNN_OK;
    return dispatch(g, engine, static_cast<hipStream_t>(stream));
}

int qnn_bitplane_conv2d(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words,
                        int64_t B, int64_t H, int64_t Wd, int64_t Cin, const uint32_t *W, int Pb,
                        const int32_t *coefW, int modeW, int64_t strideW_words, int64_t Cout, int KH, int KW,
                        int pad, int stride_hw, int32_t *out, void *stream) {
    return qnn_bitplane_conv2d_ex(A, Pa, coefA, modeA, strideA_words, B, H, Wd, Cin, W, Pb, coefW, modeW,
                                  strideW_words, Cout, KH, KW, pad, stride_hw, out, QNN_ENGINE_AUTO, stream);
}

// ---------------------------------------------------------------------------------------------------- ConvNet forward
// Alg. 4 for the binarized ConvNet of App. A: 3 x 3 "same" convolutions, some followed by 2 x 2 max-pooling, each
// followed by Sign(BatchNorm(.)); then fully connected layers.  Everything between the 8-bit input and the int32 logits
// stays packed.  A +-1 feature map that feeds a convolution is kept as the 2-bit two's-complement code of its values
// (plane 0 = "inside the image" = all ones, plane 1 = "value is -1"; +1 = 01, -1 = 11), because the zero padding of a
// "same" convolution must contribute exactly 0 and a single +-1 bit cannot say 0; the all-zero words that the
// convolution kernels read outside the image are then the code of 0.  The threshold epilogue writes plane 1 directly
// (the flip flags are inverted for those layers).  Max-pooling runs on the thresholded bits (see pool_bits_kernel).
namespace {
constexpr int kMaxNetLayers = 2 * QNN_MAX_LAYERS;
struct NetStep {
    enum Kind { kPack, kFlags, kOnes, kGemm, kPool, kFirstConv, kConvPrep, kConvPanel } kind;
    GemmArgs g;      // kGemm (convolution or fully connected)
    int engine;      // kGemm
    // kPack / kFlags / kOnes / kPool operands
    const void *src;
    void *dst, *dst2;
    int64_t rows, n;
    int a, b, c;
    const uint32_t *mask;
    bool invert;
};
struct NetPlan {
    int n;
    FlagJobs flags;     // kFlags: every layer's flip flags, one launch
    ConvPrepJobs prep;  // kConvPrep: border-class thresholds of every convolution on the panel-fed kernel, one launch
    NetStep step[6 * kMaxNetLayers + 4];
};

struct NetLayout {
    size_t planes0, flags, act[2], tmp, fc[2], total;
    size_t flag_bits[kMaxNetLayers], flag_inv[kMaxNetLayers];
    size_t class_thr[kMaxNetLayers], zero_line;  // scratch of the convolutions on the panel-fed kernel
};

// Sizes of the workspace regions; false if the shapes are not valid.
bool net_layout(int64_t B, int64_t H, int64_t Wd, int64_t C0, int in_bits, int n_conv, const int64_t *cout,
                const int32_t *pool, int n_fc, const int64_t *fc_out, NetLayout &L) {
    if (B < 0 || H < 1 || Wd < 1 || C0 < 1 || in_bits < 1 || in_bits > 8 || n_conv < 1 || n_fc < 1 ||
        n_conv + n_fc > kMaxNetLayers || !cout || !pool || !fc_out)
        return false;
    if (H > 32767 || Wd > 32767 || C0 > (1 << 24)) return false;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round256(bytes);
        return at;
    };
    L.planes0 = take((size_t)in_bits * (size_t)(B * H * Wd) * (size_t)words_for(C0) * 4);
    size_t act = 0, tmp = 0;
    int64_t h = H, w = Wd;
    for (int l = 0; l < n_conv; ++l) {
        if (cout[l] < 1 || cout[l] > (1 << 24)) return false;
        const size_t full = (size_t)(B * h * w) * (size_t)words_for(cout[l]) * 4;
        if (pool[l]) {
            if (full > tmp) tmp = full;
            h /= 2, w /= 2;
            if (h < 1 || w < 1) return false;
        }
        const size_t kept = 2 * (size_t)(B * h * w) * (size_t)words_for(cout[l]) * 4;  // two planes
        if (kept > act) act = kept;
    }
    L.act[0] = take(act);
    L.act[1] = take(act);
    L.tmp = take(tmp);
    size_t fc = 0;
    for (int j = 0; j < n_fc; ++j) {
        if (fc_out[j] < 1 || fc_out[j] > 0x7FFFFFFFLL) return false;
        const size_t b = (size_t)B * (size_t)mlp_ldw(fc_out[j]) * 4;
        if (j < n_fc - 1 && b > fc) fc = b;
    }
    L.fc[0] = take(fc);
    L.fc[1] = take(fc);
    L.flags = off;
    for (int l = 0; l < n_conv + n_fc - 1; ++l) {
        const int64_t n = l < n_conv ? cout[l] : fc_out[l - n_conv];
        L.flag_bits[l] = take((size_t)words_for(n) * 4);
        L.flag_inv[l] = take((size_t)n);
        L.class_thr[l] = l < n_conv ? take((size_t)16 * (size_t)conv_panel_class_ld(n) * 4) : 0;
    }
    L.zero_line = take(256);
    L.total = off + 256;
    return true;
}

int run_net(const NetPlan &plan, hipStream_t s) {
    g_engine_count = 0;
    for (int i = 0; i < plan.n; ++i) {
        const NetStep &st = plan.step[i];
        int rc = QNN_OK;
        switch (st.kind) {
            case NetStep::kPack:
                rc = launch_pack_bitplanes(static_cast<const uint8_t *>(st.src), st.rows, st.n, st.n, st.a,
                                           static_cast<uint32_t *>(st.dst), st.b, st.rows * st.b, s);
                break;
            case NetStep::kFlags:
                rc = launch_flags(plan.flags, s);
                break;
            case NetStep::kOnes:
                rc = launch_ones_plane(static_cast<uint32_t *>(st.dst), st.rows, st.a, st.b, s);
                break;
            case NetStep::kGemm:
                rc = launch_on(st.g, st.engine, s);
                break;
            case NetStep::kFirstConv:
                // src = image, mask = weights, dst = output bits; rows = B, a / b / c = H / W / C0, n = filters;
                // the thresholds and flips travel in g.epi
                rc = launch_conv_first(static_cast<const uint8_t *>(st.src), st.rows, st.a, st.b, st.c, st.mask, st.n, st.g.epi.T,
                                       st.g.epi.flip, static_cast<uint32_t *>(st.dst), static_cast<uint32_t *>(st.dst2), st.g.epi.ldo, s);
                if (rc == QNN_OK) {
                    g_last_engine = QNN_ENGINE_MFMA;
                    if (g_engine_count < 2 * QNN_MAX_LAYERS) g_engines[g_engine_count++] = QNN_ENGINE_MFMA;
                }
                break;
            case NetStep::kConvPrep: {  // with the layers' flip flags
                ConvPrepJobs jobs = plan.prep;
                rc = panel::launch_conv_class_thr(jobs, plan.flags, s);
                break;
            }
            case NetStep::kConvPanel:
                // src = plane "value is -1" of the input map, mask = weights, dst = output bits, dst2 = class thresholds;
                // rows = B, a / b / c = H / W / C, n = filters; thresholds, complemented flips and the output pitch in
                // g.epi; g.W = the line of zeros
                rc = launch_conv_panel(static_cast<const uint32_t *>(st.src), st.rows, st.a, st.b, st.c, st.mask, st.n, st.g.epi.T,
                                       st.g.epi.flip, static_cast<uint32_t *>(st.dst), st.g.epi.ldo, static_cast<const int32_t *>(st.dst2),
                                       st.g.W, s);
                if (rc == QNN_OK) {
                    g_last_engine = QNN_ENGINE_MFMA_FP4;
                    if (g_engine_count < 2 * QNN_MAX_LAYERS) g_engines[g_engine_count++] = QNN_ENGINE_MFMA_FP4;
                }
                break;
            case NetStep::kPool:
                rc = launch_pool_bits(static_cast<const uint32_t *>(st.src), st.rows, st.a, st.b, st.c, st.mask, st.invert,
                                      static_cast<uint32_t *>(st.dst), static_cast<uint32_t *>(st.dst2), (int)st.n, s);
                break;
        }
        if (rc) return rc;
    }
    return QNN_OK;
}
}  // namespace

size_t qnn_binary_convnet_workspace_bytes(int64_t B, int64_t H, int64_t Wd, int64_t C0, int in_bits, int n_conv,
                                          const int64_t *cout, const int32_t *pool, int n_fc, const int64_t *fc_out) {
    NetLayout L;
    return net_layout(B, H, Wd, C0, in_bits, n_conv, cout, pool, n_fc, fc_out, L) ? L.total : 0;
}

int qnn_binary_convnet_forward(const uint8_t *x, int64_t B, int64_t H, int64_t Wd, int64_t C0, int in_bits, int n_conv,
                               const int64_t *cout, const int32_t *pool, int n_fc, const int64_t *fc_out,
                               const uint32_t *const *W, const int32_t *const *T, const uint8_t *const *flip,
                               int32_t *logits, int64_t ld_logits, void *workspace, size_t workspace_bytes, int engine,
                               void *stream) {
    if (int rc = check_engine(engine)) return rc;
    NetLayout L;
    if (!net_layout(B, H, Wd, C0, in_bits, n_conv, cout, pool, n_fc, fc_out, L))
        return fail(QNN_ERR_SHAPE, "convnet: bad geometry, layer count or layer widths");
    if (!W || !T) return fail(QNN_ERR_NULL, "convnet: W / T array is NULL");
    if (ld_logits < fc_out[n_fc - 1]) return fail(QNN_ERR_SHAPE, "convnet: ld_logits below the output width");
    if (B == 0) return QNN_OK;
    if (!x || !logits) return fail(QNN_ERR_NULL, "convnet: x or logits is NULL");
    const int n_layers = n_conv + n_fc;
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l]) return fail(QNN_ERR_NULL, "convnet: W[%d] is NULL", l);
        if (l < n_layers - 1 && !T[l]) return fail(QNN_ERR_NULL, "convnet: T[%d] is NULL", l);
    }
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < L.total)
        return fail(QNN_ERR_WORKSPACE, "convnet: workspace must be 256-byte aligned and hold %zu bytes", L.total);
    if (B * H * Wd > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "convnet: too many pixels");

    uint8_t *ws = static_cast<uint8_t *>(workspace);
    auto words = [&](size_t off) { return reinterpret_cast<uint32_t *>(ws + off); };
    static thread_local NetPlan plan;  // large: kept out of the stack
    plan.n = 0;
    auto push = [&]() -> NetStep & {
        NetStep &st = plan.step[plan.n++];
        std::memset(&st, 0, sizeof(st));
        return st;
    };
    auto choose = [&](const GemmArgs &g, int &chosen) {
        int rc = resolve_engine(g, engine, chosen);
        if (rc == QNN_ERR_UNSUPPORTED && engine != QNN_ENGINE_AUTO) rc = resolve_engine(g, QNN_ENGINE_AUTO, chosen);
        return rc;
    };
    // per-layer flags: packed flip bits (for the pooling) and inverted flip bytes (for layers that emit plane 1)
    plan.flags.count = n_layers - 1;
    for (int l = 0; l < n_layers - 1; ++l) {
        plan.flags.flip[l] = flip ? flip[l] : nullptr;
        plan.flags.n[l] = l < n_conv ? cout[l] : fc_out[l - n_conv];
        plan.flags.bits[l] = words(L.flag_bits[l]);
        plan.flags.inv[l] = ws + L.flag_inv[l];
    }
    const int flags_step = plan.n;
    if (n_layers > 1) push().kind = NetStep::kFlags;
    // convolutions that take the panel-fed FP4 kernel (every one but the first, if the shapes allow): their thresholds
    // per border class, all in one launch
    plan.prep.count = 0;
    plan.prep.zero_line = words(L.zero_line);
    {
        int64_t hh = H, ww = Wd, cc = C0;
        for (int l = 0; l < n_conv; ++l) {
            if (l > 0 && (engine == QNN_ENGINE_AUTO || engine == QNN_ENGINE_MFMA_FP4) && L.total < 0xFFFF0000ull &&
                conv_panel_supports(B, hh, ww, cc, cout[l])) {
                const int j = plan.prep.count++;
                plan.prep.W[j] = W[l], plan.prep.T[j] = T[l];
                plan.prep.out[j] = reinterpret_cast<int32_t *>(ws + L.class_thr[l]);
                plan.prep.N[j] = cout[l], plan.prep.ld[j] = conv_panel_class_ld(cout[l]);
                plan.prep.Cw[j] = (int)words_for(cc);
            }
            if (pool[l]) hh /= 2, ww /= 2;
            cc = cout[l];
        }
    }
    // (one launch prepares both the thresholds and the flags)
    if (plan.prep.count > 0) {
        if (n_layers > 1)
            plan.step[flags_step].kind = NetStep::kConvPrep;
        else
            push().kind = NetStep::kConvPrep;
    }
    // The first convolution multiplies the 8-bit codes themselves when a pixel's patch fits one matrix-core operand
    // row (three channels or fewer); otherwise, and when another engine is asked for, it goes through the input's
    // bit planes (Sec. 2.6): [in_bits][pixels][words per pixel]
    const bool first_direct = (engine == QNN_ENGINE_AUTO || engine == QNN_ENGINE_MFMA) && conv_first_supports(C0, cout[0], 3, 3, 1, 1);
    const int64_t Cw0 = words_for(C0);
    if (!first_direct) {
        NetStep &st = push();
        st.kind = NetStep::kPack;
        st.src = x, st.dst = ws + L.planes0;
        st.rows = B * H * Wd, st.n = C0, st.a = in_bits, st.b = (int)Cw0;
    }
    int32_t coef_in[QNN_MAX_PLANES];
    for (int p = 0; p < in_bits; ++p) coef_in[p] = 1 << p;
    static const int32_t kCoefPm1[2] = {1, -2};  // +1 = 01, -1 = 11, padding = 00
    int64_t h = H, w = Wd, cin = C0;
    int cur = 0;
    const uint32_t *a_planes = words(L.planes0);
    int a_count = in_bits;
    const int32_t *a_coef = coef_in;
    int64_t a_stride = B * H * Wd * Cw0;
    bool empty;
    for (int l = 0; l < n_conv; ++l) {
        const bool last_conv = l == n_conv - 1;
        const bool inverted = !last_conv;  // the output feeds another convolution: write plane 1 ("value is -1")
        const int64_t co = cout[l], Cwo = words_for(co);
        const int64_t ho = pool[l] ? h / 2 : h, wo = pool[l] ? w / 2 : w;
        uint32_t *kept = words(L.act[cur ^ 1]);                       // plane 0 (ones) of the output, if it has one
        uint32_t *kept_bits = inverted ? kept + B * ho * wo * Cwo : kept;  // where the output bits go
        uint32_t *conv_dst = pool[l] ? words(L.tmp) : kept_bits;
        const uint8_t *fl = inverted ? reinterpret_cast<const uint8_t *>(ws + L.flag_inv[l]) : (flip ? flip[l] : nullptr);
        NetStep &st = push();
        st.kind = NetStep::kGemm;
        const Epilogue e{nullptr, 0, T[l], fl, conv_dst, Cwo};
        // (the panel-fed convolution addresses its input and the line of zeros, both in the workspace, with 32-bit offsets)
        const bool panel_engine = (engine == QNN_ENGINE_AUTO || engine == QNN_ENGINE_MFMA_FP4) && L.total < 0xFFFF0000ull;
        const bool on_panel = l > 0 && panel_engine && conv_panel_supports(B, h, w, cin, co);
        // the next convolution reads this layer's output: on the panel-fed kernel it takes the plane "value is -1" alone,
        // otherwise the 2-bit code, whose plane "inside the image" is then written too
        const bool ones_needed = inverted && !(panel_engine && conv_panel_supports(B, ho, wo, co, cout[l + 1]));
        if (on_panel) {
            // the map's plane "value is -1" alone; out = (conv >= T) xor fl, and the kernel takes the complement of fl:
            // the caller's flags where fl is their inversion, the inverted ones where fl is the caller's
            st.kind = NetStep::kConvPanel;
            st.src = a_planes + a_stride, st.mask = W[l], st.dst = conv_dst, st.dst2 = ws + L.class_thr[l];
            st.rows = B, st.a = (int)h, st.b = (int)w, st.c = (int)cin, st.n = co;
            st.g.epi = e;
            st.g.epi.flip = inverted ? (flip ? flip[l] : nullptr) : reinterpret_cast<const uint8_t *>(ws + L.flag_inv[l]);
            st.g.W = words(L.zero_line);
        } else if (l == 0 && first_direct) {
            st.kind = NetStep::kFirstConv;
            st.src = x, st.mask = W[0], st.dst = conv_dst;
            st.dst2 = (ones_needed && !pool[l]) ? kept : nullptr;  // the ones plane of an unpooled output, written alongside
            st.rows = B, st.a = (int)H, st.b = (int)Wd, st.c = (int)C0, st.n = co;
            st.g.epi = e;
        } else {
        if (int rc = conv_args(a_planes, a_count, a_coef, QNN_PLANE_BIT, a_stride, B, h, w, cin, W[l], 1, kOne, QNN_PLANE_SIGN, 0,
                               co, 3, 3, 1, 1, e, engine, st.g, empty))
            return rc;
        if (int rc = choose(st.g, st.engine)) return rc;
        }
        if (pool[l]) {
            NetStep &pl = push();
            pl.kind = NetStep::kPool;
            pl.src = conv_dst, pl.dst = kept_bits;
            pl.rows = B, pl.a = (int)h, pl.b = (int)w, pl.c = (int)Cwo;
            pl.mask = words(L.flag_bits[l]);
            pl.invert = inverted;
            pl.dst2 = ones_needed ? kept : nullptr;  // the ones plane of the pooled output, written alongside
            pl.n = co;
        }
        if (ones_needed && !pool[l] && !(l == 0 && first_direct)) {
            NetStep &on = push();
            on.kind = NetStep::kOnes;
            on.dst = kept, on.rows = B * ho * wo, on.a = (int)Cwo, on.b = (int)co;
        }
        h = ho, w = wo, cin = co;
        a_planes = kept, a_count = 2, a_coef = kCoefPm1, a_stride = B * h * w * Cwo;
        cur ^= 1;
    }
    // fully connected layers on the map flattened in (y, x, c) order: the packed words of a sample are contiguous, and
    // they are the packing of the flattened vector if the channels fill whole words (or the map is a single pixel)
    if (cin % 32 != 0 && h * w > 1)
        return fail(QNN_ERR_UNSUPPORTED, "convnet: the last feature map needs a multiple of 32 channels (or one pixel)");
    int64_t in = h * w * cin;
    const uint32_t *fa = a_planes;  // the last convolution wrote plain sign bits at the start of its buffer
    int64_t fa_ld = h * w * words_for(cin);
    int fcur = 0;
    for (int j = 0; j < n_fc; ++j) {
        const int l = n_conv + j;
        const bool last = j == n_fc - 1;
        const int64_t out = fc_out[j];
        uint32_t *dst = words(L.fc[fcur]);
        const Epilogue e = last ? Epilogue{logits, ld_logits, nullptr, nullptr, nullptr, 0}
                                : Epilogue{nullptr, 0, T[l], flip ? flip[l] : nullptr, dst, mlp_ldw(out)};
        NetStep &st = push();
        st.kind = NetStep::kGemm;
        if (int rc = gemm_args("convnet fc", fa, 1, kOne, QNN_PLANE_SIGN, fa_ld, 0, W[l], 1, kOne, QNN_PLANE_SIGN, words_for(in),
                               0, e, B, out, in, engine, st.g, empty))
            return rc;
        if (int rc = choose(st.g, st.engine)) return rc;
        fa = dst, fa_ld = mlp_ldw(out), in = out;
        fcur ^= 1;
    }
    return run_net(plan, static_cast<hipStream_t>(stream));
}

int qnn_last_engine(void) { return g_last_engine; }

int qnn_last_engines(int *engines, int capacity) {
    for (int i = 0; i < g_engine_count && i < capacity && engines; ++i) engines[i] = g_engines[i];
    return g_engine_count;
}

const char *qnn_last_error(void) { return g_err; }

const char *qnn_version(void) { return "libqnn 0.2 (gfx950)"; }

}  // extern "C"
