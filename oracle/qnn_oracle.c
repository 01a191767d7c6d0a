/*
 * CPU oracle for the run-time path of Quantized Neural Networks (Hubara et al., arXiv 1609.07061).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously-correct statement of what the
 * GPU library has to compute, written from the paper on UNPACKED arrays: one int8 / uint8 / int32 per value,
 * ordinary multiply-accumulate, no bit packing in the arithmetic, no popcount, no intrinsics, no blocking.
 * It shares no code, header, table or helper with the HIP path.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.
 *
 * The method is an exact re-encoding of integer arithmetic (Sec. 6: the packed kernel and the ordinary kernel
 * return identical outputs on -1/+1 inputs), so every function below is the plain definition of its result.
 * All sums are accumulated in int64 and range-checked against int32; a result that does not fit returns
 * QO_ERR_RANGE and leaves the output unspecified.
 *
 * Parity pins (tests marked "not gpu"): fp32 GEMM on +-1 matrices, the agreement-count identity of Eq. (popc),
 * brute force over all sign vectors for tiny K, Eq. (FirstLayer) (planes vs integer values), a library
 * convolution in fp64, the float BatchNorm formula evaluated in double, hand-written expected bits for
 * float edge values, a library max-pooling, and the float pipeline conv -> max-pool -> BatchNorm -> sign of a library
 * in fp64 for the ConvNet, hand-computed values and closed forms for the quantizers, and int64 library products of
 * transposed operands for the backward products.  No function here is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define QO_OK 0
#define QO_ERR_RANGE 1
#define QO_ERR_ARG 2
#define QO_ERR_NOMEM 3

static int fits_i32(int64_t v) { return v >= (int64_t)INT32_MIN && v <= (int64_t)INT32_MAX; }

/* Deterministic binarization, Sec. 2.1 Eq. (1): +1 if x >= 0, -1 otherwise.
 * The comparison is the IEEE one on the value: +0 and -0 both give +1, NaN (which is not >= 0) gives -1,
 * denormals compare by their true value. */
int qo_sign(const float *x, int64_t n, int8_t *s) {
    for (int64_t i = 0; i < n; ++i) {
        float v = x[i];
        s[i] = (v >= 0.0f) ? (int8_t)1 : (int8_t)-1;
    }
    return QO_OK;
}

/* Concatenation of 32 binary variables into one 32-bit word (Sec. 6).  The paper fixes neither the value<->bit
 * encoding nor the bit order; the reading used throughout this build is: +1 <-> bit 1, -1 (or 0) <-> bit 0,
 * element 32*j + t of a row <-> bit t (least significant first) of word j, tail bits beyond K are 0.
 * `s` may hold +-1 (sign values) or {0,1} (a bit plane): any value > 0 sets the bit. */
int qo_pack_bits(const int8_t *s, int64_t rows, int64_t K, uint32_t *words) {
    int64_t Kw = (K + 31) / 32;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t j = 0; j < Kw; ++j) {
            uint32_t w = 0;
            for (int t = 0; t < 32; ++t) {
                int64_t k = 32 * j + t;
                if (k < K && s[r * K + k] > 0) w |= (uint32_t)1 << t;
            }
            words[r * Kw + j] = w;
        }
    }
    return QO_OK;
}

/* Bit planes of an integer code, Sec. 2.6 Eq. (FirstLayer): plane n (n = 1 .. nbits) holds the n-th bit,
 * n = 1 being the least significant (weight 2^(n-1)) and n = nbits the most significant.  planes[p][i] is
 * plane n = p + 1 of value i.  For negative v the bits are those of its two's-complement representation. */
int qo_split_planes(const int32_t *v, int64_t n, int nbits, uint8_t *planes) {
    if (nbits < 1 || nbits > 31) return QO_ERR_ARG;
    for (int p = 0; p < nbits; ++p)
        for (int64_t i = 0; i < n; ++i) planes[(int64_t)p * n + i] = (uint8_t)(((uint32_t)v[i] >> p) & 1u);
    return QO_OK;
}

/* Binary matrix product on +-1 values (Alg. 4, hidden and output layers; Sec. 6):
 * C[m][n] = sum_k a[m][k] * w[n][k], a is M x K, w is N x K (one row per output neuron). */
int qo_gemm_pm1(const int8_t *a, const int8_t *w, int64_t M, int64_t N, int64_t K, int32_t *C) {
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) acc += (int64_t)a[m * K + k] * (int64_t)w[n * K + k];
            if (!fits_i32(acc)) bad = 1;
            C[m * N + n] = (int32_t)acc;
        }
    }
    return bad ? QO_ERR_RANGE : QO_OK;
}

/* Integer matrix product on the VALUES that bit planes encode (left side of Eq. (FirstLayer), s = x . w):
 * C[m][n] = sum_k u[m][k] * v[n][k]. */
int qo_gemm_int(const int32_t *u, const int32_t *v, int64_t M, int64_t N, int64_t K, int32_t *C) {
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) acc += (int64_t)u[m * K + k] * (int64_t)v[n * K + k];
            if (!fits_i32(acc)) bad = 1;
            C[m * N + n] = (int32_t)acc;
        }
    }
    return bad ? QO_ERR_RANGE : QO_OK;
}

/* Value of one plane entry: mode 0 ("bit") reads the stored bit as 0/1, mode 1 ("sign") reads it as -1/+1. */
static int plane_value(uint8_t bit, int mode) { return mode ? (bit ? 1 : -1) : (bit ? 1 : 0); }

/* Right side of Eq. (FirstLayer) generalised to both operands (Sec. 3: one binary product per pair of planes):
 * C = sum_i sum_j ca[i] * cw[j] * (A_i . W_j^T), taken plane pair by plane pair with explicit coefficients.
 * pa is [Pa][M][K], pw is [Pb][N][K], entries 0/1. */
int qo_gemm_planes(const uint8_t *pa, int Pa, const int32_t *ca, int modeA, const uint8_t *pw, int Pb,
                   const int32_t *cw, int modeW, int64_t M, int64_t N, int64_t K, int32_t *C) {
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t total = 0;
            for (int i = 0; i < Pa; ++i) {
                for (int j = 0; j < Pb; ++j) {
                    const uint8_t *ar = pa + ((int64_t)i * M + m) * K;
                    const uint8_t *wr = pw + ((int64_t)j * N + n) * K;
                    int64_t dot = 0;
                    for (int64_t k = 0; k < K; ++k) dot += plane_value(ar[k], modeA) * plane_value(wr[k], modeW);
                    total += (int64_t)ca[i] * (int64_t)cw[j] * dot;
                }
            }
            if (!fits_i32(total)) bad = 1;
            C[m * N + n] = (int32_t)total;
        }
    }
    return bad ? QO_ERR_RANGE : QO_OK;
}

/* Sign(BatchNorm(.)) of Alg. 4 once BatchNorm has been folded to an integer threshold per neuron:
 * out = +1 if (C[m][n] >= T[n]) differs from flip[n], else -1.  flip may be NULL (all zero). */
int qo_threshold(const int32_t *C, int64_t M, int64_t N, const int32_t *T, const uint8_t *flip, int8_t *out) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int ge = C[m * N + n] >= T[n];
            int f = flip ? (flip[n] != 0) : 0;
            out[m * N + n] = (ge != f) ? (int8_t)1 : (int8_t)-1;
        }
    return QO_OK;
}

/* Sign(BatchNorm(s)) straight from the float definition, in double: y = gamma * (s - mean) / sqrt(var + eps) + beta,
 * out = +1 if y >= 0 else -1 (Alg. 4 with the inference-time BatchNorm; Eq. (1)).  Used to pin the threshold fold. */
int qo_bn_sign(const int32_t *C, int64_t M, int64_t N, const double *gamma, const double *beta, const double *mean,
               const double *var, double eps, int8_t *out) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double sd = __builtin_sqrt(var[n] + eps);
            double y = gamma[n] * (((double)C[m * N + n] - mean[n]) / sd) + beta[n];
            out[m * N + n] = (y >= 0.0) ? (int8_t)1 : (int8_t)-1;
        }
    return QO_OK;
}

/* Alg. 4, "Running a BNN with L layers", up to and including the integer output-layer product:
 *   layer 1   : a_1 = x . W_1 on the 8-bit (in general unsigned integer) inputs, a_1^b = Sign(BN(a_1))
 *   layers k  : a_k = a_{k-1}^b . W_k,  a_k^b = Sign(BN(a_k))         (k = 2 .. L-1)
 *   layer L   : logits = a_{L-1}^b . W_L                              (the final float BatchNorm is left out)
 * W[l] is dims[l+1] x dims[l] in +-1; T[l], flip[l] (l < L-1) are the folded BatchNorm of layer l+1. */
int qo_mlp(const uint8_t *x, int64_t batch, int n_layers, const int64_t *dims, const int8_t *const *W,
           const int32_t *const *T, const uint8_t *const *flip, int32_t *logits) {
    if (n_layers < 1) return QO_ERR_ARG;
    int rc = QO_OK;
    int64_t maxd = 0;
    for (int l = 0; l <= n_layers; ++l)
        if (dims[l] > maxd) maxd = dims[l];
    int32_t *sum = (int32_t *)malloc(sizeof(int32_t) * (size_t)batch * (size_t)maxd);
    int8_t *act = (int8_t *)malloc((size_t)batch * (size_t)maxd);
    int32_t *x32 = (int32_t *)malloc(sizeof(int32_t) * (size_t)batch * (size_t)dims[0]);
    int32_t *w32 = (int32_t *)malloc(sizeof(int32_t) * (size_t)dims[1] * (size_t)dims[0]);
    if (!sum || !act || !x32 || !w32) {
        rc = QO_ERR_NOMEM;
        goto done;
    }
    for (int64_t i = 0; i < batch * dims[0]; ++i) x32[i] = (int32_t)x[i];
    for (int64_t i = 0; i < dims[1] * dims[0]; ++i) w32[i] = (int32_t)W[0][i];
    for (int l = 0; l < n_layers; ++l) {
        int32_t *dst = (l == n_layers - 1) ? logits : sum;
        if (l == 0)
            rc = qo_gemm_int(x32, w32, batch, dims[1], dims[0], dst);
        else
            rc = qo_gemm_pm1(act, W[l], batch, dims[l + 1], dims[l], dst);
        if (rc != QO_OK) goto done;
        if (l < n_layers - 1) qo_threshold(sum, batch, dims[l + 1], T[l], flip ? flip[l] : NULL, act);
    }
done:
    free(sum);
    free(act);
    free(x32);
    free(w32);
    return rc;
}

/* Direct 2-D convolution (cross-correlation, as in every deep-learning framework) with zero padding on integer
 * values; u is [B][H][W][Ci] (channels last), w is [Co][KH][KW][Ci] (the M_l x M_{l-1} x k x k filter bank of
 * Sec. 5, channels last), out is [B][Ho][Wo][Co] with Ho = (H + 2*pad - KH) / stride + 1.  Inputs outside the
 * image contribute exactly 0. */
int qo_conv2d(const int32_t *u, int64_t B, int64_t H, int64_t Wd, int64_t Ci, const int32_t *w, int64_t Co,
              int64_t KH, int64_t KW, int64_t pad, int64_t stride, int32_t *out) {
    if (stride < 1 || H + 2 * pad < KH || Wd + 2 * pad < KW) return QO_ERR_ARG;
    int64_t Ho = (H + 2 * pad - KH) / stride + 1, Wo = (Wd + 2 * pad - KW) / stride + 1;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : bad)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t y = 0; y < Ho; ++y)
            for (int64_t xo = 0; xo < Wo; ++xo)
                for (int64_t co = 0; co < Co; ++co) {
                    int64_t acc = 0;
                    for (int64_t ky = 0; ky < KH; ++ky)
                        for (int64_t kx = 0; kx < KW; ++kx) {
                            int64_t iy = y * stride + ky - pad, ix = xo * stride + kx - pad;
                            if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                            const int32_t *up = u + ((b * H + iy) * Wd + ix) * Ci;
                            const int32_t *wp = w + ((co * KH + ky) * KW + kx) * Ci;
                            for (int64_t ci = 0; ci < Ci; ++ci) acc += (int64_t)up[ci] * (int64_t)wp[ci];
                        }
                    if (!fits_i32(acc)) bad = 1;
                    out[((b * Ho + y) * Wo + xo) * Co + co] = (int32_t)acc;
                }
    return bad ? QO_ERR_RANGE : QO_OK;
}

/* 2 x 2 max-pooling with stride 2 on integer feature maps (App. A, CIFAR-10 ConvNet: "convolution and 2 x 2 max-pooling
 * layers" followed by "BatchNorm and Binarization layers", i.e. the pooling acts on the convolution's sums).
 * u is [B][H][W][C] (channels last), out is [B][H/2][W/2][C]; a last odd row / column is dropped (floor), as the
 * deep-learning frameworks do by default. */
int qo_maxpool2x2(const int32_t *u, int64_t B, int64_t H, int64_t Wd, int64_t C, int32_t *out) {
    int64_t Ho = H / 2, Wo = Wd / 2;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t y = 0; y < Ho; ++y)
            for (int64_t x = 0; x < Wo; ++x)
                for (int64_t c = 0; c < C; ++c) {
                    int32_t m = u[((b * H + 2 * y) * Wd + 2 * x) * C + c];
                    for (int dy = 0; dy < 2; ++dy)
                        for (int dx = 0; dx < 2; ++dx) {
                            int32_t v = u[((b * H + 2 * y + dy) * Wd + 2 * x + dx) * C + c];
                            if (v > m) m = v;
                        }
                    out[((b * Ho + y) * Wo + x) * C + c] = m;
                }
    return QO_OK;
}

/* Alg. 4 for a binarized ConvNet of the shape of App. A (CIFAR-10 ConvNet table): a run of 3 x 3 "same" convolutions
 * (zero padding, stride 1), some followed by 2 x 2 max-pooling, each followed by Sign(BatchNorm(.)) given as a folded
 * threshold; then fully connected layers on the flattened (y, x, c) feature map, the last one without threshold.
 *   x        : uint8 [B][H][W][C0] (8-bit inputs: the first layer is the integer product of Sec. 2.6)
 *   n_conv   : number of convolution layers; cout[l], pool[l] (0/1) for l < n_conv
 *   n_fc     : number of fully connected layers (>= 1); fc_out[j]
 *   W        : n_conv + n_fc pointers to +-1 weights: conv [cout][3][3][cin], fc [out][in]
 *   T, flip  : n_conv + n_fc - 1 pointers (flip, or entries of it, may be NULL)
 * Activations between layers are +-1; a padded position contributes exactly 0 to a convolution (it is not a -1).
 * logits: int32 [B][fc_out[n_fc-1]]. */
int qo_convnet(const uint8_t *x, int64_t B, int64_t H, int64_t Wd, int64_t C0, int n_conv, const int64_t *cout,
               const int32_t *pool, int n_fc, const int64_t *fc_out, const int8_t *const *W, const int32_t *const *T,
               const uint8_t *const *flip, int32_t *logits) {
    if (n_conv < 0 || n_fc < 1) return QO_ERR_ARG;
    int rc = QO_OK;
    int64_t h = H, w = Wd, c = C0;
    int32_t *act = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * H * Wd * C0));  /* integer values of the current map */
    if (!act) return QO_ERR_NOMEM;
    for (int64_t i = 0; i < B * H * Wd * C0; ++i) act[i] = (int32_t)x[i];
    for (int l = 0; l < n_conv && rc == QO_OK; ++l) {
        int64_t co = cout[l];
        int32_t *w32 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(co * 9 * c));
        int32_t *sum = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * h * w * co));
        if (!w32 || !sum) {
            free(w32), free(sum), free(act);
            return QO_ERR_NOMEM;
        }
        for (int64_t i = 0; i < co * 9 * c; ++i) w32[i] = (int32_t)W[l][i];
        rc = qo_conv2d(act, B, h, w, c, w32, co, 3, 3, 1, 1, sum);
        free(w32);
        free(act);
        act = NULL;
        int64_t ho = h, wo = w;
        if (rc == QO_OK && pool[l]) {
            ho = h / 2, wo = w / 2;
            int32_t *p = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * ho * wo * co));
            if (!p) {
                free(sum);
                return QO_ERR_NOMEM;
            }
            qo_maxpool2x2(sum, B, h, w, co, p);
            free(sum);
            sum = p;
        }
        int8_t *s8 = (int8_t *)malloc((size_t)(B * ho * wo * co));
        act = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * ho * wo * co));
        if (!s8 || !act) {
            free(s8), free(sum), free(act);
            return QO_ERR_NOMEM;
        }
        if (rc == QO_OK) {
            qo_threshold(sum, B * ho * wo, co, T[l], flip ? flip[l] : NULL, s8);
            for (int64_t i = 0; i < B * ho * wo * co; ++i) act[i] = (int32_t)s8[i];
        }
        free(s8);
        free(sum);
        h = ho, w = wo, c = co;
    }
    /* fully connected layers on the map flattened in (y, x, c) order */
    int64_t in = h * w * c;
    for (int j = 0; j < n_fc && rc == QO_OK; ++j) {
        int l = n_conv + j;
        int64_t out = fc_out[j];
        int last = j == n_fc - 1;
        int32_t *w32 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(out * in));
        int32_t *sum = last ? logits : (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * out));
        if (!w32 || !sum) {
            free(w32);
            if (!last) free(sum);
            free(act);
            return QO_ERR_NOMEM;
        }
        for (int64_t i = 0; i < out * in; ++i) w32[i] = (int32_t)W[l][i];
        rc = qo_gemm_int(act, w32, B, out, in, sum);
        free(w32);
        if (!last) {
            int8_t *s8 = (int8_t *)malloc((size_t)(B * out));
            free(act);
            act = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * out));
            if (!s8 || !act) {
                free(s8), free(sum), free(act);
                return QO_ERR_NOMEM;
            }
            if (rc == QO_OK) {
                qo_threshold(sum, B, out, T[l], flip ? flip[l] : NULL, s8);
                for (int64_t i = 0; i < B * out; ++i) act[i] = (int32_t)s8[i];
            }
            free(s8);
            free(sum);
        }
        in = out;
    }
    free(act);
    return rc;
}

/* Linear quantization of Sec. 3, LinearQuant(x, step) = Clip(round(x / step) * step, minV, maxV), returned as the
 * INTEGER code q = value / step (the bit-plane products consume codes; the value is q * step):
 *   q = Clip(round(x / step), qmin, qmax),  qmin = minV / step, qmax = maxV / step.
 * Readings (the paper's formula names the step "bitwidth" and leaves the rest open): the quotient is formed and
 * rounded in single precision, the precision of the activations; round is to nearest with ties to even (the default
 * of IEEE arithmetic and of the array libraries the paper used); NaN, which no comparison orders, quantizes like 0. */
int qo_linear_quant(const float *x, int64_t n, float step, int32_t qmin, int32_t qmax, int32_t *q) {
    if (!(step > 0.0f) || qmin > qmax) return QO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        volatile float t = x[i] / step; /* volatile: no wider intermediate */
        float r = nearbyintf(t);        /* default rounding mode: ties to even */
        if (r != r) r = 0.0f;
        int32_t v;
        if (r <= (float)qmin)
            v = qmin;
        else if (r >= (float)qmax)
            v = qmax;
        else
            v = (int32_t)r;
        q[i] = v;
    }
    return QO_OK;
}

/* Approximate power of two (caption of Alg. 2): AP2(x) = sign(x) * 2^round(log2 |x|), evaluated in double precision
 * on the single-precision input.  |x| is never exactly half way between two powers of two in the log domain
 * (2^(e + 1/2) is irrational), so no tie rule is needed.  Writes the exponent round(log2 |x|) and the sign (+1 / -1);
 * for x = 0 and NaN the sign is 0 (AP2(0) is read as 0; log2 0 has no value).  +-inf gives exponent INT32_MAX. */
int qo_ap2(const float *x, int64_t n, int32_t *exponent, int8_t *sign) {
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)x[i];
        if (v != v || v == 0.0) {
            sign[i] = 0;
            exponent[i] = 0;
            continue;
        }
        sign[i] = v > 0.0 ? 1 : -1;
        double a = fabs(v);
        if (isinf(a)) {
            exponent[i] = INT32_MAX;
            continue;
        }
        exponent[i] = (int32_t)floor(log2(a) + 0.5);
    }
    return QO_OK;
}

/* Logarithmic quantization of Sec. 3, LogQuant(x) = Clip(AP2(x), minV, maxV), as a signed code:
 *   code = 0                          if x is 0 or NaN, or AP2(x) lies below 2^emin in magnitude,
 *   code = sign(x) * (e - emin + 1)   otherwise, e = min(round(log2 |x|), emax);   value = sign * 2^(emin + |code| - 1).
 * Reading: minV and maxV bound the MAGNITUDE (2^emin and 2^emax); what rounds below the smallest magnitude is
 * flushed to zero, what rounds above the largest is clipped to it.  emax - emin + 1 <= 127. */
int qo_log_quant(const float *x, int64_t n, int32_t emin, int32_t emax, int8_t *code) {
    if (emin > emax || (int64_t)emax - emin + 1 > 127) return QO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        int32_t e;
        int8_t sg;
        qo_ap2(x + i, 1, &e, &sg);
        if (sg == 0 || e < emin) {
            code[i] = 0;
            continue;
        }
        if (e > emax) e = emax;
        code[i] = (int8_t)(sg * (e - emin + 1));
    }
    return QO_OK;
}

/* Fixed-point value of a logarithmic code (Sec. 3 LogQuant; Sec. 6: with quantized gradients the backward pass can
 * run on the bit-wise kernel): code c encodes sign(c) * 2^(emin + |c| - 1); scaled by 2^-emin that is the INTEGER
 * sign(c) * 2^(|c| - 1), which a matrix product can consume as two's-complement bit planes.  Code 0 is 0. */
int qo_log_code_value(const int8_t *code, int64_t n, int32_t *value) {
    for (int64_t i = 0; i < n; ++i) {
        int c = code[i];
        int mag = c < 0 ? -c : c;
        if (mag > 31) return QO_ERR_RANGE;
        value[i] = c == 0 ? 0 : (c < 0 ? -(int32_t)(1 << (mag - 1)) : (int32_t)(1 << (mag - 1)));
    }
    return QO_OK;
}

/* Straight-through estimator of Alg. 1 (backward block): g_a = g_{a^b} o 1_{|a| <= 1}: the gradient passes where the
 * pre-binarization activation lies in [-1, 1] and is cancelled elsewhere (NaN is not <= 1: cancelled). */
int qo_ste_mask(const float *g, const float *a, int64_t n, float *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = (fabsf(a[i]) <= 1.0f) ? g[i] : 0.0f;
    return QO_OK;
}

/* Affine form of the inference-time BatchNorm of the output layer (Alg. 4, last line): y = scale[n] * s + shift[n]
 * on the integer sums s, evaluated as ONE fused multiply-add in single precision (one rounding). */
int qo_bn_affine(const int32_t *s, int64_t M, int64_t N, const float *scale, const float *shift, float *y) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) y[m * N + n] = fmaf((float)s[m * N + n], scale[n], shift[n]);
    return QO_OK;
}

/* Backward products of Alg. 1 with binary weights and integer (quantized) gradients:
 *   g_a[m][k] = sum_n g[m][n] * W[n][k]        (g_{a_{k-1}^b} = g_{s_k} W_k^b)
 *   g_W[n][k] = sum_m g[m][n] * a[m][k]        (g_{W_k^b}   = g_{s_k}^T a_{k-1}^b)
 * g: int32 [M][N], W: int8 +-1 [N][K], a: int8 +-1 [M][K].  Plain triple loops, int64 accumulation. */
int qo_backward(const int32_t *g, const int8_t *W, const int8_t *a, int64_t M, int64_t N, int64_t K, int32_t *g_a,
                int32_t *g_W) {
    int rc = QO_OK;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            int64_t acc = 0;
            for (int64_t n = 0; n < N; ++n) acc += (int64_t)g[m * N + n] * (int64_t)W[n * K + k];
            if (!fits_i32(acc)) rc = QO_ERR_RANGE;
            g_a[m * K + k] = (int32_t)acc;
        }
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t acc = 0;
            for (int64_t m = 0; m < M; ++m) acc += (int64_t)g[m * N + n] * (int64_t)a[m * K + k];
            if (!fits_i32(acc)) rc = QO_ERR_RANGE;
            g_W[n * K + k] = (int32_t)acc;
        }
    return rc;
}

/* Repetition of binary 2-D filters (Sec. 5): a filter bank of +-1 weights w[co][ky][kx][ci] holds, for every input
 * channel ci, cout 2-D filters of kh x kw taps, of which many repeat; a filter and its negation count as one (the
 * negated filter's response is minus the original's).  counts[ci] = number of distinct 2-D filters of channel ci up
 * to negation, found by comparing every filter with every earlier one, tap by tap. */
int qo_filter_unique(const int8_t *w, int64_t cout, int64_t kh, int64_t kw, int64_t cin, int32_t *counts) {
    int64_t taps = kh * kw;
    for (int64_t ci = 0; ci < cin; ++ci) {
        int32_t n = 0;
        for (int64_t co = 0; co < cout; ++co) {
            int seen = 0;
            for (int64_t prev = 0; prev < co && !seen; ++prev) {
                int same = 1, opposite = 1;
                for (int64_t t = 0; t < taps; ++t) {
                    int a = w[(co * taps + t) * cin + ci], b = w[(prev * taps + t) * cin + ci];
                    if (a != b) same = 0;
                    if (a != -b) opposite = 0;
                }
                seen = same || opposite;
            }
            if (!seen) ++n;
        }
        counts[ci] = n;
    }
    return QO_OK;
}

/* The convolution of qo_conv2d evaluated the way Sec. 5 proposes: for every input channel only the distinct 2-D
 * filters (up to negation) are applied to that channel's map, and every output channel adds, with the sign of its own
 * filter relative to the representative, the response of the representative it repeats.  u: integer codes
 * [B][H][W][cin], w: +-1 [cout][kh][kw][cin], zero padding `pad`, stride 1; out int32 [B][Ho][Wo][cout].
 * applied[0] receives the number of 2-D filter applications (sum over channels of the distinct count). */
int qo_conv2d_dedup(const int32_t *u, int64_t B, int64_t H, int64_t W, int64_t cin, const int8_t *w, int64_t cout,
                    int64_t kh, int64_t kw, int64_t pad, int32_t *out, int64_t *applied) {
    int64_t ho = H + 2 * pad - kh + 1, wo = W + 2 * pad - kw + 1, taps = kh * kw;
    if (ho < 1 || wo < 1) return QO_ERR_ARG;
    int64_t npix = B * ho * wo;
    int64_t *acc = (int64_t *)calloc((size_t)(npix * cout), sizeof(int64_t));
    int64_t *resp = (int64_t *)malloc(sizeof(int64_t) * (size_t)npix);
    int64_t *rep = (int64_t *)malloc(sizeof(int64_t) * (size_t)cout);   /* representative filter of each output channel */
    int *sgn = (int *)malloc(sizeof(int) * (size_t)cout);
    if (!acc || !resp || !rep || !sgn) {
        free(acc), free(resp), free(rep), free(sgn);
        return QO_ERR_NOMEM;
    }
    int64_t count = 0;
    for (int64_t ci = 0; ci < cin; ++ci) {
        for (int64_t co = 0; co < cout; ++co) {
            rep[co] = co, sgn[co] = 1;
            for (int64_t prev = 0; prev < co; ++prev) {
                if (rep[prev] != prev) continue;
                int same = 1, opposite = 1;
                for (int64_t t = 0; t < taps; ++t) {
                    int a = w[(co * taps + t) * cin + ci], b = w[(prev * taps + t) * cin + ci];
                    if (a != b) same = 0;
                    if (a != -b) opposite = 0;
                }
                if (same || opposite) {
                    rep[co] = prev, sgn[co] = same ? 1 : -1;
                    break;
                }
            }
        }
        for (int64_t r = 0; r < cout; ++r) {
            if (rep[r] != r) continue;
            ++count;
            /* response of representative r on channel ci */
            for (int64_t b = 0; b < B; ++b)
                for (int64_t y = 0; y < ho; ++y)
                    for (int64_t x = 0; x < wo; ++x) {
                        int64_t s = 0;
                        for (int64_t ky = 0; ky < kh; ++ky)
                            for (int64_t kx = 0; kx < kw; ++kx) {
                                int64_t iy = y + ky - pad, ix = x + kx - pad;
                                if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                                s += (int64_t)u[((b * H + iy) * W + ix) * cin + ci] * w[((r * kh + ky) * kw + kx) * cin + ci];
                            }
                        resp[(b * ho + y) * wo + x] = s;
                    }
            for (int64_t co = 0; co < cout; ++co)
                if (rep[co] == r)
                    for (int64_t p = 0; p < npix; ++p) acc[p * cout + co] += sgn[co] * resp[p];
        }
    }
    int rc = QO_OK;
    for (int64_t i = 0; i < npix * cout; ++i) {
        if (!fits_i32(acc[i])) rc = QO_ERR_RANGE;
        out[i] = (int32_t)acc[i];
    }
    if (applied) applied[0] = count;
    free(acc), free(resp), free(rep), free(sgn);
    return rc;
}

/* Number of threads the OpenMP loops above actually use (reported beside the CPU-baseline timing). */
int qo_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
