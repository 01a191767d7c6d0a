/*
 * qnn.h - C ABI of the MI355X (gfx950) library for the run-time path of Quantized Neural Networks
 * (Hubara, Courbariaux, Soudry, El-Yaniv, Bengio; arXiv 1609.07061).
 *
 * The path: sign-binarize and bit-pack values (Sec. 2.1 Eq. (1); Sec. 6 "concatenate groups of 32 binary variables
 * into 32-bit registers"), multiply packed matrices by counting agreements (Sec. 6 Eq. (popc)), handle multi-bit
 * inputs / activations / weights as weighted sums of binary products over bit planes (Sec. 2.6 Eq. (FirstLayer);
 * Sec. 3), and apply Sign(BatchNorm(.)) between layers (Alg. 4) as an integer threshold per neuron.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Pointers marked DEVICE are HIP device pointers owned by the caller; the library never allocates, frees or keeps
 *    them.  Pointers marked HOST are read during the call only.  In-place or overlapping input/output is undefined.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work on `stream`;
 *    they do not synchronize.
 *  - Return value: QNN_OK (0), or a positive qnn_status; on error nothing has been enqueued and
 *    qnn_last_error() (thread-local) describes the problem.  Nothing throws across this boundary.
 *  - Matrices are row-major.  A is M x K (one row per sample), W is N x K (one row per output neuron),
 *    C = A . W^T is M x N.  Leading dimensions are in ELEMENTS of the pointed-to type.
 *  - Packed format (the paper leaves it open; this is the library's definition): element k of a row lives in bit
 *    (k mod 32), least significant first, of 32-bit word (k div 32); little-endian, so a 64-bit view of two words
 *    holds 64 consecutive elements.  Bit 1 means +1 (sign planes) or 1 (bit planes); bit 0 means -1 or 0.
 *    A packed row of K elements occupies ceil(K/32) words and ITS TAIL BITS (positions K .. 32*ceil(K/32)-1) MUST BE
 *    ZERO.  The packing calls guarantee it; the multiply calls rely on it.
 *  - Packed buffers must be 4-byte aligned; 16-byte aligned bases with leading dimensions that are multiples of 4
 *    words enable the wide-load paths (anything else is still computed correctly, only slower).
 *  - M == 0 or N == 0 is a successful no-op.  K must be >= 1.
 */
#ifndef QNN_H
#define QNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QNN_OK = 0,
    QNN_ERR_NULL = 1,        /* a required pointer is NULL */
    QNN_ERR_SHAPE = 2,       /* a size, leading dimension, plane count or mode is out of range */
    QNN_ERR_ALIGN = 3,       /* a pointer is not 4-byte aligned */
    QNN_ERR_OVERFLOW = 4,    /* (sum |coefA|) * (sum |coefW|) * K does not fit int32 */
    QNN_ERR_UNSUPPORTED = 5, /* requested variant cannot handle these arguments */
    QNN_ERR_WORKSPACE = 6,   /* workspace NULL, misaligned (256 B) or too small */
    QNN_ERR_HIP = 7          /* the HIP runtime reported an error at launch */
} qnn_status;

/* How the entries of a packed plane are read (Sec. 2.6 uses 0/1 bit planes of the input against -1/+1 weights). */
typedef enum {
    QNN_PLANE_BIT = 0, /* stored bit b is the number b        in {0, 1}  */
    QNN_PLANE_SIGN = 1 /* stored bit b is the number 2b - 1   in {-1, +1} */
} qnn_plane_mode;

/* Which inner product engine a multiply uses.  Results are identical bit for bit; only the speed differs. */
typedef enum {
    QNN_ENGINE_AUTO = 0, /* library's choice for the shape */
    QNN_ENGINE_VALU = 1, /* 32 connections per xor/and + popcount-accumulate pair (Sec. 6 Eq. (popc)) */
    QNN_ENGINE_MFMA = 2, /* bits expanded on chip to int8 and contracted on the matrix cores */
    QNN_ENGINE_MFMA_FP4 = 3, /* single-plane operands expanded to FP4 zeros and ones, contracted on the matrix cores
                                with fp32 accumulation (exact: the sums are integers far below 2^24) */
    QNN_ENGINE_MFMA_LDS = 4 /* as QNN_ENGINE_MFMA for operands of several bit planes, merged into int8 once: per
                               workgroup in LDS (16-byte aligned operands with rows of whole groups of four words,
                               plane counts 1, 2, 4 or 8, coefficients a common factor times 1, 2, 4, ...), or, for
                               large products with int32 output, per call in memory (see qnn_bitplane_gemm) */
} qnn_engine;

#define QNN_MAX_PLANES 8
#define QNN_MAX_LAYERS 16

/* S1. Deterministic binarization (Sec. 2.1 Eq. (1): +1 if x >= 0, -1 otherwise) fused with packing (Sec. 6).
 * x: DEVICE float32 [rows][ldx], the first K of each row used.  out: DEVICE uint32 [rows][ldo_words], the first
 * ceil(K/32) words of each row written (tail bits zero), the rest untouched.
 * The comparison is IEEE on the value: +0, -0 -> +1; NaN -> -1; denormals are not flushed.
 * Requires ldx >= K, ldo_words >= ceil(K/32). */
int qnn_pack_sign(const float *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *out, int64_t ldo_words,
                  void *stream);

/* S1b. Bit planes of integer codes (Sec. 2.6: x^n is the n-th bit, n = 1 least significant ... n = nbits most
 * significant) packed along K.  v: DEVICE uint8 [rows][ldv], one code per byte (two's-complement codes are passed
 * as their low nbits).  planes: DEVICE uint32, plane p (= the paper's n - 1) of row r starts at
 * planes + p * plane_stride_words + r * ld_words.  1 <= nbits <= 8. */
int qnn_pack_bitplanes(const uint8_t *v, int64_t rows, int64_t K, int64_t ldv, int nbits, uint32_t *planes,
                       int64_t ld_words, int64_t plane_stride_words, void *stream);

/* S2. Binary matrix product of Alg. 4 / Sec. 6 on packed +-1 operands:
 * C[m][n] = sum_k a[m][k] w[n][k] = K - 2 * popcount(A[m] xor W[n])  (Eq. (popc) counts the agreements).
 * A: DEVICE uint32 [M][lda_words], W: DEVICE uint32 [N][ldw_words], C: DEVICE int32 [M][ldc]. K < 2^31. */
int qnn_binary_gemm(const uint32_t *A, int64_t lda_words, const uint32_t *W, int64_t ldw_words, int32_t *C,
                    int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream);

/* Same product with the engine chosen by the caller (for measurements and tests). */
int qnn_binary_gemm_ex(const uint32_t *A, int64_t lda_words, const uint32_t *W, int64_t ldw_words, int32_t *C,
                       int64_t ldc, int64_t M, int64_t N, int64_t K, int engine, void *stream);

/* S2+S4 fused. a^b = Sign(BatchNorm(a . W^T)) of Alg. 4 without materialising the int32 sums:
 * bit[m][n] = (C[m][n] >= T[n]) xor flip[n], written packed along n (n is the next layer's K):
 * out: DEVICE uint32 [M][ldo_words], first ceil(N/32) words of each row, tail bits zero.
 * T: DEVICE int32 [N]; flip: DEVICE uint8 [N] (non-zero = invert) or NULL. */
int qnn_binary_gemm_sign(const uint32_t *A, int64_t lda_words, const uint32_t *W, int64_t ldw_words,
                         const int32_t *T, const uint8_t *flip, uint32_t *out, int64_t ldo_words, int64_t M,
                         int64_t N, int64_t K, int engine, void *stream);

/* S3. Multi-bit product as a weighted sum of binary products (Sec. 2.6 Eq. (FirstLayer), Sec. 3):
 * C = sum_{i<Pa} sum_{j<Pb} coefA[i] * coefW[j] * (A_i . W_j^T), plane entries read according to modeA / modeW.
 * A_i = A + i * strideA_words is [M][lda_words]; W_j = W + j * strideW_words is [N][ldw_words].
 * coefA, coefW: HOST int32 arrays (e.g. 1,2,4,...,128 for 8-bit unsigned inputs; 1,2,4,-8 for 4-bit two's
 * complement).  1 <= Pa, Pb <= QNN_MAX_PLANES.  QNN_ERR_OVERFLOW if (sum|coefA|)(sum|coefW|) K >= 2^31.
 * Large products (M, N >= 256, K >= 512, M N K >= 2^31) of multi-plane operands whose values fit int8 are computed
 * from the values: both operands' planes are merged to one byte per element in temporary device memory of
 * (M + N) * roundup(K, 128) bytes that the call takes from, and returns to, the memory pool of `stream`
 * (hipMallocAsync / hipFreeAsync: stream-ordered, no synchronization); QNN_ERR_HIP if the pool cannot supply it.
 * qnn_binary_backward's two products are of this kind. */
int qnn_bitplane_gemm(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda_words,
                      int64_t strideA_words, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
                      int64_t ldw_words, int64_t strideW_words, int32_t *C, int64_t ldc, int64_t M, int64_t N,
                      int64_t K, void *stream);

/* Same product with the engine chosen by the caller (for measurements and tests). */
int qnn_bitplane_gemm_ex(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda_words,
                         int64_t strideA_words, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
                         int64_t ldw_words, int64_t strideW_words, int32_t *C, int64_t ldc, int64_t M, int64_t N,
                         int64_t K, int engine, void *stream);

/* S3+S4 fused: the first layer of Alg. 4 (eight weighted plane products, then Sign(BatchNorm(.))), output packed. */
int qnn_bitplane_gemm_sign(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t lda_words,
                           int64_t strideA_words, const uint32_t *W, int Pb, const int32_t *coefW, int modeW,
                           int64_t ldw_words, int64_t strideW_words, const int32_t *T, const uint8_t *flip,
                           uint32_t *out, int64_t ldo_words, int64_t M, int64_t N, int64_t K, int engine,
                           void *stream);

/* S4. Sign(BatchNorm(.)) of Alg. 4 on materialised sums, with BatchNorm folded to an integer threshold:
 * bit[m][n] = (C[m][n] >= T[n]) xor flip[n], packed along n.  C: DEVICE int32 [M][ldc]; T: DEVICE int32 [N];
 * flip: DEVICE uint8 [N] or NULL; out: DEVICE uint32 [M][ldo_words] (first ceil(N/32) words per row). */
int qnn_threshold_sign(const int32_t *C, int64_t ldc, int64_t M, int64_t N, const int32_t *T, const uint8_t *flip,
                       uint32_t *out, int64_t ldo_words, void *stream);

/* Host helper: fold inference-time BatchNorm y = gamma (s - mean) / sqrt(var + eps) + beta followed by Eq. (1)
 * into (T, flip) such that for every integer s:  (y >= 0)  <=>  ((s >= T) xor flip).
 * gamma > 0: T = ceil(mean - beta sqrt(var+eps) / gamma), flip = 0;  gamma < 0: T = floor(same) + 1, flip = 1;
 * gamma == 0: T = INT32_MIN, flip = (beta < 0).  Thresholds beyond int32 saturate (the comparison then has a
 * constant outcome for every representable s).  All arrays HOST, length n; computed in double.  No GPU involved. */
int qnn_fold_batchnorm(const double *gamma, const double *beta, const double *mean, const double *var, double eps,
                       int64_t n, int32_t *T, uint8_t *flip);

/* S5. Alg. 4 end to end, up to the integer output-layer sums: in_bits-bit unsigned inputs -> bit planes -> first
 * layer as weighted plane products -> Sign(BatchNorm) -> binary layers -> int32 logits of the last layer.
 * (With 8-bit inputs in 16-byte aligned rows the first layer may be evaluated as x . W_1 straight from the codes,
 * which Eq. (FirstLayer) states to be the same sum; the planes are then not materialised.  Only the low in_bits bits
 * of a code count.)
 * x: DEVICE uint8 [batch][in_dim], dense rows; in_dim must equal dims[0].
 * dims: HOST int64 [n_layers + 1] (dims[0] = input width).
 * W: HOST array of n_layers DEVICE pointers, W[l] packed +-1 [dims[l+1]][ceil(dims[l]/32)] (dense rows).
 * T, flip: HOST arrays of n_layers - 1 DEVICE pointers (flip, or any flip[l], may be NULL).
 * logits: DEVICE int32 [batch][ld_logits].  workspace: DEVICE, 256-byte aligned, at least
 * qnn_binary_mlp_workspace_bytes(...) bytes, contents undefined before and after.
 * 2 <= n_layers <= QNN_MAX_LAYERS, 1 <= in_bits <= 8.  Every layer is validated before the first launch, so an
 * argument error enqueues nothing. */
int qnn_binary_mlp_forward(const uint8_t *x, int64_t batch, int64_t in_dim, int in_bits, int n_layers,
                           const int64_t *dims, const uint32_t *const *W, const int32_t *const *T,
                           const uint8_t *const *flip, int32_t *logits, int64_t ld_logits, void *workspace,
                           size_t workspace_bytes, void *stream);
size_t qnn_binary_mlp_workspace_bytes(int64_t batch, int in_bits, int n_layers, const int64_t *dims);

/* Same forward pass with a row pitch for x (ldx >= dims[0], in bytes) and an engine preference: a layer that the
 * requested engine cannot take runs on the library's choice. */
int qnn_binary_mlp_forward_ex(const uint8_t *x, int64_t batch, int64_t ldx, int in_bits, int n_layers,
                              const int64_t *dims, const uint32_t *const *W, const int32_t *const *T,
                              const uint8_t *const *flip, int32_t *logits, int64_t ld_logits, void *workspace,
                              size_t workspace_bytes, int engine, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): qnn_binary_mlp_forward without the workspace argument.  The scratch memory is an array
 * of qnn_static_scratch_bytes() bytes (32 MiB) that is part of the library's code object; every GPU the library runs
 * on holds its own copy until the process ends.  The call allocates and frees nothing.  A network and batch whose
 * qnn_binary_mlp_workspace_bytes() exceeds the array is refused with QNN_ERR_WORKSPACE.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams or threads) race; calls ordered
 * on one stream do not.  Nothing in the array needs to be cleared between calls (every word that is read has been
 * written earlier in the same call). */
int qnn_binary_mlp_forward_static(const uint8_t *x, int64_t batch, int64_t in_dim, int in_bits, int n_layers,
                                  const int64_t *dims, const uint32_t *const *W, const int32_t *const *T,
                                  const uint8_t *const *flip, int32_t *logits, int64_t ld_logits, void *stream);
size_t qnn_static_scratch_bytes(void);

/* Binarized convolution (Sec. 5 filter bank M_l x M_{l-1} x k x k; Sec. 3 multi-bit activations) without
 * materialising patches.  Activations: Pa bit planes, channels-last and packed along channels:
 * plane i of pixel (b, y, x) is Cw = ceil(Cin/32) words at A + i * strideA_words + ((b*H + y)*Wd + x) * Cw.
 * Weights: Pb planes, filter co is [KH][KW][Cw] words at W + j * strideW_words + co * KH*KW*Cw.
 * Output: DEVICE int32 [B][Ho][Wo][Cout] dense, Ho = (H + 2 pad - KH) / stride + 1.
 * Padding pixels contribute exactly 0, which a bit-mode activation encodes as all-zero bits; a sign-mode activation
 * cannot encode 0, so modeA == QNN_PLANE_SIGN with pad > 0 is QNN_ERR_UNSUPPORTED.
 * H, Wd, pad, stride <= 32767; KH, KW <= 255. */
int qnn_bitplane_conv2d(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words,
                        int64_t B, int64_t H, int64_t Wd, int64_t Cin, const uint32_t *W, int Pb,
                        const int32_t *coefW, int modeW, int64_t strideW_words, int64_t Cout, int KH, int KW,
                        int pad, int stride_hw, int32_t *out, void *stream);

/* Same convolution with the engine chosen by the caller (for measurements and tests). */
int qnn_bitplane_conv2d_ex(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words,
                           int64_t B, int64_t H, int64_t Wd, int64_t Cin, const uint32_t *W, int Pb,
                           const int32_t *coefW, int modeW, int64_t strideW_words, int64_t Cout, int KH, int KW,
                           int pad, int stride_hw, int32_t *out, int engine, void *stream);

/* Convolution with Sign(BatchNorm(.)) fused (a layer of a binarized ConvNet, Alg. 4 with the filter banks of Sec. 5 and
 * App. A): bit[b][y][x][co] = (sum >= T[co]) xor flip[co], written packed along the output channels, which are the
 * next layer's input channels: out_bits is DEVICE uint32 [B][Ho][Wo][ceil(Cout/32)] dense, tail bits zero.
 * T: DEVICE int32 [Cout]; flip: DEVICE uint8 [Cout] or NULL.  Other arguments as qnn_bitplane_conv2d_ex. */
int qnn_bitplane_conv2d_sign(const uint32_t *A, int Pa, const int32_t *coefA, int modeA, int64_t strideA_words,
                             int64_t B, int64_t H, int64_t Wd, int64_t Cin, const uint32_t *W, int Pb,
                             const int32_t *coefW, int modeW, int64_t strideW_words, int64_t Cout, int KH, int KW,
                             int pad, int stride_hw, const int32_t *T, const uint8_t *flip, uint32_t *out_bits,
                             int engine, void *stream);

/* Alg. 4 for a binarized ConvNet of the shape of App. A (CIFAR-10 ConvNet table): n_conv 3 x 3 "same" convolutions
 * (zero padding, stride 1), layer l followed by 2 x 2 max-pooling if pool[l] != 0 (on the convolution's sums, before
 * BatchNorm, as in the table), each followed by Sign(BatchNorm(.)) as a folded threshold; then n_fc fully connected
 * layers on the feature map flattened in (y, x, c) order, the last one giving int32 sums.
 * x: DEVICE uint8 [B][H][W][C0], in_bits-bit inputs (first layer = weighted bit-plane products, Sec. 2.6).
 * cout, pool: HOST [n_conv]; fc_out: HOST [n_fc].  W: HOST array of n_conv + n_fc DEVICE pointers, packed +-1:
 * convolution l is [cout][3][3][ceil(cin/32)] words, fully connected j is [out][ceil(in/32)] (dense rows).
 * T, flip: HOST arrays of n_conv + n_fc - 1 DEVICE pointers (flip, or entries of it, may be NULL).
 * A padded position contributes exactly 0 to a convolution (it is not a -1).  The channels of the last feature map
 * must be a multiple of 32 unless that map is a single pixel (QNN_ERR_UNSUPPORTED otherwise).
 * logits: DEVICE int32 [B][ld_logits].  workspace: DEVICE, 256-byte aligned, qnn_binary_convnet_workspace_bytes(...)
 * bytes.  `engine` is a preference, as in qnn_binary_mlp_forward_ex.  Everything is validated before the first launch.
 * 1 <= n_conv, 1 <= n_fc, n_conv + n_fc <= 2 * QNN_MAX_LAYERS. */
int qnn_binary_convnet_forward(const uint8_t *x, int64_t B, int64_t H, int64_t Wd, int64_t C0, int in_bits, int n_conv,
                               const int64_t *cout, const int32_t *pool, int n_fc, const int64_t *fc_out,
                               const uint32_t *const *W, const int32_t *const *T, const uint8_t *const *flip,
                               int32_t *logits, int64_t ld_logits, void *workspace, size_t workspace_bytes, int engine,
                               void *stream);
size_t qnn_binary_convnet_workspace_bytes(int64_t B, int64_t H, int64_t Wd, int64_t C0, int in_bits, int n_conv,
                                          const int64_t *cout, const int32_t *pool, int n_fc, const int64_t *fc_out);

/* Linear quantization of Sec. 3, LinearQuant(x, step) = Clip(round(x / step) * step, minV, maxV), fused with the
 * bit-plane split of Sec. 2.6: the integer code q = Clip(round(x / step), qmin, qmax) (value = q * step, minV =
 * qmin * step, maxV = qmax * step) is written as nbits packed planes, plane p = bit p of q in two's complement
 * (for qmin >= 0 that is the unsigned code; coefficients 1, 2, 4, ... and, for signed codes, -2^(nbits-1) for the top
 * plane turn the planes back into q in qnn_bitplane_gemm).  The quotient is formed and rounded in single precision,
 * to the nearest integer with ties to even; NaN quantizes like 0.
 * x: DEVICE float32 [rows][ldx]; planes: DEVICE uint32, layout as in qnn_pack_bitplanes.  step > 0, finite;
 * qmin .. qmax must fit nbits (0 .. 2^nbits - 1, or -2^(nbits-1) .. 2^(nbits-1) - 1); 1 <= nbits <= 8. */
int qnn_linear_quant_planes(const float *x, int64_t rows, int64_t K, int64_t ldx, float step, int32_t qmin,
                            int32_t qmax, int nbits, uint32_t *planes, int64_t ld_words, int64_t plane_stride_words,
                            void *stream);

/* Logarithmic quantization of Sec. 3, LogQuant(x) = Clip(AP2(x), minV, maxV) with AP2(x) = sign(x) 2^round(log2 |x|)
 * (caption of Alg. 2) and magnitudes 2^emin .. 2^emax: what rounds below 2^emin (and 0, NaN) becomes 0, what rounds
 * above 2^emax is clipped to it.  Written as nbits packed planes of a two's-complement integer:
 *   as_value == 0: the signed code sign(x) * (e - emin + 1), e = min(round(log2 |x|), emax)   (0 = zero);
 *   as_value != 0: the quantized value in units of 2^emin, sign(x) * 2^(e - emin), which the bit-plane products
 *                  consume directly (coefficients 1, 2, ..., -2^(nbits-1)): this is how quantized gradients enter the
 *                  backward products (Sec. 5: quantized gradients let the backward pass use the bit-wise kernel).
 * gate: optional DEVICE float32 [rows][ld_gate] (NULL = none): where |gate| <= 1 does not hold the output is 0, the
 * straight-through estimator g o 1_{|a| <= 1} of Alg. 1 applied to the gradient before it is quantized.
 * emax - emin + 1 magnitudes must fit: < 2^(nbits-1) codes, or emax - emin + 1 <= nbits - 1 for values. */
int qnn_log_quant_planes(const float *x, const float *gate, int64_t rows, int64_t K, int64_t ldx, int64_t ld_gate,
                         int32_t emin, int32_t emax, int as_value, int nbits, uint32_t *planes, int64_t ld_words,
                         int64_t plane_stride_words, void *stream);

/* Inference-time BatchNorm of the output layer (Alg. 4, last line) in its affine form on the integer sums:
 * y[m][n] = scale[n] * sums[m][n] + shift[n] as one fused multiply-add in single precision.
 * sums: DEVICE int32 [M][ld_sums]; scale, shift: DEVICE float32 [N]; y: DEVICE float32 [M][ldy]. */
int qnn_batchnorm_affine(const int32_t *sums, int64_t ld_sums, int64_t M, int64_t N, const float *scale,
                         const float *shift, float *y, int64_t ldy, void *stream);

/* Transpose of packed bit matrices: in is nplanes planes of [rows][ld_in_words] holding `cols` bits per row; out
 * receives [cols][ld_out_words] holding `rows` bits per row (first ceil(rows/32) words written, tail bits zero).
 * The backward products of Alg. 1 reduce over the axis the forward pass did not pack along. */
int qnn_transpose_bits(const uint32_t *in, int64_t rows, int64_t cols, int64_t ld_in_words,
                       int64_t in_plane_stride_words, int nplanes, uint32_t *out, int64_t ld_out_words,
                       int64_t out_plane_stride_words, void *stream);

/* Backward products of Alg. 1 for one layer with binary weights, binary activations and integer gradients given
 * as bit planes (e.g. from qnn_log_quant_planes with as_value, or a linear code):
 *   gA[m][k] = sum_n g[m][n] w[n][k]   (g_{a_{k-1}^b} = g_{s_k} W_k^b),
 *   gW[n][k] = sum_m g[m][n] a[m][k]   (g_{W_k^b} = g_{s_k}^T a_{k-1}^b),
 * g = sum_p coefG[p] * plane_p (read according to modeG).  G: DEVICE, Pg planes of [M][ldg_words] packed along n;
 * W: DEVICE packed +-1 [N][ldw_words] (along k, as the forward pass holds it); A: DEVICE packed +-1 [M][lda_words].
 * gA: DEVICE int32 [M][ld_ga]; gW: DEVICE int32 [N][ld_gw].  coefG: HOST.  workspace: DEVICE, 256-byte aligned,
 * qnn_binary_backward_workspace_bytes(...) bytes (the transposed operands).  QNN_ERR_OVERFLOW if
 * (sum |coefG|) * max(M, N) >= 2^31. */
int qnn_binary_backward(const uint32_t *G, int Pg, const int32_t *coefG, int modeG, int64_t ldg_words,
                        int64_t strideG_words, const uint32_t *W, int64_t ldw_words, const uint32_t *A,
                        int64_t lda_words, int32_t *gA, int64_t ld_ga, int32_t *gW, int64_t ld_gw, int64_t M, int64_t N,
                        int64_t K, void *workspace, size_t workspace_bytes, void *stream);
size_t qnn_binary_backward_workspace_bytes(int64_t M, int64_t N, int64_t K, int Pg);

/* Convolution evaluated through the distinct 2-D filters of every input channel (Sec. 5: with binary weights the
 * 3 x 3 slices of a filter bank repeat; apply only the distinct ones, a slice and its negation counting as one, and
 * sum the responses into each 3-D filter's result).  Same result as qnn_bitplane_conv2d with 3 x 3 filters, stride 1,
 * bit-mode activation planes and one +-1 weight plane.  unique_count: DEVICE uint32 [Cin] or NULL, receives the
 * number of distinct 2-D filters of every input channel; their sum over Cout * Cin is the fraction of filter
 * applications that remains.  It states the method and measures that fraction; the direct product is the fast path.
 * A: Pa planes as in qnn_bitplane_conv2d; W: DEVICE packed +-1 [Cout][3][3][ceil(Cin/32)]; out: DEVICE int32
 * [B][Ho][Wo][Cout].  workspace: DEVICE, 256-byte aligned, at least qnn_conv2d_dedup_workspace_bytes(...) bytes (more
 * lets the call take several images at a time).  9 * sum|coefA| <= 32767; Cout <= 32767. */
int qnn_conv2d_dedup(const uint32_t *A, int Pa, const int32_t *coefA, int64_t strideA_words, int64_t B, int64_t H,
                     int64_t Wd, int64_t Cin, const uint32_t *W, int64_t Cout, int pad, int32_t *out,
                     uint32_t *unique_count, void *workspace, size_t workspace_bytes, void *stream);
size_t qnn_conv2d_dedup_workspace_bytes(int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout, int pad);

/* Engine (QNN_ENGINE_VALU, QNN_ENGINE_MFMA or QNN_ENGINE_MFMA_FP4) that the calling thread's last successful multiply call used; 0 before
 * any.  For reports: results never depend on it. */
int qnn_last_engine(void);

/* Engines of the multiply launches made by the calling thread's last successful multiply / forward call, in launch
 * order (one entry per layer for the forward calls): writes min(count, capacity) entries, returns the count. */
int qnn_last_engines(int *engines, int capacity);

/* Measurement helper, not a step of the path: one wave spins for a few microseconds and writes to
 * out3 (DEVICE, three uint64, 8-byte aligned) {elapsed shader-clock cycles, elapsed ticks of the constant 100 MHz
 * real-time counter, a checksum}; 100 * out3[0] / out3[1] is the shader clock in MHz at that moment. */
int qnn_probe_shader_clock(unsigned long long *out3, void *stream);

/* Measurement helper: one wave writes to out3 (DEVICE, three uint64, 8-byte aligned) {shader-clock counter, 100 MHz
 * real-time counter, id of the accelerator die it ran on}, in stream order.  Two stamps around a stretch of work on
 * one stream, taken on the same die, give the average shader clock over that stretch. */
int qnn_stamp_clocks(unsigned long long *out3, void *stream);

/* Measurement helper: the rate of the vector ALU on the inner product of the vector-ALU engine (Sec. 6, Eq. (popc):
 * one xor and one popcount-accumulate per 32 connections) with all operands in registers.  `blocks` workgroups of 256
 * lanes run `iterations` times sixteen such pairs per lane, i.e. blocks * 256 * iterations * 16 * 32 MACs; sink
 * (DEVICE, blocks * 256 uint32) receives one checksum per lane.  The caller times the launch.  blocks in 1 .. 65536. */
int qnn_probe_valu_peak(uint32_t *sink, int64_t blocks, uint32_t iterations, void *stream);

/* Measurement helper: the rate the matrix cores sustain on the instruction of the FP4 path with all operands in
 * registers.  `blocks` workgroups of four waves (one per SIMD) run `iterations` times sixteen
 * v_mfma_scale_f32_32x32x64_f8f6f4 per wave, i.e. blocks * 4 * iterations * 16 * 65536 MACs.  Every operand register
 * holds operand_bits, and-ed with a per-lane hash if vary is non-zero (E2M1 nibbles: 0 all zeros, 0x22222222 all ones,
 * 0x22222222 with vary zeros and ones at random, 0xFFFFFFFF with vary random values).  sink (DEVICE, blocks * 256 float) receives one checksum per lane.  The caller times the
 * launch.  blocks in 1 .. 65536. */
int qnn_probe_mfma_fp4_peak(float *sink, int64_t blocks, uint32_t iterations, uint32_t operand_bits, int vary, void *stream);

const char *qnn_last_error(void);
const char *qnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QNN_H */
