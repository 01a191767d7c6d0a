// Matrix-core engine of the binary / bit-plane matrix product: host side (operand codes, epilogue constants, choice of
// the kernel instantiation, launch).  The kernel itself is in qnn_gemm_mfma_kernel.h.

#include "qnn_gemm_mfma_kernel.h"
#include "qnn_gemm_bytes_panel_kernel.h"
#include "qnn_gemm_panel_kernel.h"
#include "qnn_gemm_stage_kernel.h"

namespace qnn {

using namespace mfma;

namespace {

// Derives the int8 code of one operand; false if its coefficients do not fit (then the vector-ALU engine is used).
bool make_code(const Planes &pl, Code &c, int64_t &alpha, int64_t &beta, int64_t &x_pad) {
    const int P = pl.count;
    int64_t gcd = 0;
    for (int p = 0; p < P; ++p) {
        int64_t a = pl.coef[p] < 0 ? -(int64_t)pl.coef[p] : pl.coef[p];
        if (a == 0) return false;
        int64_t x = gcd, y = a;
        while (y) {
            int64_t t = x % y;
            x = y;
            y = t;
        }
        gcd = x;
    }
    if (P == 1 && pl.coef[0] < 0) gcd = -gcd;  // a single plane keeps its bit as it is; the sign goes into alpha
    uint32_t used = 0;
    int64_t U = 0, neg = 0, sum_c = 0;
    for (int p = 0; p < P; ++p) {
        const int64_t d = pl.coef[p] / gcd;
        const int64_t ad = d < 0 ? -d : d;
        if (ad > 128 || (ad & (ad - 1)) != 0) return false;  // power of two up to 128
        int lg = 0;
        while ((1 << lg) < ad) ++lg;
        if (used & (1u << lg)) return false;  // positions must be distinct for the OR
        used |= 1u << lg;
        c.lg[p] = lg;
        c.inv[p] = d < 0 ? 0xFFFFFFFFu : 0u;
        c.d[p] = (int32_t)d;
        U += ad;
        if (d < 0) neg += ad;
        sum_c += pl.coef[p];
    }
    for (int p = P; p < QNN_MAX_PLANES; ++p) c.lg[p] = 0, c.inv[p] = 0, c.d[p] = 0;
    const int64_t offp = U > 127 ? 128 : 0;
    c.bias = offp ? 0x80808080u : 0u;
    const int64_t off = offp - neg;  // x8 = sum_p d_p b_p - off
    if (pl.mode == QNN_PLANE_BIT) {
        alpha = gcd;
        beta = gcd * off;
    } else {
        alpha = 2 * gcd;
        beta = 2 * gcd * off - sum_c;
    }
    x_pad = -off;
    return true;
}


// Epilogue constants of C = aA aW (S - npad xA0 xW0) + aA bW RA[m] + bA aW RW[n] + K bA bW for a kernel that processes
// Kproc >= K elements per row (the surplus reads as zero bits); false if the sums could leave the exact range.
bool fill_consts(const GemmArgs &g, int64_t aA, int64_t bA, int64_t xA0, int64_t aW, int64_t bW, int64_t xW0,
                 int64_t Kproc, MfmaConst &mc) {
    if (g.epi.T) {
        // the threshold epilogue compares through differences, which must not wrap: |C| < 2^30
        long double bound = (long double)g.K;
        long double sa = 0, sw = 0;
        for (int p = 0; p < g.pa.count; ++p) sa += g.pa.coef[p] < 0 ? -(long double)g.pa.coef[p] : g.pa.coef[p];
        for (int p = 0; p < g.pw.count; ++p) sw += g.pw.coef[p] < 0 ? -(long double)g.pw.coef[p] : g.pw.coef[p];
        if (bound * sa * sw >= 1073741824.0L) return false;
    }
    if (Kproc >= 131072) return false;  // |S| <= Kproc * 2^14 must stay below 2^31
    const int64_t npad = Kproc - g.K;
    mc.msteps = 0;
    mc.alpha = (uint32_t)(aA * aW);
    mc.cRA = (uint32_t)(aA * bW);
    mc.cRW = (uint32_t)(bA * aW);
    mc.c0 = (uint32_t)(g.K * bA * bW - aA * aW * npad * xA0 * xW0);
    mc.needRW = mc.cRW != 0;
    // the row sums are over the true K: RA = sum_p d_p pop_p - K * off; fold the constant part into c0
    mc.c0 += (uint32_t)(aA * bW * (g.K * xA0)) + (uint32_t)(bA * aW * (g.K * xW0));
    mc.alpha_shift = -1;
    for (int sh = 0; sh < 31; ++sh)
        if (aA * aW == ((int64_t)1 << sh)) mc.alpha_shift = sh;
    return true;
}

const Variant *find_variant(const GemmArgs &g) {
    const bool pixels = g.A.rows_are_pixels != 0, sign = g.epi.T != nullptr;
    const VariantList lists[] = {variants_fp4(), variants_first_layer(), variants_multibit(), variants_conv(),
                                   variants_conv_sign()};
    for (const VariantList &l : lists)
        for (int i = 0; i < l.n; ++i) {
            const Variant &v = l.v[i];
            if (v.PA == g.pa.count && v.PW == g.pw.count && v.pixels == pixels && v.sign == sign) return &v;
        }
    return nullptr;
}

bool prepare(const GemmArgs &g, bool fp4, const Variant *&var, MfmaConst &mc, bool &vec) {
    static const Variant kBytes = {0, 1, 1, false, false, nullptr, nullptr, nullptr, nullptr};
    const bool bytes = g.A.rows_are_bytes != 0;
    int64_t aA, bA, xA0, aW, bW, xW0;
    if (bytes) {
        // x8 = code - 128, true value = x8 + 128; rows of 16-byte aligned chunks only
        if (fp4 || g.pw.count != 1 || g.K % 16 || g.A.ld % 16 || reinterpret_cast<uintptr_t>(g.A.base) % 16) return false;
        var = &kBytes;
        std::memset(&mc.a, 0, sizeof(mc.a));
        aA = 1, bA = 128, xA0 = 0;
        if (!make_code(g.pw, mc.w, aW, bW, xW0)) return false;
    } else {
        var = find_variant(g);
        if (!var) return false;
        if (fp4 && !var->fp4_vec) return false;
        if (!make_code(g.pa, mc.a, aA, bA, xA0) || !make_code(g.pw, mc.w, aW, bW, xW0)) return false;
    }
    const int64_t step_words = 2 * var->WPL;
    const int64_t msteps = 2 * ceil_div(g.Kw, 2 * step_words);
    if (!fill_consts(g, aA, bA, xA0, aW, bW, xW0, msteps * step_words * 32, mc)) return false;
    mc.msteps = (uint32_t)msteps;
    // vector loads need every row (of every plane) to start at a multiple of the load width and to be made of whole
    // chunks, so that a chunk is either all inside or all outside the row
    const int wpl = var->WPL;
    auto aligned = [&](const uint32_t *base, int64_t ld, int64_t pstride, int planes) __attribute__((always_inline)) {
        if (reinterpret_cast<uintptr_t>(base) % (4 * wpl)) return false;
        if (planes > 1 && pstride % wpl) return false;
        return ld % wpl == 0;
    };
    const bool pix = g.A.rows_are_pixels != 0;
    vec = !bytes && wpl > 1 && aligned(g.A.base, pix ? g.A.Cw : g.A.ld, g.A.plane_stride, g.pa.count) &&
          aligned(g.W, g.ldw, g.strideW, g.pw.count) && (pix ? g.A.Cw % wpl == 0 : true) && g.Kw % wpl == 0;
    return true;
}

}  // namespace

bool mfma_supports(const GemmArgs &g, bool fp4) {
    const Variant *v;
    MfmaConst mc;
    bool vec;
    return prepare(g, fp4, v, mc, vec);
}

bool mfma_preferred(const GemmArgs &g) {
    // small or skinny products (a 10-neuron output layer fills 10 of a tile's 256 columns) are better served by the
    // finer tiles of the vector-ALU engine
    if (ceil_div(g.M, BM) * ceil_div(g.N, BN) >= 32 && g.K >= 256 && g.M >= 128 && g.N >= 128) return true;
    // single planes with long rows: a few matrix-core tiles beat many vector-ALU tiles (a fully connected layer of 8192
    // inputs on a batch of 256: 27 us on eight 256 x 128 tiles against 41 us on sixty-four 64 x 64 tiles)
    return g.pa.count == 1 && g.pw.count == 1 && !g.A.rows_are_pixels && !g.A.rows_are_bytes && g.K >= 4096 && g.M >= 256 &&
           g.N >= 256;
}

static int compute_units() {
    static thread_local int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus = n;
    }
    return cus;
}

int launch_gemm_mfma(const GemmArgs &g, hipStream_t s, bool fp4) {
    const Variant *v;
    MfmaConst mc;
    bool vec;
    if (!prepare(g, fp4, v, mc, vec)) return fail(QNN_ERR_UNSUPPORTED, "matrix-core engine cannot take these arguments");
    const int64_t tiles_m = ceil_div(g.M, BM), tiles_n = ceil_div(g.N, BN);
    if (tiles_m * tiles_n > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "gemm: too many tiles");
    // one persistent workgroup per compute unit (each takes 512 registers per lane, so one fits)
    const int cus = compute_units();
    const int64_t total = tiles_m * tiles_n;
    const unsigned grid = (unsigned)(total < cus ? total : cus);
    // single-plane products on the FP4 path whose rows are made of whole, aligned 16-byte groups: the panel-fed kernel
    // (row offsets are 32-bit and formed for up to one tile beyond the last row before they are clamped)
    const bool spans32 = 4.0L * (long double)(g.M + 256) * g.A.ld < 4294967296.0L && 4.0L * (long double)(g.N + 256) * g.ldw < 4294967296.0L;
    if (fp4 && vec && spans32 && !g.A.rows_are_pixels && !g.A.rows_are_bytes && v->WPL == 4 &&
        g.Kw % panel::kGroupWords == 0) {
        const int64_t ngroups = ceil_div(g.Kw, panel::kGroupWords);
        int64_t aA, bA, xA0, aW, bW, xW0;
        MfmaConst pc = mc;
        if (make_code(g.pa, pc.a, aA, bA, xA0) && make_code(g.pw, pc.w, aW, bW, xW0) &&
            fill_consts(g, aA, bA, xA0, aW, bW, xW0, ngroups * panel::kGroupWords * 32, pc)) {
            // Tile schedule by cost, in units of a round of 256 x 128 tiles: a round of 256 x 256 tiles costs 1.86 with
            // long rows (measured at K = 4096) and two with short ones, where the epilogue dominates.  The rounds count
            // whole tiles, so the padding of a ragged edge (128 columns under 256-column tiles: half of every tile) and
            // a thinly filled last round both show.  Third schedule: wide tiles with the last round's tiles halved
            // (each half to a workgroup of its own, 1.17 for that round), possible when that round has tiles for at most
            // half of the workgroups and worth it only for long rows.
            const int64_t tiles_n2 = ceil_div(g.N, BN / 2);
            const double wide_round = ngroups >= 4 ? 1.86 : 2.0, half_round = 1.17;
            const double cost_wide = (double)ceil_div(total, cus) * wide_round;
            const double cost_narrow = (double)ceil_div(tiles_m * tiles_n2, cus);
            bool narrow = cost_narrow < cost_wide;
            bool tail = false;
            if (cus % 16 == 0 && total > cus && total % cus != 0 && 2 * (total % cus) <= cus && ngroups >= 4) {
                const double cost_tail = (double)(total / cus) * wide_round + half_round;
                tail = cost_tail < (narrow ? cost_narrow : cost_wide);
            }
            narrow = narrow && !tail;
            const panel::KernelFn pf = panel::find_kernel(g.epi.T != nullptr, narrow, tail);
            const int64_t ptotal = narrow ? tiles_m * tiles_n2 : total;
            const unsigned pgrid = (unsigned)(ptotal < cus ? ptotal : cus);
            return QNN_LAUNCH("gemm_panel", pf, dim3(pgrid), dim3(panel::kThreads), 0, s, g, pc, (uint32_t)tiles_m,
                              (uint32_t)(narrow ? tiles_n2 : tiles_n), (uint32_t)ngroups);
        }
    }
    // uint8 left operand with the weights expanded to bytes beforehand: the panel-fed kernel (threshold epilogue)
    if (g.A.rows_are_bytes && g.w_bytes && g.rw_scaled && g.epi.T && (long double)g.M * g.A.ld < 4294967296.0L &&
        (long double)g.N * g.ld_w_bytes < 4294967296.0L && g.ld_w_bytes % bytes_panel::kGroupK == 0 && g.ld_w_bytes >= g.K) {
        MfmaConst pc = mc;
        pc.alpha = 1, pc.alpha_shift = 0, pc.cRA = 0, pc.cRW = 1, pc.c0 = 0, pc.needRW = 1;
        const int64_t ngroups = ceil_div(g.K, bytes_panel::kGroupK);
        // 256 x 128 tiles where they fill the rounds of workgroups clearly better than 256 x 256 ones
        auto fill = [&](int64_t tiles) { return (double)tiles / (double)(ceil_div(tiles, cus) * cus); };
        const int64_t wide_n = ceil_div(g.N, 256), narrow_n = ceil_div(g.N, 128);
        const bool narrow = fill(tiles_m * narrow_n) > 1.1 * fill(tiles_m * wide_n);
        const int64_t tiles_nb = narrow ? narrow_n : wide_n, ptotal = tiles_m * tiles_nb;
        if (ptotal <= 0x7FFFFFFFLL) {
            const unsigned pgrid = (unsigned)(ptotal < cus ? ptotal : cus);
            return QNN_LAUNCH("gemm_bytes_panel", bytes_panel::kernel(narrow), dim3(pgrid), dim3(bytes_panel::kThreads), 0, s, g, pc,
                              (uint32_t)tiles_m, (uint32_t)tiles_nb, (uint32_t)ngroups);
        }
    }
    const KernelFn fn = g.A.rows_are_bytes ? byte_kernels()[g.epi.T ? 1 : 0]
                        : fp4              ? (vec ? v->fp4_vec : v->fp4_any)
                                           : (vec ? v->fn_vec : v->fn_any);
    return QNN_LAUNCH("gemm_mfma", fn, dim3(grid), dim3(kThreads), 0, s, g, mc, (uint32_t)tiles_m,
                       (uint32_t)tiles_n);
}

// ------------------------------------------------------------------------------------------------ convolution on the panel-fed kernel
bool conv_panel_supports(int64_t B, int64_t H, int64_t Wd, int64_t C, int64_t N) {
    // (at least two rows and columns: a pixel is then in one of three row classes and one of three column classes)
    if (B < 1 || H < 2 || Wd < 2 || H > 32767 || Wd > 32767 || C < 128 || C % 128 || N < 1) return false;
    if (16 * conv_panel_class_ld(N) >= (1 << 28)) return false;  // 32-bit byte offsets into the class table
    const int64_t cpt = C / 128;
    if (cpt & (cpt - 1)) return false;
    const int64_t M = B * H * Wd, Cw = C / 32;
    if (M < 256 || M > 0x7FFFFFFFLL) return false;
    // 32-bit byte offsets: the plane (plus the distance to the line of zeros, checked at the launch) and the weights
    if ((long double)(M + 256) * Cw * 4 >= 2147483648.0L || (long double)(N + 256) * 9 * Cw * 4 >= 4294967296.0L) return false;
    return ceil_div(M, 256) * ceil_div(N, 128) <= 0x7FFFFFFFLL;
}

int64_t conv_panel_class_ld(int64_t N) { return ceil_div(N, 128) * 128; }

int launch_conv_panel(const uint32_t *plane, int64_t B, int H, int Wd, int C, const uint32_t *W, int64_t N, const int32_t *T,
                      const uint8_t *flip_complement, uint32_t *out, int64_t ldo, const int32_t *class_thr,
                      const uint32_t *zero_line, hipStream_t s) {
    if (!conv_panel_supports(B, H, Wd, C, N)) return fail(QNN_ERR_UNSUPPORTED, "convolution on the panel-fed kernel: shape not supported");
    const int Cw = C / 32;
    const int64_t M = B * H * Wd, ld = conv_panel_class_ld(N);
    const uint8_t *pa = reinterpret_cast<const uint8_t *>(plane), *pz = reinterpret_cast<const uint8_t *>(zero_line);
    const uint8_t *base = pa < pz ? pa : pz;
    const uint64_t a_delta = (uint64_t)(pa - base), z_off = (uint64_t)(pz - base);
    if (a_delta + (uint64_t)(M + 256) * Cw * 4 >= 4294967296ULL || z_off + 256 >= 4294967296ULL)
        return fail(QNN_ERR_UNSUPPORTED, "convolution on the panel-fed kernel: scratch too far from the feature map");
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A.base = reinterpret_cast<const uint32_t *>(base);
    g.A.ld = Cw, g.A.rows_are_pixels = 1;
    g.A.H = H, g.A.Wd = Wd, g.A.Ho = H, g.A.Wo = Wd, g.A.Cw = Cw, g.A.KH = 3, g.A.KW = 3, g.A.pad = 1, g.A.stride = 1;
    g.pa.count = 1, g.pa.mode = QNN_PLANE_BIT, g.pa.coef[0] = 1;
    g.W = W, g.ldw = 9 * Cw, g.pw.count = 1, g.pw.mode = QNN_PLANE_BIT, g.pw.coef[0] = 1;
    g.epi.T = T, g.epi.flip = flip_complement, g.epi.out_bits = out, g.epi.ldo = ldo;
    g.M = M, g.N = N, g.K = 9 * (int64_t)C, g.Kw = 9 * Cw;
    g.class_thr = class_thr, g.class_ld = ld;
    g.a_delta = (uint32_t)a_delta, g.zero_off = (uint32_t)z_off;
    g.inv_w = 1.0 / (double)Wd, g.inv_hw = 1.0 / ((double)H * (double)Wd);
    int sh = 0;
    while ((1 << sh) < C / 128) ++sh;
    g.cpt_shift = sh;
    g.last_steps = (int)ceil_div(g.Kw - (ceil_div(g.Kw, panel::kGroupWords) - 1) * panel::kGroupWords, 8);
    MfmaConst mc;
    std::memset(&mc, 0, sizeof(mc));
    mc.alpha = 1u;  // (the convolution's epilogue compares the sums as they are)
    const int64_t tiles_m = ceil_div(M, 256), tiles_n = ceil_div(N, 128), total = tiles_m * tiles_n;
    const int cus = compute_units();
    const unsigned grid = (unsigned)(total < cus ? total : cus);
    return QNN_LAUNCH("conv_panel", panel::conv_kernel(), dim3(grid), dim3(panel::kThreads), 0, s, g, mc, (uint32_t)tiles_m,
                      (uint32_t)tiles_n, (uint32_t)ceil_div(g.Kw, panel::kGroupWords));
}

// ------------------------------------------------------------------------------------------------ staged kernels
namespace {

using stage::StageConst;
typedef void (*StageFn)(const GemmArgs, const MfmaConst, const StageConst, uint32_t, uint32_t);

// One operand for the merge network: bit position q of the code comes from plane order[q]; false if the positions
// are not exactly 0 .. P-1 or the plane count has no network.
bool stage_operand(const Planes &pl, const Code &c, int64_t plane_stride, int64_t (&off)[QNN_MAX_PLANES],
                   uint32_t (&inv)[QNN_MAX_PLANES], int32_t (&d)[QNN_MAX_PLANES]) {
    const int P = pl.count;
    if (P != 1 && P != 2 && P != 4 && P != 8) return false;
    for (int q = 0; q < QNN_MAX_PLANES; ++q) off[q] = 0, inv[q] = 0, d[q] = 0;
    uint32_t seen = 0;
    for (int p = 0; p < P; ++p) {
        const int q = c.lg[p];
        if (q < 0 || q >= P || (seen & (1u << q))) return false;
        seen |= 1u << q;
        off[q] = (int64_t)p * plane_stride;
        inv[q] = c.inv[p];
        d[q] = c.d[p];
    }
    return true;
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

bool prepare_stage(const GemmArgs &g, MfmaConst &mc, StageConst &sc, StageFn &fn) {
    const bool pix = g.A.rows_are_pixels != 0, sign = g.epi.T != nullptr;
    if (g.A.rows_are_bytes) return false;
    std::memset(&sc, 0, sizeof(sc));
    int64_t aA, bA, xA0, aW, bW, xW0;
    if (!make_code(g.pa, mc.a, aA, bA, xA0) || !make_code(g.pw, mc.w, aW, bW, xW0)) return false;
    if (!stage_operand(g.pa, mc.a, g.A.plane_stride, sc.offA, sc.invA, sc.dA)) return false;
    if (!stage_operand(g.pw, mc.w, g.strideW, sc.offW, sc.invW, sc.dW)) return false;
    sc.biasA = mc.a.bias, sc.biasW = mc.w.bias;
    // 16-byte loads: every row of every plane starts on a 16-byte boundary and holds whole groups of four words
    const bool w_vec = aligned16(g.W) && g.ldw % 4 == 0 && (g.pw.count == 1 || g.strideW % 4 == 0) && g.Kw % 4 == 0;
    const bool a_vec = aligned16(g.A.base) && (g.pa.count == 1 || g.A.plane_stride % 4 == 0) &&
                       (pix ? g.A.Cw % 4 == 0 : (g.A.ld % 4 == 0 && g.Kw % 4 == 0));
    if (!a_vec || !w_vec) return false;
    // the kernel addresses rows with 32-bit offsets from a plane's base
    const long double a_span = pix ? 4.0L * (long double)g.M / ((long double)g.A.Ho * g.A.Wo) * g.A.H * g.A.Wd * g.A.Cw
                                   : 4.0L * (long double)g.M * g.A.ld;
    if (a_span >= 4294967296.0L || 4.0L * (long double)g.N * g.ldw >= 4294967296.0L) return false;
    const int64_t nmacro = ceil_div(g.Kw, 4);
    sc.nmacro = (uint32_t)nmacro;
    if (!fill_consts(g, aA, bA, xA0, aW, bW, xW0, nmacro * 4 * 32, mc)) return false;
    fn = stage::find_kernel(g.pa.count, g.pw.count, pix ? stage::kPixelPlanes : stage::kPlanes, sign);
    return fn != nullptr;
}

// Large products of multi-plane operands with int32 output: the planes of both operands are merged to int8 values once
// per call, into memory borrowed from the stream's pool, and the panel-fed byte kernel multiplies them.  (Merging in
// every workgroup repeats the work for every tile of a row of tiles and holds the multiplication up behind loads of
// one row per lane.)
// Row pitch of the merged operands: whole groups of k.
int64_t values_pitch(int64_t K) {
    const int64_t p = ceil_div(K, bytes_panel::kGroupK) * bytes_panel::kGroupK;
    return p;
}
bool values_path(const GemmArgs &g) {
    if (g.A.rows_are_pixels || g.A.rows_are_bytes || g.epi.T) return false;
    if (g.pa.count == 1 && g.pw.count == 1) return false;
    if (g.K < 512 || g.K >= 131072 || g.M < 256 || g.N < 256) return false;  // |S| <= K 2^14 stays below 2^31
    if ((long double)g.M * (long double)g.N * (long double)g.K < 2147483648.0L) return false;  // small: not worth three launches
    const int64_t pitch = values_pitch(g.K);
    if ((long double)(g.M + 256) * pitch >= 4294967296.0L || (long double)(g.N + 256) * pitch >= 4294967296.0L) return false;
    if (ceil_div(g.M, 256) * ceil_div(g.N, 128) > 0x7FFFFFFFLL) return false;
    return bytes_panel::merge_supports(g.pa, g.pw);
}

int launch_values(const GemmArgs &g, hipStream_t s) {
    const int64_t pitch = values_pitch(g.K);
    const size_t bytes_a = (size_t)g.M * (size_t)pitch, bytes_w = (size_t)g.N * (size_t)pitch;
    void *mem = nullptr;
    if (hipMallocAsync(&mem, bytes_a + bytes_w, s) != hipSuccess || !mem) {
        (void)hipGetLastError();
        return fail(QNN_ERR_HIP, "gemm: no memory for the merged operands (%zu bytes)", bytes_a + bytes_w);
    }
    int8_t *a8 = static_cast<int8_t *>(mem), *w8 = a8 + bytes_a;  // (bytes_a is a multiple of 128)
    int64_t scale = 0;
    int rc = bytes_panel::launch_merge_planes(g, a8, w8, pitch, scale, s);
    if (rc == QNN_OK) {
        GemmArgs v = g;
        v.A.base = reinterpret_cast<const uint32_t *>(a8);
        v.A.ld = pitch;
        v.A.plane_stride = 0;
        v.A.rows_are_bytes = 1;
        v.w_bytes = w8;
        v.ld_w_bytes = pitch;
        v.rw_scaled = nullptr;
        MfmaConst mc;
        std::memset(&mc, 0, sizeof(mc));
        mc.alpha = (uint32_t)scale;
        mc.alpha_shift = -1;
        for (int sh = 0; sh < 31; ++sh)
            if (scale == ((int64_t)1 << sh)) mc.alpha_shift = sh;
        const int cus = compute_units();
        const int64_t tiles_m = ceil_div(g.M, 256);
        const int64_t wide_n = ceil_div(g.N, 256), narrow_n = ceil_div(g.N, 128);
        // The narrow tile has room for three group buffers and keeps more bytes on their way from memory, which is what
        // bounds this kernel (a byte per element, eight times the traffic of packed bits): the wide tile only where its
        // tiles come out cheaper by a count of rounds of whole tiles (a round of wide tiles = 1.9 rounds of narrow ones),
        // which sees padded columns as well as thin last rounds.
        const bool narrow = tiles_m * wide_n < cus ||
                            (double)ceil_div(tiles_m * narrow_n, cus) <= 1.9 * (double)ceil_div(tiles_m * wide_n, cus);
        const int64_t tiles_n = narrow ? narrow_n : wide_n, total = tiles_m * tiles_n;
        const unsigned grid = (unsigned)(total < cus ? total : cus);
        rc = QNN_LAUNCH("gemm_values", bytes_panel::kernel_values(narrow), dim3(grid), dim3(bytes_panel::kThreads), 0, s, v, mc,
                        (uint32_t)tiles_m, (uint32_t)tiles_n, (uint32_t)ceil_div(g.K, bytes_panel::kGroupK));
    }
    if (hipFreeAsync(mem, s) != hipSuccess) {
        (void)hipGetLastError();
        if (rc == QNN_OK) rc = fail(QNN_ERR_HIP, "gemm: returning the merged operands' memory failed");
    }
    return rc;
}

}  // namespace

bool stage_supports(const GemmArgs &g) {
    if (values_path(g)) return true;
    MfmaConst mc;
    StageConst sc;
    StageFn fn;
    return prepare_stage(g, mc, sc, fn);
}

int launch_gemm_stage(const GemmArgs &g, hipStream_t s) {
    if (values_path(g)) return launch_values(g, s);
    MfmaConst mc;
    StageConst sc;
    StageFn fn;
    if (!prepare_stage(g, mc, sc, fn))
        return fail(QNN_ERR_UNSUPPORTED, "staged matrix-core kernels cannot take these arguments");
    const int64_t tiles_m = ceil_div(g.M, 256), tiles_n = ceil_div(g.N, 256);
    if (tiles_m * tiles_n > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "gemm: too many tiles");
    const int64_t total = tiles_m * tiles_n;
    const int cus = compute_units();
    const unsigned grid = (unsigned)(total < cus ? total : cus);
    return QNN_LAUNCH("gemm_stage", fn, dim3(grid), dim3(stage::kThreads), 0, s, g, mc, sc, (uint32_t)tiles_m,
                      (uint32_t)tiles_n);
}

}  // namespace qnn
