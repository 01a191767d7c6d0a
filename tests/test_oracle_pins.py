"""Pins of the CPU oracle against things other than itself: the paper's definitions worked by hand (tests/golden),
library routines (fp32 / fp64 matmul and convolution, numpy.packbits), closed forms and brute force.
None of these tests touches the HIP library."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_rows(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows.setdefault(parts[0], []).append(parts[1:])
    return rows


# ---------------------------------------------------------------- sign / pack (Sec. 2.1 Eq. (1), Sec. 6)
def test_sign_edge_values_golden():
    bits, want = [], []
    with open(os.path.join(GOLDEN, "sign_edge_values.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            h, s = line.split()[:2]
            bits.append(int(h, 16))
            want.append(int(s))
    x = np.array(bits, dtype=np.uint32).view(np.float32)
    got = oracle.sign(x)
    assert got.tolist() == want
    # the generator's edge-value list is the same set of patterns (first 17 rows of the fixture)
    assert np.array_equal(qi.special_floats().view(np.uint32), np.array(bits[:17], dtype=np.uint32))


def test_sign_matches_library_compare(seed):
    x = qi.with_special_floats(qi.normal_f32(seed, 1, (37, 61)), seed, 2)
    want = torch.where(torch.from_numpy(x) >= 0, 1, -1).to(torch.int8).numpy()
    assert np.array_equal(oracle.sign(x), want)
    assert abs(float(oracle.sign(qi.normal_f32(seed, 3, (200000,))).mean())) < 0.01


@pytest.mark.parametrize("K", [1, 5, 31, 32, 33, 63, 64, 65, 100, 784])
def test_pack_bits_matches_numpy_packbits(seed, K):
    s = qi.pm1(seed, 100 + K, (7, K))
    got = oracle.pack_bits(s)
    Kw = (K + 31) // 32
    padded = np.zeros((7, Kw * 32), dtype=np.uint8)
    padded[:, :K] = s > 0
    want = np.packbits(padded, axis=1, bitorder="little").view("<u4")
    assert got.dtype == np.uint32 and got.shape == (7, Kw)
    assert np.array_equal(got, want)
    # tail bits are zero and the packing is invertible
    un = np.unpackbits(got.view(np.uint8), axis=1, bitorder="little")
    assert not un[:, K:].any()
    assert np.array_equal(2 * un[:, :K].astype(np.int8) - 1, s)


def test_pack_bits_single_positions():
    for t in [0, 1, 31, 32, 45, 63]:
        s = -np.ones((1, 64), dtype=np.int8)
        s[0, t] = 1
        w = oracle.pack_bits(s)[0]
        assert int(w[t // 32]) == 1 << (t % 32) and int(w[1 - t // 32]) == 0


# ---------------------------------------------------------------- +-1 GEMM (Alg. 4, Sec. 6)
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 31), (17, 9, 64), (33, 40, 1000), (128, 1024, 1024)])
def test_gemm_pm1_equals_fp32_gemm(seed, M, N, K):
    a = qi.pm1(seed, 10, (M, K))
    w = qi.pm1(seed, 11, (N, K))
    want = (torch.from_numpy(a).float() @ torch.from_numpy(w).float().T).numpy()  # exact: K < 2^24
    got = oracle.gemm_pm1(a, w)
    assert got.dtype == np.int32
    assert np.array_equal(got.astype(np.float32), want)


def test_gemm_pm1_is_not_symmetric_in_its_operands(seed):
    # a transposed/ swapped operand would pass a square symmetric test: use M != N and check one entry by hand
    a = qi.pm1(seed, 12, (2, 6))
    w = qi.pm1(seed, 13, (3, 6))
    got = oracle.gemm_pm1(a, w)
    assert got.shape == (2, 3)
    for m in range(2):
        for n in range(3):
            assert got[m, n] == sum(int(a[m, k]) * int(w[n, k]) for k in range(6))


def test_gemm_pm1_closed_forms(seed):
    K = 77
    a = qi.pm1(seed, 14, (9, K))
    ones = np.ones((1, K), dtype=np.int8)
    assert np.array_equal(oracle.gemm_pm1(a, ones)[:, 0], a.astype(np.int64).sum(axis=1))
    g = oracle.gemm_pm1(a, a)
    assert np.array_equal(np.diag(g), np.full(9, K))
    assert np.array_equal(np.diag(oracle.gemm_pm1(a, -a)), np.full(9, -K))
    assert np.array_equal(g, g.T)
    assert ((g - K) % 2 == 0).all()  # every +-1 dot product has the parity of K


@pytest.mark.parametrize("K", [1, 2, 7, 10])
def test_gemm_pm1_brute_force_all_sign_vectors(seed, K):
    w = qi.pm1(seed, 15, (1, K))
    wbits = sum(1 << t for t in range(K) if w[0, t] > 0)
    allv = np.array(list(itertools.product([-1, 1], repeat=K)), dtype=np.int8)  # 2^K x K
    got = oracle.gemm_pm1(allv, w)[:, 0]
    for row, g in zip(allv, got):
        abits = sum(1 << t for t in range(K) if row[t] > 0)
        hamming = bin(abits ^ wbits).count("1")
        assert g == K - 2 * hamming


def test_popcount_identity_golden():
    r = _golden_rows("popcount_worked.txt")
    a = np.array([[int(v) for v in r["a"][0]]], dtype=np.int8)
    w = np.array([[int(v) for v in r["w"][0]]], dtype=np.int8)
    assert int(oracle.pack_bits(a)[0, 0]) == int(r["a_word"][0][0], 16)
    assert int(oracle.pack_bits(w)[0, 0]) == int(r["w_word"][0][0], 16)
    assert oracle.gemm_pm1(a, w)[0, 0] == int(r["dot"][0][0])
    x = int(oracle.pack_bits(a)[0, 0]) ^ int(oracle.pack_bits(w)[0, 0])
    assert bin(x).count("1") == int(r["xor_popcount"][0][0])


@pytest.mark.parametrize("K", [1, 31, 32, 33, 95, 96, 97, 200, 784])
def test_popcount_identity_random(seed, K):
    # Eq. (popc): agreements P = popcount(xnor) over the K real positions; dot = 2P - K = K - 2 popcount(xor)
    a = qi.pm1(seed, 16, (6, K))
    w = qi.pm1(seed, 17, (5, K))
    pa, pw = oracle.pack_bits(a), oracle.pack_bits(w)
    direct = oracle.gemm_pm1(a, w)
    for m in range(6):
        am = int.from_bytes(pa[m].tobytes(), "little")
        for n in range(5):
            wn = int.from_bytes(pw[n].tobytes(), "little")
            assert direct[m, n] == K - 2 * bin(am ^ wn).count("1")
            mask = (1 << K) - 1
            agreements = bin(~(am ^ wn) & mask).count("1")
            assert direct[m, n] == 2 * agreements - K


# ---------------------------------------------------------------- bit planes (Sec. 2.6 Eq. (FirstLayer), Sec. 3)
def test_first_layer_golden():
    r = _golden_rows("first_layer_worked.txt")
    x = np.array([[int(v) for v in r["x"][0]]], dtype=np.int32)
    w = np.array([[int(v) for v in r["w"][0]]], dtype=np.int32)
    s = int(r["s"][0][0])
    assert oracle.gemm_int(x, w)[0, 0] == s
    planes = oracle.split_planes(x, 8)
    wbit = (w > 0).astype(np.uint8)[None]
    for p in range(8):
        d = oracle.gemm_planes(planes[p : p + 1], [1], 0, wbit, [1], 1)[0, 0]
        assert d == int(r["plane_dots"][0][p])
    coef = [1 << p for p in range(8)]
    assert oracle.gemm_planes(planes, coef, 0, wbit, [1], 1)[0, 0] == s


def test_split_planes_msb_is_last():
    v = np.array([128, 1, 0x55, 255], dtype=np.int32)
    p = oracle.split_planes(v, 8)
    assert p[7].tolist() == [1, 0, 0, 1] and p[0].tolist() == [0, 1, 1, 1]
    assert p[:, 2].tolist() == [1, 0, 1, 0, 1, 0, 1, 0]
    assert np.array_equal(sum(p[i].astype(np.int32) << i for i in range(8)), v)


@pytest.mark.parametrize("M,N,K", [(4, 3, 1), (5, 7, 33), (16, 12, 784)])
def test_gemm_int_equals_int64_matmul(seed, M, N, K):
    u = qi.uniform_int(seed, 20, (M, K), 0, 255)
    v = qi.uniform_int(seed, 21, (N, K), -8, 7)
    want = u.astype(np.int64) @ v.astype(np.int64).T
    assert np.array_equal(oracle.gemm_int(u, v), want)


def test_planes_u8_times_sign(seed):
    M, N, K = 9, 11, 100
    x = qi.uniform_int(seed, 22, (M, K), 0, 255)
    w = qi.pm1(seed, 23, (N, K))
    want = x.astype(np.int64) @ w.astype(np.int64).T
    got = oracle.gemm_planes(oracle.split_planes(x, 8), [1 << p for p in range(8)], 0, (w > 0).astype(np.uint8)[None],
                             [1], 1)
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.gemm_int(x, w.astype(np.int32)), want)
    # all planes set: x = 255 everywhere gives 255 * sum(w)
    x255 = np.full((1, K), 255, dtype=np.int32)
    got = oracle.gemm_planes(oracle.split_planes(x255, 8), [1 << p for p in range(8)], 0,
                             (w > 0).astype(np.uint8)[None], [1], 1)
    assert np.array_equal(got[0], 255 * w.astype(np.int64).sum(axis=1))


def test_planes_twos_complement_4bit(seed):
    M, N, K = 6, 5, 70
    a = qi.uniform_int(seed, 24, (M, K), -8, 7)
    w = qi.uniform_int(seed, 25, (N, K), -8, 7)
    coef = [1, 2, 4, -8]
    got = oracle.gemm_planes(oracle.split_planes(a, 4), coef, 0, oracle.split_planes(w, 4), coef, 0)
    assert np.array_equal(got, a.astype(np.int64) @ w.astype(np.int64).T)


def test_planes_all_sign_code(seed):
    # "apply the XNOR kernel several times": every plane read as +-1, value = sum 2^p s_p (odd integers)
    M, N, K, P = 4, 6, 45, 3
    pa = qi.bernoulli_bits(seed, 26, (P, M, K))
    pw = qi.bernoulli_bits(seed, 27, (2, N, K))
    va = sum((2 * pa[p].astype(np.int64) - 1) << p for p in range(P))
    vw = sum((2 * pw[p].astype(np.int64) - 1) << p for p in range(2))
    got = oracle.gemm_planes(pa, [1, 2, 4], 1, pw, [1, 2], 1)
    assert np.array_equal(got, va @ vw.T)
    # a single sign plane on each side is the +-1 product
    one = oracle.gemm_planes(pa[:1], [1], 1, pw[:1], [1], 1)
    assert np.array_equal(one, oracle.gemm_pm1(2 * pa[0].astype(np.int8) - 1, 2 * pw[0].astype(np.int8) - 1))


@pytest.mark.parametrize("modeA,modeW", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_planes_every_mode_pair_equals_int64_matmul_of_plane_values(seed, modeA, modeW):
    """Each of the four (mode A, mode W) pairs, the mixed ones included ((sign A, bit W) is the transposed first
    layer: +-1 activations against 0/1 weight planes), against numpy int64 on the values the planes encode with odd
    and negative coefficients.  A swapped mode argument, a mode applied to the wrong operand or a lost coefficient
    sign changes the result."""
    M, N, K, Pa, Pb = 5, 7, 53, 3, 2
    pa = qi.bernoulli_bits(seed, 28, (Pa, M, K)).astype(np.int64)
    pw = qi.bernoulli_bits(seed, 29, (Pb, N, K)).astype(np.int64)
    ca, cw = [1, -2, 5], [3, -4]
    va = sum(c * ((2 * pa[i] - 1) if modeA else pa[i]) for i, c in enumerate(ca))
    vw = sum(c * ((2 * pw[j] - 1) if modeW else pw[j]) for j, c in enumerate(cw))
    assert np.array_equal(oracle.gemm_planes(pa, ca, modeA, pw, cw, modeW), va @ vw.T)
    if modeA != modeW:  # the two mixed pairs must differ from each other on the same planes (operands not swapped)
        other = oracle.gemm_planes(pa, ca, modeW, pw, cw, modeA)
        assert not np.array_equal(other, va @ vw.T)


def test_range_check_reports_overflow():
    u = np.full((1, 4), 2**30, dtype=np.int32)
    with pytest.raises(oracle.OracleRangeError):
        oracle.gemm_int(u, np.full((1, 4), 2, dtype=np.int32))


# ---------------------------------------------------------------- threshold (Alg. 4: Sign(BatchNorm(.)))
def test_threshold_hand_table():
    C = np.array([[-2, -1, 0, 1, 2]], dtype=np.int32).T.copy()  # 5 samples, 1 neuron
    assert oracle.threshold(C, [0]).ravel().tolist() == [-1, -1, 1, 1, 1]  # tie C == T gives +1
    assert oracle.threshold(C, [0], [1]).ravel().tolist() == [1, 1, -1, -1, -1]
    assert oracle.threshold(C, [2]).ravel().tolist() == [-1, -1, -1, -1, 1]
    assert oracle.threshold(C, [-(2**31)]).ravel().tolist() == [1] * 5
    assert oracle.threshold(C, [-(2**31)], [1]).ravel().tolist() == [-1] * 5
    # the threshold is per neuron (column), not per sample
    C2 = np.array([[0, 0], [5, 5]], dtype=np.int32)
    assert oracle.threshold(C2, [1, 6]).tolist() == [[-1, -1], [1, -1]]


def test_threshold_equals_float_batchnorm_sign_exhaustive():
    s = np.arange(-70, 71, dtype=np.int32)
    Ts = np.arange(-66, 67, dtype=np.int32)
    C = np.repeat(s[:, None], Ts.size, axis=1)
    n = Ts.size
    one, zero = np.ones(n), np.zeros(n)
    # gamma = +1: y = s - T >= 0  <=>  s >= T
    want = oracle.bn_sign(C, one, -Ts.astype(np.float64), zero, one, 0.0)
    assert np.array_equal(oracle.threshold(C, Ts), want)
    assert np.array_equal(want > 0, s[:, None] >= Ts[None, :])
    # gamma = -1: y = -(s) + (T - 1) >= 0  <=>  s <= T - 1  <=>  not (s >= T)
    want = oracle.bn_sign(C, -one, Ts.astype(np.float64) - 1.0, zero, one, 0.0)
    assert np.array_equal(oracle.threshold(C, Ts, np.ones(n, dtype=np.uint8)), want)


def test_bn_sign_matches_torch_batchnorm(seed):
    N = 13
    C = qi.uniform_int(seed, 30, (50, N), -300, 300)
    g = qi.normal_f32(seed, 31, (N,)).astype(np.float64)
    b = qi.normal_f32(seed, 32, (N,)).astype(np.float64) * 3
    mu = qi.normal_f32(seed, 33, (N,)).astype(np.float64) * 20
    var = np.abs(qi.normal_f32(seed, 34, (N,)).astype(np.float64)) * 50 + 0.5
    y = torch.nn.functional.batch_norm(torch.from_numpy(C).double(), torch.from_numpy(mu), torch.from_numpy(var),
                                       torch.from_numpy(g), torch.from_numpy(b), False, 0.0, 1e-4).numpy()
    safe = np.abs(y) > 1e-9
    got = oracle.bn_sign(C, g, b, mu, var, 1e-4)
    assert np.array_equal(got[safe] > 0, y[safe] >= 0)


# ---------------------------------------------------------------- MLP (Alg. 4)
def test_mlp_equals_float_layers(seed):
    dims = [50, 40, 33, 7]
    B = 19
    x = qi.uniform_int(seed, 40, (B, dims[0]), 0, 255, dtype=np.uint8)
    W = [qi.pm1(seed, 41 + l, (dims[l + 1], dims[l])) for l in range(3)]
    T = [qi.uniform_int(seed, 45 + l, (dims[l + 1],), -40 if l else -2000, 40 if l else 2000) for l in range(2)]
    flip = [qi.bernoulli_bits(seed, 48 + l, (dims[l + 1],)) for l in range(2)]
    # "the MLP accuracy does not depend on which kernel is used": float GEMMs layer by layer give the same outputs
    a = torch.from_numpy(x).double()
    for l in range(3):
        s = a @ torch.from_numpy(W[l]).double().T
        if l < 2:
            ge = s >= torch.from_numpy(T[l]).double()
            bit = ge ^ torch.from_numpy(flip[l]).bool()
            a = torch.where(bit, 1.0, -1.0).double()
    got = oracle.mlp(x, W, T, flip)
    assert np.array_equal(got, s.numpy().astype(np.int64))
    # flip omitted == all-zero flip
    z = [np.zeros_like(f) for f in flip]
    assert np.array_equal(oracle.mlp(x, W, T), oracle.mlp(x, W, T, z))
    # layer by layer with the oracle's own pieces
    a1 = oracle.threshold(oracle.gemm_int(x, W[0]), T[0], flip[0])
    a2 = oracle.threshold(oracle.gemm_pm1(a1, W[1]), T[1], flip[1])
    assert np.array_equal(got, oracle.gemm_pm1(a2, W[2]))


# ---------------------------------------------------------------- convolution (Sec. 5 filter bank; AlexNet 3x3 layers)
@pytest.mark.parametrize("B,H,W,Ci,Co,KH,pad,stride", [(2, 5, 6, 7, 4, 3, 1, 1), (1, 13, 13, 40, 9, 3, 1, 1),
                                                       (2, 8, 7, 5, 3, 5, 2, 2), (1, 4, 4, 3, 2, 1, 0, 1)])
def test_conv_equals_library_conv(seed, B, H, W, Ci, Co, KH, pad, stride):
    u = qi.uniform_int(seed, 50, (B, H, W, Ci), 0, 3)
    w = qi.pm1(seed, 51, (Co, KH, KH, Ci)).astype(np.int32)
    want = torch.nn.functional.conv2d(torch.from_numpy(u).double().permute(0, 3, 1, 2),
                                      torch.from_numpy(w).double().permute(0, 3, 1, 2), padding=pad, stride=stride)
    want = want.permute(0, 2, 3, 1).numpy()
    got = oracle.conv2d(u, w, pad, stride)
    assert got.shape == want.shape
    assert np.array_equal(got.astype(np.float64), want)


def test_conv_equals_im2col_gemm(seed):
    B, H, W, Ci, Co = 2, 6, 5, 9, 4
    u = qi.uniform_int(seed, 52, (B, H, W, Ci), 0, 3)
    w = qi.pm1(seed, 53, (Co, 3, 3, Ci)).astype(np.int32)
    up = np.zeros((B, H + 2, W + 2, Ci), dtype=np.int32)
    up[:, 1:-1, 1:-1] = u
    patches = np.stack([up[:, ky : ky + H, kx : kx + W] for ky in range(3) for kx in range(3)], axis=3)
    got = oracle.gemm_int(patches.reshape(B * H * W, 9 * Ci), w.reshape(Co, 9 * Ci)).reshape(B, H, W, Co)
    assert np.array_equal(got, oracle.conv2d(u, w, 1))
    # 1x1 kernel: a plain matrix product per pixel
    w1 = qi.pm1(seed, 54, (Co, 1, 1, Ci)).astype(np.int32)
    assert np.array_equal(oracle.conv2d(u, w1, 0).reshape(-1, Co), oracle.gemm_int(u.reshape(-1, Ci), w1.reshape(Co, Ci)))


FROZEN_PM1 = [[1, -1, 1, -1, 1, -1, -1, 1], [1, 1, -1, -1, 1, 1, 1, 1]]
FROZEN_UNIFORM = [51, -63, -61, -35, 45, 42]


# ---------------------------------------------------------------- the input generators are frozen
def test_generator_is_frozen():
    assert qi.raw_u64(qi.SEED_BASE, 7, 3).tolist() == qi.raw_u64(qi.SEED_BASE, 7, 5, 0)[:3].tolist()
    assert qi.raw_u64(qi.SEED_BASE, 7, 3, offset=2)[0] == qi.raw_u64(qi.SEED_BASE, 7, 3)[2]
    assert qi.pm1(qi.SEED_BASE, 30, (2, 8)).tolist() == FROZEN_PM1
    assert qi.uniform_int(qi.SEED_BASE, 25, (6,), -64, 64).tolist() == FROZEN_UNIFORM


# ---------------------------------------------------------------- ConvNet of App. A (CIFAR-10 ConvNet table)
def test_maxpool_hand_values_and_library(seed):
    """2 x 2 / stride 2 max-pooling on channels-last integer maps: a hand-written 4 x 4 case (negative values, the
    maximum in every corner of a window), odd sizes dropped, and torch's max_pool2d in fp64 on random maps."""
    u = np.array([[1, -5, 7, 7], [0, 2, -9, 8], [-1, -2, 3, 3], [-3, -4, 3, 4]], dtype=np.int32)[None, :, :, None]
    assert oracle.maxpool2x2(u)[0, :, :, 0].tolist() == [[2, 8], [-1, 4]]
    v = qi.uniform_int(seed, 70, (3, 7, 9, 5), -1000, 1000)
    want = torch.nn.functional.max_pool2d(torch.from_numpy(v).double().permute(0, 3, 1, 2), 2).permute(0, 2, 3, 1)
    got = oracle.maxpool2x2(v)
    assert got.shape == (3, 3, 4, 5)
    assert np.array_equal(got, want.numpy().astype(np.int32))


def _float_convnet(x, conv_w, pool, fc_w, T, flip):
    """The float definition with a library in fp64: conv ("same", zero padding) -> max-pool -> BatchNorm -> sign, then
    fully connected layers on the (y, x, c)-flattened map.  BatchNorm parameters are chosen so that its zero crossing
    lies half way between two integers: y = gamma * (s - (T - 0.5)), gamma = +1 (flip 0) or -1 (flip 1)."""
    F = torch.nn.functional
    a = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)  # NCHW
    l = 0
    for w, p in zip(conv_w, pool):
        s = F.conv2d(a, torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2), padding=1)
        if p:
            s = F.max_pool2d(s, 2)
        gamma = torch.from_numpy(np.where(flip[l] != 0, -1.0, 1.0))
        mean = torch.from_numpy(T[l].astype(np.float64) - 0.5)
        eps = 2.0 ** -20  # var + eps is exactly 1
        y = F.batch_norm(s, mean, torch.full_like(mean, 1.0 - eps), gamma, torch.zeros_like(mean), False, 0.0, eps)
        a = torch.where(y >= 0, 1.0, -1.0).double()
        l += 1
    a = a.permute(0, 2, 3, 1).reshape(a.shape[0], -1)  # (y, x, c) order
    for j, w in enumerate(fc_w):
        s = a @ torch.from_numpy(w.astype(np.float64)).T
        if j == len(fc_w) - 1:
            return s.numpy().astype(np.int64)
        gamma = torch.from_numpy(np.where(flip[l] != 0, -1.0, 1.0))
        y = gamma * (s - torch.from_numpy(T[l].astype(np.float64) - 0.5))
        a = torch.where(y >= 0, 1.0, -1.0).double()
        l += 1


def _convnet_case(seed, B, H, Wd, C0, couts, pools, fcs, stream0):
    x = qi.uniform_int(seed, stream0, (B, H, Wd, C0), 0, 255, dtype=np.uint8)
    conv_w, cin = [], C0
    for l, co in enumerate(couts):
        conv_w.append(qi.pm1(seed, stream0 + 1 + l, (co, 3, 3, cin)))
        cin = co
    h, w = H, Wd
    for p in pools:
        if p:
            h, w = h // 2, w // 2
    fc_w, fin = [], h * w * cin
    for j, fo in enumerate(fcs):
        fc_w.append(qi.pm1(seed, stream0 + 20 + j, (fo, fin)))
        fin = fo
    widths = list(couts) + list(fcs[:-1])
    T, flip = [], []
    for l, n in enumerate(widths):
        span = 2000 if l == 0 else 12  # first-layer sums are sums of 8-bit inputs
        T.append(qi.uniform_int(seed, stream0 + 40 + l, (n,), -span, span))
        flip.append(qi.bernoulli_bits(seed, stream0 + 60 + l, (n,)))
    return x, conv_w, list(pools), fc_w, T, flip


@pytest.mark.parametrize("B,H,Wd,C0,couts,pools,fcs", [(2, 8, 8, 3, [8, 8, 16, 16], [0, 1, 0, 1], [24, 10]),
                                                      (3, 6, 10, 3, [5, 7], [1, 0], [9, 6, 4]),
                                                      (2, 5, 7, 2, [6], [1], [3])])
def test_convnet_equals_float_pipeline(seed, B, H, Wd, C0, couts, pools, fcs):
    """Pins: zero padding of the +-1 maps (a padded tap adds 0, not -1), pooling before BatchNorm (so that a negative
    BatchNorm scale turns the maximum into the deciding MINIMUM of the window), ties, the (y, x, c) flattening."""
    x, conv_w, pools, fc_w, T, flip = _convnet_case(seed, B, H, Wd, C0, couts, pools, fcs, 1300)
    got = oracle.convnet(x, conv_w, pools, fc_w, T, flip)
    want = _float_convnet(x, conv_w, pools, fc_w, T, flip)
    assert np.array_equal(got.astype(np.int64), want)


def test_convnet_without_convolutions_is_the_mlp(seed):
    """With no convolution layer and a 1 x 1 map the ConvNet forward is Alg. 4's MLP forward."""
    B, dims = 7, [30, 12, 9, 5]
    x = qi.uniform_int(seed, 1400, (B, dims[0]), 0, 255, dtype=np.uint8)
    W = [qi.pm1(seed, 1401 + l, (dims[l + 1], dims[l])) for l in range(3)]
    T = [qi.uniform_int(seed, 1405 + l, (dims[l + 1],), -300 if l == 0 else -4, 300 if l == 0 else 4) for l in range(2)]
    flip = [qi.bernoulli_bits(seed, 1408 + l, (dims[l + 1],)) for l in range(2)]
    got = oracle.convnet(x.reshape(B, 1, 1, dims[0]), [], [], W, T, flip)
    assert np.array_equal(got, oracle.mlp(x, W, T, flip))


# ---------------------------------------------------------------- quantizers of Sec. 3 and AP2 of Alg. 2's caption
def test_linear_quant_hand_values_and_library(seed):
    """LinearQuant(x, step) = Clip(round(x / step) * step, minV, maxV) on hand-computed cases (step 0.25, range
    [-2, 1.75] = codes [-8, 7]): interior values, both clips, ties to even, signed zero, NaN; then numpy's single
    precision rint / clip on random values."""
    x = np.array([0.26, 0.37, 0.38, 0.125, 0.375, -0.125, -0.375, 0.625, 5.0, -9.0, 1.75, 1.8, -2.0, 0.0, -0.0, np.nan,
                  np.inf, -np.inf], dtype=np.float32)
    want = [1, 1, 2, 0, 2, 0, -2, 2, 7, -8, 7, 7, -8, 0, 0, 0, 7, -8]
    assert oracle.linear_quant(x, 0.25, -8, 7).tolist() == want
    assert oracle.linear_quant(np.array([0.5, 1.5, 2.5, 3.5], dtype=np.float32), 1.0, 0, 3).tolist() == [0, 2, 2, 3]
    v = qi.normal_f32(seed, 1800, (4000,)) * np.float32(3.0)
    for step, lo, hi in [(0.1, 0, 15), (0.3, -8, 7), (1.0 / 3.0, -2, 1)]:
        lib_q = np.clip(np.rint(v / np.float32(step)), lo, hi).astype(np.int32)  # float32 division, ties to even
        assert np.array_equal(oracle.linear_quant(v, step, lo, hi), lib_q)
    with pytest.raises(RuntimeError):
        oracle.linear_quant(v, 0.0, 0, 3)


def test_ap2_closed_forms_and_library(seed):
    """AP2(x) = sign(x) 2^round(log2 |x|): exact powers of two map to themselves; 3 -> 4 (log2 3 = 1.58), 2.8 -> 2
    (1.485), 2.83 -> 4 (1.5008), 0.7 -> 0.5 (-0.515), 0.71 -> 1 (-0.494); the two floats next to sqrt(2); a denormal;
    then numpy's log2 / round in double on random values."""
    x = np.array([1.0, 2.0, 0.5, -8.0, 3.0, -3.0, 2.8, 2.83, 0.7, 0.71, 0.0, -0.0, np.nan], dtype=np.float32)
    e, s = oracle.ap2(x)
    assert e.tolist() == [0, 1, -1, 3, 2, 2, 1, 2, -1, 0, 0, 0, 0]
    assert s.tolist() == [1, 1, 1, -1, 1, -1, 1, 1, 1, 1, 0, 0, 0]
    below, above = np.array([0x3FB504F3, 0x3FB504F4], dtype=np.uint32).view(np.float32)  # neighbours of sqrt(2)
    assert oracle.ap2(np.array([below, above, below * 4, above / 8], dtype=np.float32))[0].tolist() == [0, 1, 2, -2]
    assert oracle.ap2(np.array([2.0 ** -140, 3.0 * 2.0 ** -149], dtype=np.float32))[0].tolist() == [-140, -147]
    v = qi.normal_f32(seed, 1801, (5000,)) * np.float32(40.0)
    v = v[v != 0]
    e, s = oracle.ap2(v)
    assert np.array_equal(e, np.round(np.log2(np.abs(v.astype(np.float64)))).astype(np.int32))
    assert np.array_equal(s, np.sign(v).astype(np.int8))
    # the defining property: |x| / AP2(x) lies in [2^-1/2, 2^1/2)
    ratio = np.abs(v.astype(np.float64)) / 2.0 ** e
    assert (ratio >= 2 ** -0.5).all() and (ratio < 2 ** 0.5).all()


def test_log_quant_hand_values():
    """LogQuant(x) = Clip(AP2(x), minV, maxV) with magnitudes 2^-3 .. 2^2 (emin = -3, emax = 2): codes 1 .. 6 with the
    sign; below 2^-3.5 flushed to 0, above clipped."""
    x = np.array([1.0, -1.0, 0.125, 0.1, 0.09, 0.08, 4.0, 5.0, 100.0, -100.0, 0.0, np.nan, np.inf, -0.7, 3.0],
                 dtype=np.float32)
    #            1    -1   2^-3  ~2^-3 ~2^-3  <2^-3.5 2^2  2^2   clip   clip   0    nan     inf   2^-1  2^2
    assert oracle.log_quant(x, -3, 2).tolist() == [4, -4, 1, 1, 1, 0, 6, 6, 6, -6, 0, 0, 6, -3, 6]
    codes = oracle.log_quant(x, -3, 2).astype(np.int64)
    vals = np.sign(codes) * 2.0 ** (-3 + np.abs(codes) - 1) * (codes != 0)
    assert vals.tolist()[:7] == [1.0, -1.0, 0.125, 0.125, 0.125, 0.0, 4.0]


# ---------------------------------------------------------------- backward pass of Alg. 1 with quantized gradients
def test_log_code_value_and_ste_hand_values():
    """Fixed-point value of a logarithmic code: code c is sign(c) 2^(|c| - 1) (1, 2, 4, ... and 0 for code 0); the
    straight-through estimator of Alg. 1 passes g where |a| <= 1 (bounds included) and cancels it elsewhere."""
    codes = np.array([0, 1, -1, 2, -2, 3, 6, -6, 7], dtype=np.int8)
    assert oracle.log_code_value(codes).tolist() == [0, 1, -1, 2, -2, 4, 32, -32, 64]
    g = np.array([0.5, -2.0, 3.0, 4.0, 5.0, 6.0, 7.0, 8.0], dtype=np.float32)
    a = np.array([0.0, 1.0, -1.0, 1.0000001, -1.5, np.nan, np.inf, -0.99], dtype=np.float32)
    assert oracle.ste_mask(g, a).tolist() == [0.5, -2.0, 3.0, 0.0, 0.0, 0.0, 0.0, 8.0]


def test_bn_affine_exact_cases_and_double(seed):
    """y = scale * s + shift with one rounding: exact whenever the true result is representable (integer sums, powers
    of two as scale, small shifts), and within half an ulp of the double-precision value otherwise."""
    s = np.array([[0, 1, -3, 1000], [7, -8, 12345, -2 ** 20]], dtype=np.int32)
    scale = np.array([0.5, 2.0, -0.25, 1.0], dtype=np.float32)
    shift = np.array([1.0, -3.0, 0.5, 0.25], dtype=np.float32)
    want = [[1.0, -1.0, 1.25, 1000.25], [4.5, -19.0, -3085.75, -1048575.75]]
    assert oracle.bn_affine(s, scale, shift).tolist() == want
    M, N = 50, 37
    s = qi.uniform_int(seed, 1900, (M, N), -5000, 5000)
    scale = qi.normal_f32(seed, 1901, (N,))
    shift = qi.normal_f32(seed, 1902, (N,)) * np.float32(10.0)
    got = oracle.bn_affine(s, scale, shift).astype(np.float64)
    exact = s.astype(np.float64) * scale.astype(np.float64) + shift.astype(np.float64)  # error below 2^-52 relative
    ulp = np.spacing(np.abs(got).astype(np.float32)).astype(np.float64)
    assert (np.abs(got - exact) <= 0.5 * ulp * (1 + 1e-6)).all()
    # a case where rounding the product first would differ: 3 * (1 + 2^-23) + (-3) = 3 * 2^-23 exactly
    one_eps = np.array([1.0 + 2.0 ** -23], dtype=np.float32)
    assert oracle.bn_affine(np.array([[3]], dtype=np.int32), one_eps, np.array([-3.0], dtype=np.float32))[0, 0] == np.float32(3 * 2.0 ** -23)


def test_backward_products_against_library(seed):
    """g_a = g W and g_W = g^T a (Alg. 1, backward block) against int64 library products of the same matrices, a case
    worked by hand, and the closed form for constant operands."""
    g = np.array([[1, -2], [4, 0], [-8, 16]], dtype=np.int32)          # M = 3, N = 2
    w = np.array([[1, -1, 1, 1], [-1, -1, 1, -1]], dtype=np.int8)      # N = 2, K = 4
    a = np.array([[1, 1, -1, 1], [-1, 1, 1, 1], [1, -1, -1, -1]], dtype=np.int8)
    ga, gw = oracle.backward(g, w, a)
    assert ga.tolist() == [[3, 1, -1, 3], [4, -4, 4, 4], [-24, -8, 8, -24]]
    assert gw.tolist() == [[-11, 13, 11, 13], [14, -18, -14, -18]]
    M, N, K = 37, 29, 45
    g = qi.uniform_int(seed, 1910, (M, N), -64, 64)
    w = qi.pm1(seed, 1911, (N, K))
    a = qi.pm1(seed, 1912, (M, K))
    ga, gw = oracle.backward(g, w, a)
    assert np.array_equal(ga, (g.astype(np.int64) @ w.astype(np.int64)).astype(np.int32))
    assert np.array_equal(gw, (g.astype(np.int64).T @ a.astype(np.int64)).astype(np.int32))
    ones_w, ones_a = np.ones((N, K), dtype=np.int8), np.ones((M, K), dtype=np.int8)
    ga, gw = oracle.backward(g, ones_w, ones_a)
    assert np.array_equal(ga, np.repeat(g.sum(axis=1, keepdims=True), K, axis=1))
    assert np.array_equal(gw, np.repeat(g.sum(axis=0)[:, None], K, axis=1))
    with pytest.raises(oracle.OracleRangeError):
        oracle.backward(np.full((2, 2), 2 ** 30, dtype=np.int32), np.ones((2, 3), dtype=np.int8), np.ones((2, 3), dtype=np.int8))


# ---------------------------------------------------------------- repetition of binary 2-D filters (Sec. 5)
def test_filter_unique_hand_cases_and_expectation(seed):
    """Distinct 3 x 3 filters per input channel up to negation: a bank of copies has 1, a filter and its negation count
    once, a hand-built bank with known repeats; for random +-1 banks the expected count per channel is
    256 (1 - (255/256)^cout) (each filter falls into one of 2^9 / 2 classes uniformly)."""
    base = qi.pm1(seed, 3000, (1, 3, 3, 5))
    assert oracle.filter_unique(np.repeat(base, 7, axis=0)).tolist() == [1] * 5
    both = np.concatenate([base, -base, base], axis=0)
    assert oracle.filter_unique(both).tolist() == [1] * 5
    w = np.ones((4, 3, 3, 2), dtype=np.int8)
    w[1, 0, 0, 0] = -1                      # channel 0: filters {A, B, A, -B}; channel 1: {A, A, A, C}
    w[3, :, :, 0] = -w[1, :, :, 0]
    w[3, 2, 2, 1] = -1
    assert oracle.filter_unique(w).tolist() == [2, 2]
    cout, cin = 128, 64
    counts = oracle.filter_unique(qi.pm1(seed, 3001, (cout, 3, 3, cin)))
    expect = 256.0 * (1.0 - (255.0 / 256.0) ** cout)   # 100.9
    assert abs(counts.mean() - expect) < 2.0 and counts.min() >= 80 and counts.max() <= 128


def test_conv2d_dedup_equals_direct_convolution(seed):
    """Summing the responses of the distinct 2-D filters gives the same sums as the direct convolution (Sec. 5), for
    +-1 and for multi-bit activations, with and without padding; the number of filter applications is the sum of the
    per-channel distinct counts."""
    for (B, H, W, cin, cout, pad, lo, hi) in [(2, 6, 5, 7, 40, 1, 0, 3), (1, 8, 8, 3, 600, 1, -1, 1), (3, 4, 4, 5, 9, 0, 0, 1)]:
        u = qi.uniform_int(seed, 3010, (B, H, W, cin), lo, hi)
        if (lo, hi) == (-1, 1):
            u = qi.pm1(seed, 3011, (B, H, W, cin)).astype(np.int32)
        w = qi.pm1(seed, 3012, (cout, 3, 3, cin))
        got, applied = oracle.conv2d_dedup(u, w, pad)
        assert np.array_equal(got, oracle.conv2d(u, w.astype(np.int32), pad))
        assert applied == int(oracle.filter_unique(w).sum())
        if cout == 600:
            assert applied < 0.45 * cout * cin   # 600 filters per channel fall into at most 256 classes
