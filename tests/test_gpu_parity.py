"""Parity of the HIP path against the CPU oracle, call by call through the C ABI, element by element, bit exact.
Inputs are seeded and synthetic; expected values come only from the oracle on unpacked arrays."""
import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi
from qnn_testlib import (dev, engine_takes, host, host_u32, np_pack_bits, np_pack_pm1, np_unpack_bits,
                         run_on_engine)

pytestmark = pytest.mark.gpu

q = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global q
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_1609_07061_amd as mod

    q = mod
    yield
    torch.cuda.synchronize()


ENGINES = [1, 2, 3, 0]  # VALU, int8 MFMA, FP4 MFMA, AUTO
PLANE_ENGINES = [1, 2, 3, 4, 0]  # ... and the int8 kernel that merges planes once per workgroup, for multi-plane operands


# ------------------------------------------------------------------ S1 pack_sign
@pytest.mark.parametrize("rows,K", [(1, 1), (3, 31), (5, 32), (7, 33), (2, 63), (4, 64), (3, 65), (9, 1000), (17, 513),
                                    (128, 1024), (1024, 1024), (33, 4099)])
def test_pack_sign(seed, rows, K):
    x = qi.with_special_floats(qi.normal_f32(seed, 10, (rows, K)), seed, 12)
    want = oracle.pack_bits(oracle.sign(x))
    got = host_u32(q.qnn_pack_sign(dev(x)))
    assert np.array_equal(got, want)


def test_pack_sign_strided_leaves_padding_untouched(seed):
    rows, K, ldx, ldo = 6, 70, 96, 5
    buf = qi.normal_f32(seed, 13, (rows, ldx))
    x = dev(buf)[:, :K]
    out = torch.full((rows, ldo), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_pack_sign(x, out=out[:, :3])
    got = host_u32(out)
    assert np.array_equal(got[:, :3], oracle.pack_bits(oracle.sign(buf[:, :K])))
    assert (got[:, 3:] == 0x5A5A5A5A).all()


def test_pack_sign_every_edge_value_in_every_lane():
    sp = qi.special_floats()
    x = np.stack([np.roll(np.resize(sp, 128), i) for i in range(64)])
    assert np.array_equal(host_u32(q.qnn_pack_sign(dev(x))), oracle.pack_bits(oracle.sign(x)))


@pytest.mark.parametrize("rows,K", [(5, 2048), (3, 2052), (7, 4100), (2, 6148), (64, 8192), (3, 2050), (2, 4099)])
def test_pack_sign_long_rows(seed, rows, K):
    """Rows of 2048 elements and more made of whole aligned groups of four take the 16-byte-load kernel (several
    chunks per row, ragged last chunk); K = 2050 and 4099 stay on the one-element-per-lane kernel."""
    x = qi.with_special_floats(qi.normal_f32(seed, 14, (rows, K)), seed, 15)
    assert np.array_equal(host_u32(q.qnn_pack_sign(dev(x))), oracle.pack_bits(oracle.sign(x)))


def test_pack_sign_long_rows_strided_and_edge_values(seed):
    """16-byte-load kernel on a strided view (pitch 2304 floats, output pitch 80 words): padding stays untouched, and
    every special value visits every position of a four-element group and of a 32-bit word."""
    rows, K, ldx, ldo = 67, 2240, 2304, 80
    sp = qi.special_floats()
    buf = np.stack([np.roll(np.resize(sp, ldx), i) for i in range(rows)]).astype(np.float32)
    buf[::3] = qi.normal_f32(seed, 16, (len(buf[::3]), ldx))
    out = torch.full((rows, ldo), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_pack_sign(dev(buf)[:, :K], out=out[:, :K // 32])
    got = host_u32(out)
    assert np.array_equal(got[:, :K // 32], oracle.pack_bits(oracle.sign(buf[:, :K])))
    assert (got[:, K // 32:] == 0x5A5A5A5A).all()
    # a view that starts 4 bytes off the 16-byte grid must give the same bits through the other kernel
    got2 = host_u32(q.qnn_pack_sign(dev(buf)[:, 1:K + 1]))
    assert np.array_equal(got2, oracle.pack_bits(oracle.sign(buf[:, 1:K + 1])))


# ------------------------------------------------------------------ S1b pack_bitplanes
@pytest.mark.parametrize("rows,K,nbits", [(1, 1, 1), (3, 33, 2), (5, 64, 4), (4, 257, 8), (10, 784, 8), (7, 2048, 4),
                                          (6, 255, 3)])
def test_pack_bitplanes(seed, rows, K, nbits):
    v = qi.uniform_int(seed, 14, (rows, K), 0, (1 << nbits) - 1)
    planes = oracle.split_planes(v, nbits)  # [nbits][rows][K] of 0/1
    want = np.stack([oracle.pack_bits(planes[p].astype(np.int8)) for p in range(nbits)])
    got = host_u32(q.qnn_pack_bitplanes(dev(v.astype(np.uint8)), nbits))
    assert np.array_equal(got, want)


def test_pack_bitplanes_twos_complement_codes(seed):
    v = qi.uniform_int(seed, 15, (5, 100), -8, 7)
    planes = oracle.split_planes(v, 4)
    want = np.stack([oracle.pack_bits(planes[p].astype(np.int8)) for p in range(4)])
    codes = (v & 0xF).astype(np.uint8)
    assert np.array_equal(host_u32(q.qnn_pack_bitplanes(dev(codes), 4)), want)


@pytest.mark.parametrize("rows,K,nbits", [(5, 512, 8), (3, 784, 8), (9, 1028, 3), (7, 2048, 2), (4, 2052, 4),
                                          (2, 4100, 1), (64, 8192, 8), (3, 786, 8), (2, 2049, 4), (5, 1024, 8),
                                          (3, 1040, 5), (6, 2064, 8), (2, 4112, 3), (9, 6160, 7)])
def test_pack_bitplanes_long_rows(seed, rows, K, nbits):
    """Rows of 1024 codes and more made of whole aligned groups of 16 take the kernel in which a lane owns a whole
    output word (K = 1024, 1040, 2048, 2064, 4112, 6160, 8192: half-used words, ragged last chunk); shorter ones and
    multiples of 4 only the 4-byte-load kernel; K = 786 and 2049 stay on the one-code-per-lane kernel."""
    v = qi.uniform_int(seed, 19, (rows, K), 0, (1 << nbits) - 1)
    planes = oracle.split_planes(v, nbits)
    want = np.stack([oracle.pack_bits(planes[p].astype(np.int8)) for p in range(nbits)])
    assert np.array_equal(host_u32(q.qnn_pack_bitplanes(dev(v.astype(np.uint8)), nbits)), want)


def test_pack_bitplanes_long_rows_strided(seed):
    """4-byte-load kernel on a strided view with padded output planes: padding untouched; a view one byte off the
    4-byte grid gives the same through the other kernel."""
    rows, K, ldv, nbits, ldo = 37, 1200, 1280, 8, 40  # 1200 = 16 * 75: the word-per-lane kernel; K + 4 below: 4-byte
    buf = qi.uniform_int(seed, 20, (rows, ldv), 0, 255).astype(np.uint8)
    out = torch.full((nbits, rows, ldo), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_pack_bitplanes(dev(buf)[:, :K], nbits, out=out[:, :, :38])
    got = host_u32(out)
    planes = oracle.split_planes(buf[:, :K].astype(np.int64), nbits)
    want = np.stack([oracle.pack_bits(planes[p].astype(np.int8)) for p in range(nbits)])
    assert np.array_equal(got[:, :, :38], want)
    assert (got[:, :, 38:] == 0x5A5A5A5A).all()
    K4 = K + 4
    planes4 = oracle.split_planes(buf[:, :K4].astype(np.int64), nbits)
    want4 = np.stack([oracle.pack_bits(planes4[p].astype(np.int8)) for p in range(nbits)])
    assert np.array_equal(host_u32(q.qnn_pack_bitplanes(dev(buf)[:, :K4], nbits)), want4)
    planes1 = oracle.split_planes(buf[:, 1:K + 1].astype(np.int64), nbits)
    want1 = np.stack([oracle.pack_bits(planes1[p].astype(np.int8)) for p in range(nbits)])
    assert np.array_equal(host_u32(q.qnn_pack_bitplanes(dev(buf)[:, 1:K + 1], nbits)), want1)


# ------------------------------------------------------------------ S4 threshold_sign
@pytest.mark.parametrize("M,N", [(37, 256), (9, 260), (70, 1024), (33, 4100), (8, 512), (1, 300)])
@pytest.mark.parametrize("with_flip", [False, True])
def test_threshold_sign_wide_rows(seed, M, N, with_flip):
    """N >= 256 and a multiple of 4 takes the 16-byte-load kernel: row counts that are not multiples of 8, a last
    span of fewer than 256 neurons, sums equal to their threshold, extreme thresholds."""
    Cm = qi.uniform_int(seed, 21, (M, N), -70, 70)
    T = qi.uniform_int(seed, 22, (N,), -64, 64)
    T[0], T[1], T[N - 1] = -(2**31), 2**31 - 1, -(2**31)
    flip = qi.bernoulli_bits(seed, 23, (N,)) if with_flip else None
    want = oracle.pack_bits(oracle.threshold(Cm, T, flip))
    got = host_u32(q.qnn_threshold_sign(dev(Cm), dev(T), dev(flip) if with_flip else None))
    assert np.array_equal(got, want)


def test_threshold_sign_wide_rows_strided(seed):
    M, N, ldc, ldo = 45, 520, 640, 20
    buf = qi.uniform_int(seed, 24, (M, ldc), -70, 70)
    T = qi.uniform_int(seed, 25, (N,), -64, 64)
    flip = qi.bernoulli_bits(seed, 26, (N,))
    out = torch.full((M, ldo), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_threshold_sign(dev(buf)[:, :N], dev(T), dev(flip), out=out[:, :17])
    got = host_u32(out)
    assert np.array_equal(got[:, :17], oracle.pack_bits(oracle.threshold(buf[:, :N], T, flip)))
    assert (got[:, 17:] == 0x5A5A5A5A).all()
    # one element off the 16-byte grid: the other kernel, same answer
    got1 = host_u32(q.qnn_threshold_sign(dev(buf)[:, 1:N + 1], dev(T), dev(flip)))
    assert np.array_equal(got1, oracle.pack_bits(oracle.threshold(buf[:, 1:N + 1], T, flip)))


@pytest.mark.parametrize("M,N", [(1, 1), (3, 31), (5, 64), (17, 65), (40, 4096), (33, 1000)])
@pytest.mark.parametrize("with_flip", [False, True])
def test_threshold_sign(seed, M, N, with_flip):
    Cm = qi.uniform_int(seed, 16, (M, N), -70, 70)
    T = qi.uniform_int(seed, 17, (N,), -64, 64)
    T[0] = -(2**31)
    flip = qi.bernoulli_bits(seed, 18, (N,)) if with_flip else None
    want = oracle.pack_bits(oracle.threshold(Cm, T, flip))
    got = host_u32(q.qnn_threshold_sign(dev(Cm), dev(T), dev(flip) if with_flip else None))
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ S2 binary_gemm
SHAPES = [(1, 1, 1), (3, 5, 31), (17, 3, 32), (64, 17, 33), (130, 64, 63), (5, 130, 64), (64, 64, 65),
          (17, 130, 784), (130, 17, 1000), (128, 1024, 1024), (257, 300, 4096), (300, 10, 4096)]


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_binary_gemm(seed, M, N, K, engine):
    a = qi.pm1(seed, 20, (M, K))
    w = qi.pm1(seed, 21, (N, K))
    want = oracle.gemm_pm1(a, w)
    got = run_on_engine(q.qnn_binary_gemm, dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, engine=engine)
    assert np.array_equal(host(got), want)


@pytest.mark.parametrize("M,N,K", [(256, 1, 32), (300, 8, 1000), (1000, 9, 4096), (257, 16, 16384), (4000, 10, 700),
                                   (300, 16, 16416), (255, 10, 512)])
def test_binary_gemm_skinny_outputs(seed, M, N, K):
    """Few output neurons (an MLP's output layer): AUTO and VALU take the one-row-per-wave kernel when it applies
    (at most 16 neurons, at least 256 rows) and the tiled one otherwise."""
    a = qi.pm1(seed, 20, (M, K))
    w = qi.pm1(seed, 21, (N, K))
    want = oracle.gemm_pm1(a, w)
    for engine in (0, 1):
        out = torch.full((M, N + 3), 99, dtype=torch.int32, device="cuda")
        q.qnn_binary_gemm(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, out=out[:, :N], engine=engine)
        got = host(out)
        assert np.array_equal(got[:, :N], want)
        assert (got[:, N:] == 99).all()


@pytest.mark.parametrize("engine", ENGINES)
def test_binary_gemm_strided_operands_and_output(seed, engine):
    M, N, K = 70, 90, 200  # 7 words per row, held in rows of 9 / 12 words; C rows of 100
    a = qi.pm1(seed, 22, (M, K))
    w = qi.pm1(seed, 23, (N, K))
    A = dev(np_pack_pm1(a, 9))[:, :7]
    W = dev(np_pack_pm1(w, 12))[:, :7]
    out = torch.full((M, 100), -77, dtype=torch.int32, device="cuda")
    run_on_engine(q.qnn_binary_gemm, A, W, K, out=out[:, :N], engine=engine)
    got = host(out)
    assert np.array_equal(got[:, :N], oracle.gemm_pm1(a, w))
    assert (got[:, N:] == -77).all()


@pytest.mark.parametrize("engine", ENGINES)
def test_binary_gemm_from_packed_floats(seed, engine):
    """Config 1 end to end: fp32 N(0,1) -> sign + pack on the GPU -> product."""
    xa = qi.normal_f32(seed, 10, (128, 1024))
    xw = qi.normal_f32(seed, 11, (1024, 1024))
    want = oracle.gemm_pm1(oracle.sign(xa), oracle.sign(xw))
    A = q.qnn_pack_sign(dev(xa))
    W = q.qnn_pack_sign(dev(xw))
    got = run_on_engine(q.qnn_binary_gemm, A, W, 1024, engine=engine)
    assert np.array_equal(host(got), want)


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (17, 33, 65), (130, 100, 784), (64, 4096, 4096), (200, 1000, 96)])
@pytest.mark.parametrize("with_flip", [False, True])
def test_binary_gemm_sign(seed, M, N, K, with_flip, engine):
    a = qi.pm1(seed, 24, (M, K))
    w = qi.pm1(seed, 25, (N, K))
    T = qi.uniform_int(seed, 26, (N,), -8, 8)  # ties C == T are frequent
    flip = qi.bernoulli_bits(seed, 27, (N,)) if with_flip else None
    want = oracle.pack_bits(oracle.threshold(oracle.gemm_pm1(a, w), T, flip))
    got = run_on_engine(q.qnn_binary_gemm_sign, dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, dev(T),
                          dev(flip) if with_flip else None, engine=engine)
    assert np.array_equal(host_u32(got), want)


@pytest.mark.parametrize("engine", ENGINES)
def test_binary_gemm_sign_extreme_thresholds(seed, engine):
    """Thresholds far outside the range of C (including both int32 ends) must act as always / never."""
    M, N, K = 70, 96, 160
    a = qi.pm1(seed, 28, (M, K))
    w = qi.pm1(seed, 29, (N, K))
    T = qi.uniform_int(seed, 26, (N,), -8, 8)
    T[0::7] = -(2**31)
    T[1::7] = 2**31 - 1
    T[2::7] = -(2**30) - 5
    T[3::7] = 2**30 + 5
    T[4::7] = K      # reachable only by an exact match of all K signs
    T[5::7] = K + 1  # never reached
    flip = qi.bernoulli_bits(seed, 27, (N,))
    want = oracle.pack_bits(oracle.threshold(oracle.gemm_pm1(a, w), T, flip))
    got = run_on_engine(q.qnn_binary_gemm_sign, dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, dev(T), dev(flip),
                          engine=engine)
    assert np.array_equal(host_u32(got), want)


@pytest.mark.parametrize("engine", [2, 3])
@pytest.mark.parametrize("K", [65536, 130000])
def test_binary_gemm_long_k_on_matrix_cores(seed, engine, K):
    """Largest K the matrix-core engine accepts (sums stay exact in int32 / fp32); a != w and a == w rows."""
    M, N = 40, 33
    a = qi.pm1(seed, 30, (M, K))
    w = qi.pm1(seed, 31, (N, K))
    w[0] = a[0]
    w[1] = -a[1]
    got = run_on_engine(q.qnn_binary_gemm, dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, engine=engine)
    assert np.array_equal(host(got), oracle.gemm_pm1(a, w))


# ------------------------------------------------------------------ S3 bitplane_gemm
def _planes_of(v, nbits):
    """integer codes -> ([nbits][rows][K] 0/1 planes from the oracle, packed uint32 planes for the GPU)"""
    p = oracle.split_planes(v, nbits)
    return p, np_pack_bits(p)


@pytest.mark.parametrize("engine", PLANE_ENGINES)
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (9, 11, 100), (70, 130, 784), (130, 70, 33), (256, 512, 800), (300, 260, 1024),
                                   (70, 33, 128)])
def test_bitplane_u8_times_sign(seed, M, N, K, engine):
    x = qi.uniform_int(seed, 30, (M, K), 0, 255)
    w = qi.pm1(seed, 31, (N, K))
    want = oracle.gemm_int(x, w.astype(np.int32))
    _, xp = _planes_of(x, 8)
    got = run_on_engine(q.qnn_bitplane_gemm, dev(xp), [1 << p for p in range(8)], q.PLANE_BIT,
                        dev(np_pack_pm1(w)[None]), [1], q.PLANE_SIGN, K, engine=engine,
                        takes=engine_takes(engine, 8, 1, [1 << p for p in range(8)], row_words=(K + 31) // 32))
    if got is not None:
        assert np.array_equal(host(got), want)
        if engine:
            assert q.qnn_last_engine() == engine


@pytest.mark.parametrize("engine", PLANE_ENGINES)
@pytest.mark.parametrize("M,N,K", [(5, 7, 70), (64, 64, 2048), (150, 200, 257), (300, 520, 384)])
def test_bitplane_int4_times_int4(seed, M, N, K, engine):
    a = qi.uniform_int(seed, 32, (M, K), -8, 7)
    w = qi.uniform_int(seed, 33, (N, K), -8, 7)
    want = oracle.gemm_int(a, w)
    coef = [1, 2, 4, -8]
    _, ap = _planes_of(a, 4)
    _, wp = _planes_of(w, 4)
    got = run_on_engine(q.qnn_bitplane_gemm, dev(ap), coef, q.PLANE_BIT, dev(wp), coef, q.PLANE_BIT, K,
                        engine=engine, takes=engine_takes(engine, 4, 4, coef, coef, row_words=(K + 31) // 32))
    if got is not None:
        assert np.array_equal(host(got), want)


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("modeA,modeW", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_bitplane_every_mode_pair_against_plane_oracle(seed, modeA, modeW, engine):
    M, N, K, Pa, Pb = 37, 45, 333, 3, 2
    pa = qi.bernoulli_bits(seed, 34, (Pa, M, K))
    pw = qi.bernoulli_bits(seed, 35, (Pb, N, K))
    ca, cw = [1, -2, 5], [3, -4]
    want = oracle.gemm_planes(pa, ca, modeA, pw, cw, modeW)
    got = run_on_engine(q.qnn_bitplane_gemm, dev(np_pack_bits(pa)), ca, modeA, dev(np_pack_bits(pw)), cw, modeW, K,
                        engine=engine, takes=engine_takes(engine, Pa, Pb, ca, cw))
    if got is not None:
        assert np.array_equal(host(got), want)


@pytest.mark.parametrize("engine", PLANE_ENGINES)
@pytest.mark.parametrize("modeA,modeW", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("Pa,Pb,ca,cw", [(2, 2, [1, -2], [2, 1]), (4, 1, [1, 2, 4, -8], [-1]), (2, 1, [6, 3], [5]),
                                         (4, 4, [-8, 4, 2, 1], [3, 6, 12, -24]), (8, 1, [1 << p for p in range(7)] + [-128], [7])])
def test_bitplane_every_mode_pair_with_power_of_two_codes(seed, Pa, Pb, ca, cw, modeA, modeW, engine):
    """Coefficient sets the int8 matrix-core engine takes (a common factor times distinct powers of two, either sign,
    any order), in all four mode pairs, so that the affine correction of every pair is exercised on that engine too."""
    M, N, K = 70, 45, 384 if engine == 4 else 333
    pa = qi.bernoulli_bits(seed, 42, (Pa, M, K))
    pw = qi.bernoulli_bits(seed, 43, (Pb, N, K))
    want = oracle.gemm_planes(pa, ca, modeA, pw, cw, modeW)
    got = run_on_engine(q.qnn_bitplane_gemm, dev(np_pack_bits(pa)), ca, modeA, dev(np_pack_bits(pw)), cw, modeW, K,
                        engine=engine, takes=engine_takes(engine, Pa, Pb, ca, cw, row_words=(K + 31) // 32))
    if got is not None:
        assert np.array_equal(host(got), want)
        if engine in (1, 2, 4):
            assert q.qnn_last_engine() == engine


@pytest.mark.parametrize("engine", ENGINES)
def test_bitplane_large_coefficients_fall_back_correctly(seed, engine):
    M, N, K = 20, 24, 90
    pa = qi.bernoulli_bits(seed, 36, (2, M, K))
    pw = qi.bernoulli_bits(seed, 37, (2, N, K))
    ca, cw = [1000, -3], [7, 300]
    want = oracle.gemm_planes(pa, ca, 0, pw, cw, 1)
    got = run_on_engine(q.qnn_bitplane_gemm, dev(np_pack_bits(pa)), ca, 0, dev(np_pack_bits(pw)), cw, 1, K,
                        engine=engine, takes=engine_takes(engine, 2, 2, ca, cw))
    if got is not None:
        assert np.array_equal(host(got), want)


@pytest.mark.parametrize("engine", PLANE_ENGINES)
@pytest.mark.parametrize("K", [784, 896])
def test_bitplane_gemm_sign_first_layer(seed, engine, K):
    M, N = 100, 200
    x = qi.uniform_int(seed, 38, (M, K), 0, 255)
    w = qi.pm1(seed, 39, (N, K))
    T = qi.uniform_int(seed, 40, (N,), -3000, 3000)
    flip = qi.bernoulli_bits(seed, 41, (N,))
    want = oracle.pack_bits(oracle.threshold(oracle.gemm_int(x, w.astype(np.int32)), T, flip))
    _, xp = _planes_of(x, 8)
    got = run_on_engine(q.qnn_bitplane_gemm_sign, dev(xp), [1 << p for p in range(8)], q.PLANE_BIT,
                        dev(np_pack_pm1(w)[None]), [1], q.PLANE_SIGN, K, dev(T), dev(flip), engine=engine,
                        takes=engine_takes(engine, 8, 1, [1 << p for p in range(8)], sign_out=True,
                                           row_words=(K + 31) // 32))
    if got is not None:
        assert np.array_equal(host_u32(got), want)


# ------------------------------------------------------------------ S5 MLP (Alg. 4)
def _mlp_case(seed, batch, dims, stream0, t_hidden=64):
    L = len(dims) - 1
    x = qi.uniform_int(seed, stream0, (batch, dims[0]), 0, 255, dtype=np.uint8)
    W = [qi.pm1(seed, stream0 + 1 + l, (dims[l + 1], dims[l])) for l in range(L)]
    T = [qi.uniform_int(seed, stream0 + 5 + l, (dims[l + 1],), -t_hidden, t_hidden) for l in range(L - 1)]
    return x, W, T


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("batch,dims", [(1, [1, 1, 1]), (37, [50, 70, 33, 10]), (300, [784, 256, 192, 128, 10])])
def test_mlp_forward_small(seed, batch, dims, engine):
    x, W, T = _mlp_case(seed, batch, dims, 50)
    flip = [qi.bernoulli_bits(seed, 60 + l, (dims[l + 1],)) for l in range(len(dims) - 2)]
    want = oracle.mlp(x, W, T, flip)
    got = run_on_engine(q.qnn_binary_mlp_forward, dev(x), 8, dims, [dev(np_pack_pm1(w)) for w in W],
                          [dev(t) for t in T], [dev(f) for f in flip], engine=engine)
    assert np.array_equal(host(got), want)


@pytest.mark.parametrize("engine", [0, 2])
@pytest.mark.parametrize("batch,dims,ldx", [(1100, [784, 2048, 64, 10], 800), (520, [1008, 4096, 10], 1008),
                                            (1030, [16, 2048, 10], 16), (1100, [784, 2048, 64, 10], 788),
                                            (700, [144, 2000, 10], 160), (300, [2064, 1100, 10], 2064),
                                            (2600, [272, 4096, 10], 272), (257, [48, 129, 10], 64)])
def test_mlp_forward_first_layer_from_codes(seed, batch, dims, ldx, engine):
    """Large enough for the matrix-core engine: the first layer reads the 8-bit codes directly when rows are 16-byte
    aligned (ldx a multiple of 16) and falls back to bit planes otherwise; both must give the oracle's logits."""
    x, W, T = _mlp_case(seed, batch, dims, 80, t_hidden=40)
    T[0] = qi.uniform_int(seed, 89, (dims[1],), -3000, 3000)
    flip = [qi.bernoulli_bits(seed, 90 + l, (dims[l + 1],)) for l in range(len(dims) - 2)]
    want = oracle.mlp(x, W, T, flip)
    xb = qi.uniform_int(seed, 95, (batch, ldx), 0, 255, dtype=np.uint8)  # garbage in the row padding
    xb[:, : dims[0]] = x
    xd = dev(xb)[:, : dims[0]]
    got = run_on_engine(q.qnn_binary_mlp_forward, xd, 8, dims, [dev(np_pack_pm1(w)) for w in W],
                          [dev(t) for t in T], [dev(f) for f in flip], engine=engine)
    assert np.array_equal(host(got), want)


# ------------------------------------------------------------------ convolution
def _conv_case(seed, B, H, Wd, Cin, Cout, KH, abits, stream0):
    u = qi.uniform_int(seed, stream0, (B, H, Wd, Cin), 0, (1 << abits) - 1)
    w = qi.pm1(seed, stream0 + 1, (Cout, KH, KH, Cin))
    up = np_pack_bits(oracle.split_planes(u, abits))  # [abits][B][H][W][Cw]
    wp = np_pack_pm1(w)[None]  # [1][Cout][KH][KW][Cw]
    return u, w, up, wp


@pytest.mark.parametrize("engine", PLANE_ENGINES)
@pytest.mark.parametrize("B,H,Wd,Cin,Cout,KH,pad,stride", [(2, 5, 6, 7, 4, 3, 1, 1), (3, 13, 13, 96, 40, 3, 1, 1),
                                                           (2, 8, 7, 40, 33, 5, 2, 2), (1, 4, 4, 64, 8, 1, 0, 1),
                                                           (4, 13, 13, 384, 256, 3, 1, 1), (3, 9, 10, 128, 70, 3, 1, 2)])
def test_conv2d(seed, B, H, Wd, Cin, Cout, KH, pad, stride, engine):
    u, w, up, wp = _conv_case(seed, B, H, Wd, Cin, Cout, KH, 2, 70)
    want = oracle.conv2d(u, w.astype(np.int32), pad, stride)
    got = run_on_engine(q.qnn_bitplane_conv2d, dev(up), [1, 2], q.PLANE_BIT, Cin, dev(wp), [1], q.PLANE_SIGN, pad,
                        stride, engine=engine, takes=engine_takes(engine, 2, 1, [1, 2], conv=True, row_words=(Cin + 31) // 32))
    if got is not None:
        assert np.array_equal(host(got), want)


@pytest.mark.parametrize("engine", PLANE_ENGINES)
@pytest.mark.parametrize("abits,B,H,Wd,Cin,Cout,KH,pad,stride", [(2, 2, 5, 6, 7, 4, 3, 1, 1), (2, 3, 13, 13, 128, 70, 3, 1, 1),
                                                                 (1, 3, 8, 8, 128, 100, 3, 1, 1), (1, 2, 9, 7, 40, 33, 3, 0, 2),
                                                                 (2, 5, 13, 13, 384, 256, 3, 1, 1), (1, 5, 16, 16, 256, 256, 3, 1, 1)])
def test_conv2d_with_fused_threshold(seed, abits, B, H, Wd, Cin, Cout, KH, pad, stride, engine):
    """A layer of a binarized ConvNet: convolution, Sign(BatchNorm(.)) as threshold (ties, flips, extreme values), output
    packed along the channels.  One-bit activations here are 0/1 codes (zero padding is exact for them)."""
    u, w, up, wp = _conv_case(seed, B, H, Wd, Cin, Cout, KH, abits, 74)
    T = qi.uniform_int(seed, 76, (Cout,), -20, 20)
    T[0], T[Cout - 1] = -(2**31), 2**31 - 1
    flip = qi.bernoulli_bits(seed, 77, (Cout,))
    sums = oracle.conv2d(u, w.astype(np.int32), pad, stride)
    Bo, Ho, Wo, _ = sums.shape
    want = oracle.pack_bits(oracle.threshold(sums.reshape(-1, Cout), T, flip)).reshape(Bo, Ho, Wo, -1)
    ca = [1, 2][:abits]
    got = run_on_engine(q.qnn_bitplane_conv2d_sign, dev(up), ca, q.PLANE_BIT, Cin, dev(wp), [1], q.PLANE_SIGN, pad, stride,
                        dev(T), dev(flip), engine=engine,
                        takes=engine_takes(engine, abits, 1, ca, conv=True, sign_out=True, row_words=(Cin + 31) // 32))
    if got is not None:
        assert np.array_equal(host_u32(got), want)
        if engine:
            assert q.qnn_last_engine() == engine


@pytest.mark.parametrize("engine", ENGINES)
def test_conv2d_sign_activations_without_padding(seed, engine):
    B, H, Wd, Cin, Cout = 2, 6, 7, 50, 12
    a = qi.pm1(seed, 72, (B, H, Wd, Cin))
    w = qi.pm1(seed, 73, (Cout, 3, 3, Cin))
    want = oracle.conv2d(a.astype(np.int32), w.astype(np.int32), 0, 1)
    got = run_on_engine(q.qnn_bitplane_conv2d, dev(np_pack_pm1(a)[None]), [1], q.PLANE_SIGN, Cin,
                        dev(np_pack_pm1(w)[None]), [1], q.PLANE_SIGN, 0, 1, engine=engine,
                        takes=engine_takes(engine, 1, 1, conv=True))
    if got is not None:
        assert np.array_equal(host(got), want)


# ------------------------------------------------------------------ degenerate sizes
def test_empty_inputs_are_no_ops():
    e = torch.empty((0, 4), dtype=torch.int32, device="cuda")
    w = torch.zeros((8, 4), dtype=torch.int32, device="cuda")
    assert q.qnn_binary_gemm(e, w, 128).shape == (0, 8)
    assert q.qnn_binary_gemm(w, e, 128).shape == (8, 0)
    assert q.qnn_pack_sign(torch.empty((0, 5), dtype=torch.float32, device="cuda")).shape == (0, 1)
