"""The five benchmark configurations at full size, in the launch configuration the benchmark times (AUTO, with the
engine it picks asserted), and on every other engine that takes them: EVERY output element is compared with the
oracle's.  Further down: whole-output comparisons on shapes with more tiles than the chip has compute units, so that
the persistent kernels' second and later tiles (next tile's operands prefetched during the epilogue, register buffers
re-used) are checked element by element as well."""
import functools

import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi
from qnn_testlib import dev, host, host_u32, np_pack_bits, np_pack_pm1

pytestmark = pytest.mark.gpu

q = None
VALU, MFMA, FP4, MFMA_LDS = 1, 2, 3, 4
# engine AUTO picks per configuration; bench.py reports the same ones
AUTO_ENGINE = {"c1": VALU, "c3": FP4, "c4": MFMA_LDS, "c5": MFMA_LDS}
AUTO_ENGINES_C2 = [MFMA, FP4, FP4, VALU]  # first layer from the 8-bit codes, two hidden layers, 10-neuron output layer


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global q
    assert torch.cuda.is_available()
    import paper_1609_07061_amd as mod

    q = mod
    yield
    torch.cuda.synchronize()


def first_difference(got: np.ndarray, want: np.ndarray) -> str:
    """Names the first differing element (row-major), for the assertion message."""
    if got.shape != want.shape:
        return f"shape {got.shape} != {want.shape}"
    bad = np.argwhere(got != want)
    if bad.size == 0:
        return ""
    i = tuple(int(v) for v in bad[0])
    return f"{len(bad)} of {got.size} elements differ, first at {i}: got {got[i]}, oracle {want[i]}"


def assert_same(got, want):
    assert np.array_equal(got, want), first_difference(got, want)


def check_engine(engine, auto_choice):
    used = q.qnn_last_engine()
    assert used == (engine if engine else auto_choice), f"engine {used} ran, expected {engine or auto_choice}"


# ---------------------------------------------------------------------------------------------------------- C1
@functools.lru_cache(maxsize=None)
def _c1(seed):
    xa, xw = qi.normal_f32(seed, 10, (128, 1024)), qi.normal_f32(seed, 11, (1024, 1024))
    sa, sw = oracle.sign(xa), oracle.sign(xw)
    return xa, xw, sa, sw, oracle.gemm_pm1(sa, sw)


@pytest.mark.parametrize("engine", [0, VALU, MFMA, FP4])
def test_config1_sign_pack_gemm_128x1024x1024(seed, engine):
    """fp32 N(0,1) -> qnn_pack_sign (both operands) -> product; also the Bernoulli +-1 operands packed on the host."""
    xa, xw, sa, sw, want = _c1(seed)
    A, W = q.qnn_pack_sign(dev(xa)), q.qnn_pack_sign(dev(xw))
    assert_same(host_u32(A), oracle.pack_bits(sa))
    assert_same(host_u32(W), oracle.pack_bits(sw))
    assert_same(host(q.qnn_binary_gemm(A, W, 1024, engine=engine)), want)
    check_engine(engine, AUTO_ENGINE["c1"])
    a = qi.pm1(seed, 10, (128, 1024))
    w = qi.pm1(seed, 11, (1024, 1024))
    assert_same(host(q.qnn_binary_gemm(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), 1024, engine=engine)),
                oracle.gemm_pm1(a, w))


# ---------------------------------------------------------------------------------------------------------- C3
@functools.lru_cache(maxsize=None)
def _c3(seed):
    n = 8192
    a = qi.pm1(seed, 30, (n, n))
    w = qi.pm1(seed, 31, (n, n))
    return np_pack_pm1(a), np_pack_pm1(w), oracle.gemm_pm1(a, w)


@pytest.mark.parametrize("engine", [0, FP4, MFMA, VALU])
def test_config3_gemm_8192_cubed_every_element(seed, engine):
    A, W, want = _c3(seed)
    got = host(q.qnn_binary_gemm(dev(A), dev(W), 8192, engine=engine))
    check_engine(engine, AUTO_ENGINE["c3"])
    assert_same(got, want)


def test_config3_plain_entry_point(seed):
    """qnn_binary_gemm itself (no engine argument), as the benchmark calls it."""
    A, W, want = _c3(seed)
    assert_same(host(q.qnn_binary_gemm(dev(A), dev(W), 8192)), want)
    assert q.qnn_last_engine() == AUTO_ENGINE["c3"]


# ---------------------------------------------------------------------------------------------------------- C2
@functools.lru_cache(maxsize=None)
def _c2(seed):
    dims = [784, 4096, 4096, 4096, 10]
    batch = 10000
    x = qi.uniform_int(seed, 20, (batch, 784), 0, 255, dtype=np.uint8)
    W = [qi.pm1(seed, 21 + l, (dims[l + 1], dims[l])) for l in range(4)]
    T = [qi.uniform_int(seed, 25 + l, (dims[l + 1],), -64, 64) for l in range(3)]
    return dims, x, [np_pack_pm1(w) for w in W], T, oracle.mlp(x, W, T)


@pytest.mark.parametrize("engine", [None, MFMA, VALU])
def test_config2_mlp_mnist_shaped_every_logit(seed, engine):
    dims, x, Wp, T, want = _c2(seed)
    got = host(q.qnn_binary_mlp_forward(dev(x), 8, dims, [dev(w) for w in Wp], [dev(t) for t in T], engine=engine))
    if engine is None:
        assert q.qnn_last_engines() == AUTO_ENGINES_C2
    elif engine == VALU:
        assert q.qnn_last_engines() == [VALU] * 4
    assert_same(got, want)


# ---------------------------------------------------------------------------------------------------------- C4
@functools.lru_cache(maxsize=None)
def _c4(seed):
    B, H, Wd, Cin, Cout = 256, 13, 13, 384, 256
    u = qi.uniform_int(seed, 40, (B, H, Wd, Cin), 0, 3)
    w = qi.pm1(seed, 41, (Cout, 3, 3, Cin))
    return np_pack_bits(oracle.split_planes(u, 2)), np_pack_pm1(w)[None], oracle.conv2d(u, w.astype(np.int32), 1, 1)


@pytest.mark.parametrize("engine", [None, MFMA_LDS, MFMA, VALU])
def test_config4_alexnet_conv_every_element(seed, engine):
    up, wp, want = _c4(seed)
    got = host(q.qnn_bitplane_conv2d(dev(up), [1, 2], q.PLANE_BIT, 384, dev(wp), [1], q.PLANE_SIGN, 1, 1, engine=engine))
    check_engine(engine, AUTO_ENGINE["c4"])
    assert_same(got, want)


# ---------------------------------------------------------------------------------------------------------- C5
@functools.lru_cache(maxsize=None)
def _c5(seed):
    M, K, N = 64 * 35, 2048, 4096
    a = qi.uniform_int(seed, 50, (M, K), -8, 7)
    w = qi.uniform_int(seed, 51, (N, K), -8, 7)
    return np_pack_bits(oracle.split_planes(a, 4)), np_pack_bits(oracle.split_planes(w, 4)), oracle.gemm_int(a, w)


@pytest.mark.parametrize("engine", [None, MFMA_LDS, MFMA, VALU])
def test_config5_lstm_gates_int4_every_element(seed, engine):
    ap, wp, want = _c5(seed)
    coef = [1, 2, 4, -8]
    got = host(q.qnn_bitplane_gemm(dev(ap), coef, q.PLANE_BIT, dev(wp), coef, q.PLANE_BIT, 2048, engine=engine))
    check_engine(engine, AUTO_ENGINE["c5"])
    assert_same(got, want)


# ------------------------------------------------------------------------- more tiles than compute units, whole output
@pytest.mark.parametrize("engine", [0, MFMA, FP4])
@pytest.mark.parametrize("M,N,ldc", [(4200, 4200, 4200), (4200, 4197, 4197), (4104, 4360, 4400)])
def test_large_ragged_gemm_interior_and_edge_tiles(seed, M, N, ldc, engine):
    """K = 8192 and ragged edges: interior tiles take the whole-line store path (when the row pitch allows it), edge
    tiles the bounds-checked one, in the same launch; 289 to 306 tiles on 256 persistent workgroups."""
    K = 8192
    a = qi.pm1(seed, 60, (M, K))
    w = qi.pm1(seed, 61, (N, K))
    out = torch.full((M, ldc), -7, dtype=torch.int32, device="cuda")
    q.qnn_binary_gemm(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, out=out[:, :N], engine=engine)
    check_engine(engine, FP4)
    got = host(out)
    assert (got[:, N:] == -7).all()
    assert_same(got[:, :N], oracle.gemm_pm1(a, w))


MANY_TILES = [(4200, 4360, 256), (4360, 4104, 320), (4104, 4200, 800)]


@pytest.mark.parametrize("engine", [0, MFMA, FP4])
@pytest.mark.parametrize("M,N,K", MANY_TILES)
def test_many_tiles_short_k_int32_output(seed, M, N, K, engine):
    """17 x 18 tiles and short K: tile changes (prefetch across the epilogue, buffer re-use) dominate."""
    a = qi.pm1(seed, 64, (M, K))
    w = qi.pm1(seed, 65, (N, K))
    ldc = N + 4 * (K % 7)  # a padded row pitch in two of the three cases
    out = torch.full((M, ldc), -7, dtype=torch.int32, device="cuda")
    q.qnn_binary_gemm(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, out=out[:, :N], engine=engine)
    check_engine(engine, FP4)
    got = host(out)
    assert (got[:, N:] == -7).all()
    assert_same(got[:, :N], oracle.gemm_pm1(a, w))


@pytest.mark.parametrize("engine", [0, MFMA, FP4])
@pytest.mark.parametrize("M,N,K", MANY_TILES)
def test_many_tiles_short_k_threshold_output(seed, M, N, K, engine):
    a = qi.pm1(seed, 66, (M, K))
    w = qi.pm1(seed, 67, (N, K))
    T = qi.uniform_int(seed, 68, (N,), -10, 10)
    flip = qi.bernoulli_bits(seed, 69, (N,))
    ldo = (N + 31) // 32 + 3
    out = torch.full((M, ldo), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_binary_gemm_sign(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, dev(T), dev(flip), out=out[:, :ldo - 3],
                           engine=engine)
    check_engine(engine, FP4)
    got = host_u32(out)
    assert (got[:, ldo - 3:] == 0x5A5A5A5A).all()
    assert_same(got[:, :ldo - 3], oracle.pack_bits(oracle.threshold(oracle.gemm_pm1(a, w), T, flip)))


# K a multiple of 1024 and 16-byte aligned rows: the kernel that is fed from LDS panels.  (4000, 8100): 16 x 32 tiles of
# 256 x 256, two per workgroup, ragged on both edges; (4200, 4360): 17 x 35 tiles of 256 x 128 (chosen because 17 x 18
# large tiles would leave 40 % of the second round idle); (1000, 700): fewer tiles than workgroups, three groups of K;
# (6000, 8500): 24 x 34 tiles, three or four per workgroup; (5000, 7000) with K = 4096: 20 x 28 = 560 tiles of
# 256 x 256, two whole rounds of 256 workgroups and 48 tiles that are halved and shared out among 96 workgroups.
# (9000, 128, 2048): 128 columns, which 256-column tiles would pad to twice the work: 36 tiles of 256 x 128.
PANEL_TILES = [(4000, 8100, 1024), (4200, 4360, 2048), (1000, 700, 3072), (6000, 8500, 1024), (5000, 7000, 4096),
               (9000, 128, 2048)]


@pytest.mark.parametrize("engine", [0, FP4])
@pytest.mark.parametrize("M,N,K", PANEL_TILES)
def test_panel_fed_kernel_int32_output(seed, M, N, K, engine):
    a = qi.pm1(seed, 74, (M, K))
    w = qi.pm1(seed, 75, (N, K))
    ldc = N + 4 * (K // 1024 - 1)
    out = torch.full((M, ldc), -7, dtype=torch.int32, device="cuda")
    q.qnn_binary_gemm(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, out=out[:, :N], engine=engine)
    check_engine(engine, FP4 if M >= 4000 else 1)
    got = host(out)
    assert (got[:, N:] == -7).all()
    assert_same(got[:, :N], oracle.gemm_pm1(a, w))


@pytest.mark.parametrize("engine", [0, FP4])
@pytest.mark.parametrize("M,N,K", PANEL_TILES)
def test_panel_fed_kernel_threshold_output(seed, M, N, K, engine):
    a = qi.pm1(seed, 76, (M, K))
    w = qi.pm1(seed, 77, (N, K))
    T = qi.uniform_int(seed, 78, (N,), -20, 20)
    flip = qi.bernoulli_bits(seed, 79, (N,))
    ldo = (N + 31) // 32 + 2
    out = torch.full((M, ldo), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_binary_gemm_sign(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, dev(T), dev(flip), out=out[:, :ldo - 2],
                           engine=engine)
    check_engine(engine, FP4 if M >= 4000 else 1)
    got = host_u32(out)
    assert (got[:, ldo - 2:] == 0x5A5A5A5A).all()
    assert_same(got[:, :ldo - 2], oracle.pack_bits(oracle.threshold(oracle.gemm_pm1(a, w), T, flip)))


@pytest.mark.parametrize("engine", [None, MFMA])
def test_many_tiles_first_layer_from_codes(seed, engine):
    """The byte-operand kernel of the MLP's first layer over 17 x 17 tiles, then a 10-neuron output layer."""
    batch, dims = 4200, [784, 4200, 10]
    x = qi.uniform_int(seed, 70, (batch, 784), 0, 255, dtype=np.uint8)
    W = [qi.pm1(seed, 71 + l, (dims[l + 1], dims[l])) for l in range(2)]
    T = [qi.uniform_int(seed, 73, (dims[1],), -3000, 3000)]
    flip = [qi.bernoulli_bits(seed, 74, (dims[1],))]
    got = host(q.qnn_binary_mlp_forward(dev(x), 8, dims, [dev(np_pack_pm1(w)) for w in W], [dev(t) for t in T],
                                        [dev(f) for f in flip], engine=engine))
    assert q.qnn_last_engines()[0] == MFMA
    assert_same(got, oracle.mlp(x, W, T, flip))


@pytest.mark.parametrize("engine", [None, MFMA_LDS, MFMA])
def test_many_tiles_first_layer_planes_threshold_output(seed, engine):
    """Eight input planes x one weight plane with the fused threshold (the plane fall-back of the first layer)."""
    M, N, K = 4200, 4200, 384
    x = qi.uniform_int(seed, 75, (M, K), 0, 255)
    w = qi.pm1(seed, 76, (N, K))
    T = qi.uniform_int(seed, 77, (N,), -1500, 1500)
    xp = np_pack_bits(oracle.split_planes(x, 8))
    kw = {} if engine is None else {"engine": engine}
    got = q.qnn_bitplane_gemm_sign(dev(xp), [1 << p for p in range(8)], q.PLANE_BIT, dev(np_pack_pm1(w)[None]), [1],
                                   q.PLANE_SIGN, K, dev(T), None, **kw)
    check_engine(engine or 0, MFMA_LDS)
    assert_same(host_u32(got), oracle.pack_bits(oracle.threshold(oracle.gemm_int(x, w.astype(np.int32)), T)))


@pytest.mark.parametrize("engine", [None, MFMA_LDS, MFMA])
def test_many_tiles_int4_times_int4(seed, engine):
    M, N, K = 4200, 4360, 256
    a = qi.uniform_int(seed, 78, (M, K), -8, 7)
    w = qi.uniform_int(seed, 79, (N, K), -8, 7)
    coef = [1, 2, 4, -8]
    got = q.qnn_bitplane_gemm(dev(np_pack_bits(oracle.split_planes(a, 4))), coef, q.PLANE_BIT,
                              dev(np_pack_bits(oracle.split_planes(w, 4))), coef, q.PLANE_BIT, K, engine=engine)
    check_engine(engine or 0, MFMA_LDS)
    assert_same(host(got), oracle.gemm_int(a, w))


# Large products of multi-plane operands with int32 output: the library merges the planes of both operands to int8
# values once per call and multiplies bytes.  Coefficients with a common factor that is not a power of two, both plane
# modes, eight planes, K that is not a multiple of 32, ragged tiles on both edges.
MERGED = [(1100, 1000, 2000, [3, -6, 15], 1, [5, 10], 0),
          (1300, 1400, 1237, [1, 2, 4, 8, 16, 32, 64, -128], 0, [1], 1),
          (2100, 1300, 800, [1, 2, 4, -8], 0, [-7, 2, 1], 1),
          (1024, 1024, 2048, [64, 32, 16], 1, [1, 2], 0),
          (2100, 1100, 1050, [1, 2, -4], 0, [1, -2], 0)]   # K ends in the first half of its last group of 128


@pytest.mark.parametrize("engine", [None, MFMA_LDS])
@pytest.mark.parametrize("M,N,K,ca,modeA,cw,modeW", MERGED)
def test_large_multi_plane_products_merged_to_bytes(seed, M, N, K, ca, modeA, cw, modeW, engine):
    pa = qi.bernoulli_bits(seed, 86, (len(ca), M, K))
    pw = qi.bernoulli_bits(seed, 87, (len(cw), N, K))
    want = oracle.gemm_planes(pa, ca, modeA, pw, cw, modeW)
    # padded row pitches, plane strides beyond the rows used, padded output pitch
    Kw = (K + 31) // 32
    A = dev(np_pack_bits(np.concatenate([pa, pa[:, :3]], axis=1), Kw + 3))[:, :M, :Kw]
    W = dev(np_pack_bits(np.concatenate([pw, pw[:, :2]], axis=1), Kw + 1))[:, :N, :Kw]
    out = torch.full((M, N + 5), -7, dtype=torch.int32, device="cuda")
    q.qnn_bitplane_gemm(A, ca, modeA, W, cw, modeW, K, out=out[:, :N], engine=engine)
    if engine is not None:
        check_engine(engine, MFMA_LDS)
    got = host(out)
    assert (got[:, N:] == -7).all()
    assert_same(got[:, :N], want)


def test_large_multi_plane_product_whose_values_exceed_a_byte(seed):
    """127 b0 + 2 b1 reaches 129: no int8 value and no power-of-two code, so the library's choice falls on another
    engine, with the same result."""
    M, N, K = 1100, 1000, 2000
    pa = qi.bernoulli_bits(seed, 88, (2, M, K))
    pw = qi.bernoulli_bits(seed, 89, (2, N, K))
    ca, cw = [127, 2], [1, -1]
    want = oracle.gemm_planes(pa, ca, 0, pw, cw, 1)
    got = q.qnn_bitplane_gemm(dev(np_pack_bits(pa)), ca, 0, dev(np_pack_bits(pw)), cw, 1, K)
    assert_same(host(got), want)
    with pytest.raises(q.QnnError):
        q.qnn_bitplane_gemm(dev(np_pack_bits(pa)), ca, 0, dev(np_pack_bits(pw)), cw, 1, K, engine=MFMA_LDS)


@pytest.mark.parametrize("Cin,auto", [(64, MFMA), (128, MFMA_LDS)])
@pytest.mark.parametrize("engine", [None, MFMA])
def test_many_tiles_conv(seed, engine, Cin, auto):
    """26 images of 13 x 13 pixels, 64 or 128 -> 4200 channels: 18 x 17 tiles of the implicit-im2col kernels (128
    channels are four words per pixel, which AUTO gives to the kernel that merges the planes in LDS)."""
    B, H, Wd, Cout = 26, 13, 13, 4200
    u = qi.uniform_int(seed, 80, (B, H, Wd, Cin), 0, 3)
    w = qi.pm1(seed, 81, (Cout, 3, 3, Cin))
    got = q.qnn_bitplane_conv2d(dev(np_pack_bits(oracle.split_planes(u, 2))), [1, 2], q.PLANE_BIT, Cin,
                                dev(np_pack_pm1(w)[None]), [1], q.PLANE_SIGN, 1, 1, engine=engine)
    check_engine(engine or 0, auto)
    assert_same(host(got), oracle.conv2d(u, w.astype(np.int32), 1, 1))
