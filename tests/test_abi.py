"""CPU-side checks of the C ABI: the built library loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qnn_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_1609_07061_amd as q

    lib = C.CDLL(q.LIB_PATH)
    names = _declared_symbols()
    assert len(names) >= 20
    for five in ('qnn_pack_sign', 'qnn_binary_gemm', 'qnn_bitplane_gemm', 'qnn_threshold_sign', 'qnn_binary_mlp_forward'):
        assert five in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in qnn.h but not exported"
    assert sorted(q.EXPORTS) == names
    assert "gfx950" in q.qnn_version()


@pytest.fixture(scope="module")
def lib():
    import paper_1609_07061_amd as q

    return q._lib


FAKE = 0x1000  # a non-NULL, 4-byte aligned address that is never dereferenced: every call below fails validation first
ONE = (C.c_int32 * 1)(1)


def _err(lib):
    return lib.qnn_last_error().decode()


def test_pack_sign_argument_errors(lib):
    assert lib.qnn_pack_sign(None, 4, 8, 8, FAKE, 1, None) == 1
    assert lib.qnn_pack_sign(FAKE, 4, 0, 8, FAKE, 1, None) == 2
    assert lib.qnn_pack_sign(FAKE, 4, 64, 32, FAKE, 2, None) == 2  # ldx < K
    assert lib.qnn_pack_sign(FAKE, 4, 64, 64, FAKE, 1, None) == 2  # ldo < ceil(K/32)
    assert lib.qnn_pack_sign(FAKE + 2, 4, 64, 64, FAKE, 2, None) == 3
    assert "aligned" in _err(lib)
    assert lib.qnn_pack_sign(None, 0, 8, 8, None, 1, None) == 0  # rows == 0: no-op


def test_pack_bitplanes_argument_errors(lib):
    assert lib.qnn_pack_bitplanes(FAKE, 4, 8, 8, 0, FAKE, 1, 4, None) == 2
    assert lib.qnn_pack_bitplanes(FAKE, 4, 8, 8, 9, FAKE, 1, 4, None) == 2
    assert lib.qnn_pack_bitplanes(None, 4, 8, 8, 8, FAKE, 1, 4, None) == 1
    assert lib.qnn_pack_bitplanes(FAKE, 4, 40, 40, 2, FAKE, 1, 4, None) == 2


def test_binary_gemm_argument_errors(lib):
    f = lib.qnn_binary_gemm
    assert f(None, 1, FAKE, 1, FAKE, 4, 4, 4, 32, None) == 1
    assert f(FAKE, 1, FAKE, 1, None, 4, 4, 4, 32, None) == 1
    assert f(FAKE, 1, FAKE, 1, FAKE, 4, 4, 4, 0, None) == 2  # K < 1
    assert f(FAKE, 1, FAKE, 1, FAKE, 4, 4, 4, 33, None) == 2  # lda < ceil(K/32)
    assert f(FAKE, 2, FAKE, 2, FAKE, 3, 4, 4, 33, None) == 2  # ldc < N
    assert f(FAKE, 1, FAKE, 1, FAKE, 4, -1, 4, 32, None) == 2
    assert f(FAKE + 1, 1, FAKE, 1, FAKE, 4, 4, 4, 32, None) == 3
    assert f(None, 1, None, 1, None, 4, 0, 4, 32, None) == 0  # M == 0: no-op
    assert lib.qnn_binary_gemm_ex(FAKE, 1, FAKE, 1, FAKE, 4, 4, 4, 32, 7, None) == 2  # unknown engine
    assert lib.qnn_binary_gemm_sign(FAKE, 1, FAKE, 1, None, None, FAKE, 1, 4, 4, 32, 0, None) == 1  # T is NULL
    assert lib.qnn_binary_gemm_sign(FAKE, 1, FAKE, 1, FAKE, None, FAKE, 1, 4, 40, 32, 0, None) == 2  # ldo too small


def test_bitplane_gemm_argument_errors(lib):
    f = lib.qnn_bitplane_gemm_ex
    plain = lib.qnn_bitplane_gemm
    assert plain(FAKE, 0, ONE, 0, 1, 4, FAKE, 1, ONE, 1, 1, 0, FAKE, 4, 4, 4, 32, None) == 2  # no engine argument here
    assert plain(None, 1, ONE, 0, 1, 4, None, 1, ONE, 1, 1, 0, None, 4, 0, 4, 32, None) == 0  # M == 0
    assert f(FAKE, 1, ONE, 0, 1, 4, FAKE, 1, ONE, 1, 1, 0, FAKE, 4, 4, 4, 32, 9, None) == 2  # unknown engine
    c8 = (C.c_int32 * 8)(1, 2, 4, 8, 16, 32, 64, 128)
    assert f(FAKE, 0, c8, 0, 1, 4, FAKE, 1, ONE, 1, 1, 0, FAKE, 4, 4, 4, 32, 0, None) == 2
    assert f(FAKE, 9, c8, 0, 1, 4, FAKE, 1, ONE, 1, 1, 0, FAKE, 4, 4, 4, 32, 0, None) == 2
    assert f(FAKE, 8, None, 0, 1, 4, FAKE, 1, ONE, 1, 1, 0, FAKE, 4, 4, 4, 32, 0, None) == 1
    assert f(FAKE, 8, c8, 2, 1, 4, FAKE, 1, ONE, 1, 1, 0, FAKE, 4, 4, 4, 32, 0, None) == 2  # bad mode
    # int32 range: 255 * 1 * K must stay below 2^31
    big = (C.c_int32 * 2)(2**30, 2**30)
    K = 64
    assert f(FAKE, 2, big, 0, 2, 8, FAKE, 1, ONE, 1, 2, 0, FAKE, 4, 4, 4, K, 0, None) == 4
    assert "int32" in _err(lib)
    Kbig = 2**31 - 1
    Kw = (Kbig + 31) // 32
    assert f(FAKE, 8, c8, 0, Kw, 4 * Kw, FAKE, 1, ONE, 1, Kw, 0, FAKE, 4, 4, 4, Kbig, 0, None) == 4


def test_threshold_argument_errors(lib):
    f = lib.qnn_threshold_sign
    assert f(None, 4, 4, 4, FAKE, None, FAKE, 1, None) == 1
    assert f(FAKE, 4, 4, 4, None, None, FAKE, 1, None) == 1
    assert f(FAKE, 3, 4, 4, FAKE, None, FAKE, 1, None) == 2
    assert f(FAKE, 40, 4, 40, FAKE, None, FAKE, 1, None) == 2
    assert f(FAKE, 4, 0, 4, FAKE, None, FAKE, 1, None) == 0


def test_mlp_argument_errors(lib):
    import paper_1609_07061_amd as q

    dims = (C.c_int64 * 4)(784, 64, 64, 10)
    need = q.qnn_binary_mlp_workspace_bytes(100, 8, [784, 64, 64, 10])
    assert need > 0 and need % 256 == 0
    assert q.qnn_binary_mlp_workspace_bytes(100, 9, [784, 64, 64, 10]) == 0
    Wp = (C.c_void_p * 3)(FAKE, FAKE, FAKE)
    Tp = (C.c_void_p * 2)(FAKE, FAKE)
    f = lib.qnn_binary_mlp_forward
    assert f(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, None, 0, None) == 6  # no workspace
    assert f(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10000, need - 1, None) == 6  # too small
    assert f(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10010, need, None) == 6  # misaligned
    assert f(FAKE, 100, 784, 8, 1, dims, Wp, Tp, None, FAKE, 10, 0x10000, need, None) == 2  # n_layers < 2
    assert f(FAKE, 100, 700, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10000, need, None) == 2  # in_dim != dims[0]
    assert f(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 9, 0x10000, need, None) == 2  # ld_logits
    Wbad = (C.c_void_p * 3)(FAKE, None, FAKE)
    assert f(FAKE, 100, 784, 8, 3, dims, Wbad, Tp, None, FAKE, 10, 0x10000, need, None) == 1
    assert f(None, 0, 784, 8, 3, dims, Wp, Tp, None, None, 10, None, 0, None) == 0  # batch 0
    g = lib.qnn_binary_mlp_forward_ex
    assert g(FAKE, 100, 700, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10000, need, 0, None) == 2  # ldx < dims[0]
    assert g(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10000, need, 9, None) == 2  # unknown engine


def test_mlp_validates_every_layer_before_the_first_launch(lib):
    """A fault in a LATER layer (here: a misaligned weight pointer of the last layer, a misaligned threshold pointer
    of the second) is reported without anything having been enqueued: the addresses are fake, so a launch of the
    first layer would have been a GPU fault on a GPU machine, and on a CPU-only box a HIP error (status 7) instead of the
    argument error."""
    import paper_1609_07061_amd as q

    dims = (C.c_int64 * 4)(784, 64, 64, 10)
    need = q.qnn_binary_mlp_workspace_bytes(100, 8, [784, 64, 64, 10])
    f = lib.qnn_binary_mlp_forward
    Wp = (C.c_void_p * 3)(FAKE, FAKE, FAKE + 2)
    Tp = (C.c_void_p * 2)(FAKE, FAKE)
    assert f(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10000, need, None) == 3
    assert "aligned" in _err(lib)
    Wp = (C.c_void_p * 3)(FAKE, FAKE, FAKE)
    Tp = (C.c_void_p * 2)(FAKE, FAKE + 1)
    assert f(FAKE, 100, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, 0x10000, need, None) == 3
    # a first layer whose sums cannot fit int32: 255 * 2^24 inputs
    big = (C.c_int64 * 3)(1 << 24, 64, 10)
    Wp2 = (C.c_void_p * 2)(FAKE, FAKE)
    Tp1 = (C.c_void_p * 1)(FAKE)
    need2 = q.qnn_binary_mlp_workspace_bytes(4, 8, [1 << 24, 64, 10])
    assert f(FAKE, 4, 1 << 24, 8, 2, big, Wp2, Tp1, None, FAKE, 10, 0x10000, need2, None) == 4


def test_static_scratch_entry_point_argument_errors(lib):
    """The entry point for callers that cannot allocate refuses what does not fit its built-in 32 MiB array, and
    validates like qnn_binary_mlp_forward; nothing here reaches the GPU."""
    import paper_1609_07061_amd as q

    assert q.qnn_static_scratch_bytes() == 32 << 20
    f = lib.qnn_binary_mlp_forward_static
    dims = (C.c_int64 * 4)(784, 4096, 4096, 10)
    Wp = (C.c_void_p * 3)(FAKE, FAKE, FAKE)
    Tp = (C.c_void_p * 2)(FAKE, FAKE)
    assert q.qnn_binary_mlp_workspace_bytes(10000, 8, [784, 4096, 4096, 10]) <= 32 << 20
    assert q.qnn_binary_mlp_workspace_bytes(40000, 8, [784, 4096, 4096, 10]) > 32 << 20
    assert f(FAKE, 40000, 784, 8, 3, dims, Wp, Tp, None, FAKE, 10, None) == 6
    assert "built-in" in _err(lib)
    assert f(FAKE, 100, 700, 8, 3, dims, Wp, Tp, None, FAKE, 10, None) == 2  # in_dim != dims[0]
    assert f(None, 0, 784, 8, 3, dims, Wp, Tp, None, None, 10, None) == 0  # batch 0: no-op, the array is not touched


def test_conv_argument_errors(lib):
    f = lib.qnn_bitplane_conv2d_ex
    assert lib.qnn_bitplane_conv2d(None, 2, None, 0, 100, 0, 5, 5, 32, None, 1, ONE, 1, 0, 4, 3, 3, 1, 1, None, None) == 1
    c2 = (C.c_int32 * 2)(1, 2)
    ok = [FAKE, 2, c2, 0, 100, 1, 5, 5, 32, FAKE, 1, ONE, 1, 0, 4, 3, 3, 1, 1, FAKE, 0, None]

    def call(**kw):
        names = ["A", "Pa", "coefA", "modeA", "sA", "B", "H", "W", "Cin", "Wt", "Pb", "coefW", "modeW", "sW", "Cout",
                 "KH", "KW", "pad", "stride", "out", "engine", "stream"]
        a = list(ok)
        for k, v in kw.items():
            a[names.index(k)] = v
        return f(*a)

    assert call(A=None) == 1
    assert call(stride=0) == 2
    assert call(KH=9, pad=0) == 2  # kernel larger than image
    assert call(modeA=1) == 5  # sign-mode activations cannot be zero padded
    assert call(B=0) == 0
    assert call(pad=40000) == 2  # padding beyond the supported range
    assert call(engine=9) == 2


def test_fold_batchnorm_matches_float_definition():
    """Host helper of the product against the oracle's direct evaluation of Sign(BatchNorm(s)) in double."""
    import oracle
    import paper_1609_07061_amd as q
    import qnn_inputs as qi

    n = 64
    seed = qi.SEED_BASE
    g = qi.normal_f32(seed, 60, (n,)).astype(np.float64)
    g[:4] = [0.0, 0.0, 1e-3, -1e-3]
    b = qi.normal_f32(seed, 61, (n,)).astype(np.float64) * 2
    b[0], b[1] = 0.7, -0.7
    mu = qi.normal_f32(seed, 62, (n,)).astype(np.float64) * 30
    var = np.abs(qi.normal_f32(seed, 63, (n,)).astype(np.float64)) * 100 + 0.1
    eps = 1e-4
    T, flip = q.qnn_fold_batchnorm(g, b, mu, var, eps)
    s = np.arange(-400, 401, dtype=np.int32)
    Cm = np.repeat(s[:, None], n, axis=1)
    want = oracle.bn_sign(Cm, g, b, mu, var, eps)
    got = oracle.threshold(Cm, T, flip)
    # exclude the measure-zero set where the float formula is within rounding of 0
    y = g * (Cm - mu) / np.sqrt(var + eps) + b
    safe = np.abs(y) > 1e-9
    assert np.array_equal(got[safe], want[safe])
    assert T[0] == -(2**31) and flip[0] == 0 and T[1] == -(2**31) and flip[1] == 1
    assert set(flip[2:].tolist()) == {0, 1}
    assert np.array_equal(flip[2:], (g[2:] < 0).astype(np.uint8))


def test_fold_batchnorm_saturates():
    import oracle
    import paper_1609_07061_amd as q

    g = np.array([1e-12, -1e-12, 1e-12, -1e-12])
    b = np.array([1.0, 1.0, -1.0, -1.0])
    T, flip = q.qnn_fold_batchnorm(g, b, np.zeros(4), np.ones(4), 0.0)
    Cm = np.array([[-(2**31), 0, 2**31 - 1]] * 1, dtype=np.int32).T.repeat(4, axis=1)
    want = oracle.bn_sign(Cm, g, b, np.zeros(4), np.ones(4), 0.0)
    assert np.array_equal(oracle.threshold(Cm, T, flip), want)
