"""ctypes front end of the CPU oracle (test infrastructure: only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product never does).

Every function takes and returns numpy arrays of UNPACKED values and forwards to the plain C loops in
qnn_oracle.c; there is no arithmetic in this file beyond dtype/shape marshalling.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qnn_oracle.c")
# QNN_ORACLE_SANITIZE=1: a second build with the undefined-behaviour sanitizer (signed overflow, shifts, bounds of
# arrays with known size, alignment), every finding fatal; `QNN_ORACLE_SANITIZE=1 pytest tests -m "not gpu"` runs the
# pins on it.  (The address sanitizer would have to be preloaded into the interpreter and is not used.)
_SANITIZE = os.environ.get("QNN_ORACLE_SANITIZE", "") not in ("", "0")
_SO = os.path.join(_HERE, "libqnn_oracle_ubsan.so" if _SANITIZE else "libqnn_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over output rows)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"] if _SANITIZE else ["-O3", "-march=native"]
        cmd = ["gcc", "-std=c11", *opt, "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
    return _lib


class OracleRangeError(ArithmeticError):
    pass


def _check(rc: int, what: str):
    if rc == 1:
        raise OracleRangeError(f"{what}: a result does not fit int32")
    if rc != 0:
        raise RuntimeError(f"{what}: oracle returned {rc}")


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def sign(x: np.ndarray) -> np.ndarray:
    x = _c(x, np.float32)
    s = np.empty(x.shape, dtype=np.int8)
    _check(lib().qo_sign(_p(x), C.c_int64(x.size), _p(s)), "sign")
    return s


def pack_bits(s: np.ndarray) -> np.ndarray:
    """[rows][K] int8 (+1/-1 or 1/0) -> [rows][ceil(K/32)] uint32, element 32j+t at bit t of word j."""
    s = _c(s, np.int8)
    rows, K = s.shape
    out = np.zeros((rows, (K + 31) // 32), dtype=np.uint32)
    _check(lib().qo_pack_bits(_p(s), C.c_int64(rows), C.c_int64(K), _p(out)), "pack_bits")
    return out


def split_planes(v: np.ndarray, nbits: int) -> np.ndarray:
    v = _c(v, np.int32)
    out = np.empty((nbits,) + v.shape, dtype=np.uint8)
    _check(lib().qo_split_planes(_p(v), C.c_int64(v.size), C.c_int(nbits), _p(out)), "split_planes")
    return out


def gemm_pm1(a: np.ndarray, w: np.ndarray) -> np.ndarray:
    a = _c(a, np.int8)
    w = _c(w, np.int8)
    M, K = a.shape
    N, K2 = w.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.int32)
    _check(lib().qo_gemm_pm1(_p(a), _p(w), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(out)), "gemm_pm1")
    return out


def gemm_int(u: np.ndarray, v: np.ndarray) -> np.ndarray:
    u = _c(u, np.int32)
    v = _c(v, np.int32)
    M, K = u.shape
    N, K2 = v.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.int32)
    _check(lib().qo_gemm_int(_p(u), _p(v), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(out)), "gemm_int")
    return out


def gemm_planes(pa, ca, mode_a: int, pw, cw, mode_w: int) -> np.ndarray:
    pa = _c(pa, np.uint8)
    pw = _c(pw, np.uint8)
    ca = _c(ca, np.int32)
    cw = _c(cw, np.int32)
    Pa, M, K = pa.shape
    Pb, N, K2 = pw.shape
    assert K == K2 and ca.size == Pa and cw.size == Pb
    out = np.empty((M, N), dtype=np.int32)
    rc = lib().qo_gemm_planes(_p(pa), C.c_int(Pa), _p(ca), C.c_int(mode_a), _p(pw), C.c_int(Pb), _p(cw),
                              C.c_int(mode_w), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(out))
    _check(rc, "gemm_planes")
    return out


def threshold(Cm: np.ndarray, T: np.ndarray, flip=None) -> np.ndarray:
    Cm = _c(Cm, np.int32)
    T = _c(T, np.int32)
    M, N = Cm.shape
    assert T.size == N
    f = None if flip is None else _c(flip, np.uint8)
    out = np.empty((M, N), dtype=np.int8)
    _check(lib().qo_threshold(_p(Cm), C.c_int64(M), C.c_int64(N), _p(T), _p(f) if f is not None else None,
                              _p(out)), "threshold")
    return out


def bn_sign(Cm, gamma, beta, mean, var, eps: float) -> np.ndarray:
    Cm = _c(Cm, np.int32)
    M, N = Cm.shape
    g, b, mu, v = (_c(t, np.float64) for t in (gamma, beta, mean, var))
    out = np.empty((M, N), dtype=np.int8)
    _check(lib().qo_bn_sign(_p(Cm), C.c_int64(M), C.c_int64(N), _p(g), _p(b), _p(mu), _p(v), C.c_double(eps),
                            _p(out)), "bn_sign")
    return out


def mlp(x: np.ndarray, W: list, T: list, flip: list | None = None) -> np.ndarray:
    """x uint8 [batch][dims[0]]; W[l] int8 +-1 [dims[l+1]][dims[l]]; T[l] int32 [dims[l+1]] for l < L-1."""
    x = _c(x, np.uint8)
    L = len(W)
    Ws = [_c(w, np.int8) for w in W]
    Ts = [_c(t, np.int32) for t in T]
    assert len(Ts) == L - 1
    dims = np.array([x.shape[1]] + [w.shape[0] for w in Ws], dtype=np.int64)
    for l, w in enumerate(Ws):
        assert w.shape[1] == dims[l]
    Wp = (C.c_void_p * L)(*[w.ctypes.data for w in Ws])
    Tp = (C.c_void_p * max(L - 1, 1))(*[t.ctypes.data for t in Ts])
    if flip is None:
        Fp = None
        Fs = []
    else:
        Fs = [_c(f, np.uint8) for f in flip]
        Fp = (C.c_void_p * max(L - 1, 1))(*[f.ctypes.data for f in Fs])
    out = np.empty((x.shape[0], int(dims[-1])), dtype=np.int32)
    rc = lib().qo_mlp(_p(x), C.c_int64(x.shape[0]), C.c_int(L), _p(dims), Wp, Tp, Fp, _p(out))
    _check(rc, "mlp")
    return out


def conv2d(u: np.ndarray, w: np.ndarray, pad: int, stride: int = 1) -> np.ndarray:
    """u int [B][H][W][Ci], w int [Co][KH][KW][Ci] -> int32 [B][Ho][Wo][Co], zero padding."""
    u = _c(u, np.int32)
    w = _c(w, np.int32)
    B, H, Wd, Ci = u.shape
    Co, KH, KW, Ci2 = w.shape
    assert Ci == Ci2
    Ho = (H + 2 * pad - KH) // stride + 1
    Wo = (Wd + 2 * pad - KW) // stride + 1
    out = np.empty((B, Ho, Wo, Co), dtype=np.int32)
    rc = lib().qo_conv2d(_p(u), C.c_int64(B), C.c_int64(H), C.c_int64(Wd), C.c_int64(Ci), _p(w), C.c_int64(Co),
                         C.c_int64(KH), C.c_int64(KW), C.c_int64(pad), C.c_int64(stride), _p(out))
    _check(rc, "conv2d")
    return out


def maxpool2x2(u: np.ndarray) -> np.ndarray:
    """int [B][H][W][C] -> int32 [B][H//2][W//2][C]."""
    u = _c(u, np.int32)
    B, H, Wd, Cc = u.shape
    out = np.empty((B, H // 2, Wd // 2, Cc), dtype=np.int32)
    _check(lib().qo_maxpool2x2(_p(u), C.c_int64(B), C.c_int64(H), C.c_int64(Wd), C.c_int64(Cc), _p(out)), "maxpool2x2")
    return out


def convnet(x: np.ndarray, conv_w: list, pool: list, fc_w: list, T: list, flip: list | None = None) -> np.ndarray:
    """x uint8 [B][H][W][C0]; conv_w[l] int8 +-1 [cout][3][3][cin]; pool[l] 0/1; fc_w[j] int8 +-1 [out][in] with `in`
    of the first one counting the last feature map in (y, x, c) order; T[l] int32 for every layer but the last."""
    x = _c(x, np.uint8)
    B, H, Wd, C0 = x.shape
    Ws = [_c(w, np.int8) for w in list(conv_w) + list(fc_w)]
    L = len(Ws)
    Ts = [_c(t, np.int32) for t in T]
    assert len(Ts) == L - 1 and len(pool) == len(conv_w)
    cout = np.array([w.shape[0] for w in conv_w], dtype=np.int64)
    pl = np.array([1 if p else 0 for p in pool], dtype=np.int32)
    fc_out = np.array([w.shape[0] for w in fc_w], dtype=np.int64)
    Wp = (C.c_void_p * L)(*[w.ctypes.data for w in Ws])
    Tp = (C.c_void_p * max(L - 1, 1))(*[t.ctypes.data for t in Ts])
    Fs = []
    Fp = None
    if flip is not None:
        Fs = [_c(f, np.uint8) for f in flip]
        Fp = (C.c_void_p * max(L - 1, 1))(*[f.ctypes.data for f in Fs])
    out = np.empty((B, int(fc_out[-1])), dtype=np.int32)
    rc = lib().qo_convnet(_p(x), C.c_int64(B), C.c_int64(H), C.c_int64(Wd), C.c_int64(C0), C.c_int(len(conv_w)),
                          _p(cout), _p(pl), C.c_int(len(fc_w)), _p(fc_out), Wp, Tp, Fp, _p(out))
    _check(rc, "convnet")
    return out


def linear_quant(x: np.ndarray, step: float, qmin: int, qmax: int) -> np.ndarray:
    """fp32 values -> int32 codes q = Clip(round(x / step), qmin, qmax) (single precision, ties to even)."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, dtype=np.int32)
    rc = lib().qo_linear_quant(_p(x), C.c_int64(x.size), C.c_float(step), C.c_int32(qmin), C.c_int32(qmax), _p(out))
    _check(rc, "linear_quant")
    return out


def ap2(x: np.ndarray):
    """fp32 values -> (exponent round(log2 |x|) as int32, sign as int8 with 0 for x = 0 / NaN)."""
    x = _c(x, np.float32)
    e = np.empty(x.shape, dtype=np.int32)
    s = np.empty(x.shape, dtype=np.int8)
    _check(lib().qo_ap2(_p(x), C.c_int64(x.size), _p(e), _p(s)), "ap2")
    return e, s


def log_quant(x: np.ndarray, emin: int, emax: int) -> np.ndarray:
    """fp32 values -> int8 codes: 0, or sign * (e - emin + 1) with e = min(round(log2 |x|), emax) >= emin."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, dtype=np.int8)
    _check(lib().qo_log_quant(_p(x), C.c_int64(x.size), C.c_int32(emin), C.c_int32(emax), _p(out)), "log_quant")
    return out


def log_code_value(code: np.ndarray) -> np.ndarray:
    """int8 logarithmic codes -> int32 fixed-point values sign(c) * 2^(|c| - 1) (0 for code 0)."""
    code = _c(code, np.int8)
    out = np.empty(code.shape, dtype=np.int32)
    _check(lib().qo_log_code_value(_p(code), C.c_int64(code.size), _p(out)), "log_code_value")
    return out


def ste_mask(g: np.ndarray, a: np.ndarray) -> np.ndarray:
    """fp32 gradient g where |a| <= 1, else 0 (straight-through estimator of Alg. 1)."""
    g = _c(g, np.float32)
    a = _c(a, np.float32)
    assert g.shape == a.shape
    out = np.empty(g.shape, dtype=np.float32)
    _check(lib().qo_ste_mask(_p(g), _p(a), C.c_int64(g.size), _p(out)), "ste_mask")
    return out


def bn_affine(s: np.ndarray, scale: np.ndarray, shift: np.ndarray) -> np.ndarray:
    """int32 sums [M][N] -> fp32 fma(s, scale[n], shift[n])."""
    s = _c(s, np.int32)
    scale = _c(scale, np.float32)
    shift = _c(shift, np.float32)
    M, N = s.shape
    assert scale.shape == (N,) and shift.shape == (N,)
    out = np.empty((M, N), dtype=np.float32)
    _check(lib().qo_bn_affine(_p(s), C.c_int64(M), C.c_int64(N), _p(scale), _p(shift), _p(out)), "bn_affine")
    return out


def backward(g: np.ndarray, w: np.ndarray, a: np.ndarray):
    """g int32 [M][N], w int8 +-1 [N][K], a int8 +-1 [M][K] -> (g_a = g w  [M][K], g_W = g^T a  [N][K]), int32."""
    g = _c(g, np.int32)
    w = _c(w, np.int8)
    a = _c(a, np.int8)
    M, N = g.shape
    K = w.shape[1]
    assert w.shape == (N, K) and a.shape == (M, K)
    ga = np.empty((M, K), dtype=np.int32)
    gw = np.empty((N, K), dtype=np.int32)
    rc = lib().qo_backward(_p(g), _p(w), _p(a), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(ga), _p(gw))
    _check(rc, "backward")
    return ga, gw


def filter_unique(w: np.ndarray) -> np.ndarray:
    """w int8 +-1 [cout][kh][kw][cin] -> int32 [cin]: distinct 2-D filters per input channel, up to negation."""
    w = _c(w, np.int8)
    co, kh, kw, ci = w.shape
    out = np.empty((ci,), dtype=np.int32)
    _check(lib().qo_filter_unique(_p(w), C.c_int64(co), C.c_int64(kh), C.c_int64(kw), C.c_int64(ci), _p(out)), "filter_unique")
    return out


def conv2d_dedup(u: np.ndarray, w: np.ndarray, pad: int):
    """conv2d (stride 1) evaluated through the distinct 2-D filters of every input channel; returns (out, number of
    2-D filter applications)."""
    u = _c(u, np.int32)
    w = _c(w, np.int8)
    B, H, Wd, Ci = u.shape
    Co, KH, KW, Ci2 = w.shape
    assert Ci == Ci2
    out = np.empty((B, H + 2 * pad - KH + 1, Wd + 2 * pad - KW + 1, Co), dtype=np.int32)
    applied = np.zeros(1, dtype=np.int64)
    rc = lib().qo_conv2d_dedup(_p(u), C.c_int64(B), C.c_int64(H), C.c_int64(Wd), C.c_int64(Ci), _p(w), C.c_int64(Co),
                               C.c_int64(KH), C.c_int64(KW), C.c_int64(pad), _p(out), _p(applied))
    _check(rc, "conv2d_dedup")
    return out, int(applied[0])


def num_threads() -> int:
    return int(lib().qo_num_threads())
