"""Python binding of libqnn (the C ABI in include/qnn.h): argument marshalling only.

Every function has the name of the C entry point it forwards to, takes torch tensors that live on the GPU (PyTorch is
used for device memory and streams, nothing else), passes their data pointers plus the current HIP stream, and raises
QnnError on a non-zero status.  Packed words are carried in torch.int32 tensors (same 32 bits as the uint32 of the ABI).
There is no CPU fallback: importing this package fails if the built library is missing.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

PLANE_BIT, PLANE_SIGN = 0, 1
ENGINE_AUTO, ENGINE_VALU, ENGINE_MFMA, ENGINE_MFMA_FP4, ENGINE_MFMA_LDS = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqnn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first with `python paper_1609_07061_amd/build.py` "
        "(or __graft_entry__.build()); this package has no fallback path"
    )
_lib = C.CDLL(LIB_PATH)

_i64, _int, _vp, _sz = C.c_int64, C.c_int, C.c_void_p, C.c_size_t
_SIGS = {
    "qnn_pack_sign": [_vp, _i64, _i64, _i64, _vp, _i64, _vp],
    "qnn_pack_bitplanes": [_vp, _i64, _i64, _i64, _int, _vp, _i64, _i64, _vp],
    "qnn_binary_gemm": [_vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _vp],
    "qnn_binary_gemm_ex": [_vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _int, _vp],
    "qnn_binary_gemm_sign": [_vp, _i64, _vp, _i64, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _int, _vp],
    "qnn_bitplane_gemm": [_vp, _int, _vp, _int, _i64, _i64, _vp, _int, _vp, _int, _i64, _i64, _vp, _i64, _i64, _i64,
                          _i64, _vp],
    "qnn_bitplane_gemm_ex": [_vp, _int, _vp, _int, _i64, _i64, _vp, _int, _vp, _int, _i64, _i64, _vp, _i64, _i64, _i64,
                             _i64, _int, _vp],
    "qnn_bitplane_gemm_sign": [_vp, _int, _vp, _int, _i64, _i64, _vp, _int, _vp, _int, _i64, _i64, _vp, _vp, _vp, _i64,
                               _i64, _i64, _i64, _int, _vp],
    "qnn_threshold_sign": [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _vp],
    "qnn_probe_shader_clock": [_vp, _vp],
    "qnn_stamp_clocks": [_vp, _vp],
    "qnn_probe_valu_peak": [_vp, C.c_int64, C.c_uint32, _vp],
    "qnn_probe_mfma_fp4_peak": [_vp, C.c_int64, C.c_uint32, C.c_uint32, C.c_int, _vp],
    "qnn_fold_batchnorm": [_vp, _vp, _vp, _vp, C.c_double, _i64, _vp, _vp],
    "qnn_binary_mlp_forward": [_vp, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp],
    "qnn_binary_mlp_forward_ex": [_vp, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _int, _vp],
    "qnn_binary_mlp_forward_static": [_vp, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp, _vp, _i64, _vp],
    "qnn_bitplane_conv2d": [_vp, _int, _vp, _int, _i64, _i64, _i64, _i64, _i64, _vp, _int, _vp, _int, _i64, _i64, _int,
                            _int, _int, _int, _vp, _vp],
    "qnn_bitplane_conv2d_sign": [_vp, _int, _vp, _int, _i64, _i64, _i64, _i64, _i64, _vp, _int, _vp, _int, _i64, _i64, _int,
                                 _int, _int, _int, _vp, _vp, _vp, _int, _vp],
    "qnn_binary_convnet_forward": [_vp, _i64, _i64, _i64, _i64, _int, _int, _vp, _vp, _int, _vp, _vp, _vp, _vp, _vp, _i64,
                                   _vp, _sz, _int, _vp],
    "qnn_linear_quant_planes": [_vp, _i64, _i64, _i64, C.c_float, C.c_int32, C.c_int32, _int, _vp, _i64, _i64, _vp],
    "qnn_log_quant_planes": [_vp, _vp, _i64, _i64, _i64, _i64, C.c_int32, C.c_int32, _int, _int, _vp, _i64, _i64, _vp],
    "qnn_batchnorm_affine": [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _vp],
    "qnn_transpose_bits": [_vp, _i64, _i64, _i64, _i64, _int, _vp, _i64, _i64, _vp],
    "qnn_binary_backward": [_vp, _int, _vp, _int, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64,
                            _vp, _sz, _vp],
    "qnn_conv2d_dedup": [_vp, _int, _vp, _i64, _i64, _i64, _i64, _i64, _vp, _i64, _int, _vp, _vp, _vp, _sz, _vp],
    "qnn_bitplane_conv2d_ex": [_vp, _int, _vp, _int, _i64, _i64, _i64, _i64, _i64, _vp, _int, _vp, _int, _i64, _i64, _int,
                               _int, _int, _int, _vp, _int, _vp],
}
for _name, _args in _SIGS.items():
    _f = getattr(_lib, _name)
    _f.argtypes = _args
    _f.restype = C.c_int
_lib.qnn_binary_mlp_workspace_bytes.argtypes = [_i64, _int, _int, _vp]
_lib.qnn_binary_mlp_workspace_bytes.restype = _sz
_lib.qnn_static_scratch_bytes.restype = _sz
_lib.qnn_binary_convnet_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, _int, _int, _vp, _vp, _int, _vp]
_lib.qnn_binary_convnet_workspace_bytes.restype = _sz
_lib.qnn_conv2d_dedup_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, _i64, _int]
_lib.qnn_conv2d_dedup_workspace_bytes.restype = _sz
_lib.qnn_binary_backward_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
_lib.qnn_binary_backward_workspace_bytes.restype = _sz
_lib.qnn_last_engine.restype = C.c_int
_lib.qnn_last_error.restype = C.c_char_p
_lib.qnn_version.restype = C.c_char_p

_lib.qnn_last_engines.argtypes = [_vp, _int]
_lib.qnn_last_engines.restype = C.c_int

EXPORTS = sorted(list(_SIGS) + ["qnn_binary_mlp_workspace_bytes", "qnn_static_scratch_bytes", "qnn_binary_convnet_workspace_bytes",
                               "qnn_binary_backward_workspace_bytes", "qnn_conv2d_dedup_workspace_bytes", "qnn_last_engine",
                               "qnn_last_engines", "qnn_last_error", "qnn_version"])


class QnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"qnn status {status}: {message}")
        self.status = status


def _check(status: int):
    if status != 0:
        raise QnnError(status, _lib.qnn_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: Optional[torch.Tensor], dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _rows_ld(t: torch.Tensor, name: str):
    """(rows, cols, leading dimension) of a 2-D tensor whose rows are contiguous."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with contiguous rows")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)
    return t.shape[0], t.shape[1], ld


def _planes_ld(t: torch.Tensor, name: str):
    """(planes, rows, words, ld, plane stride) of a [P][rows][words] tensor."""
    if t.dim() != 3 or (t.shape[2] > 1 and t.stride(2) != 1):
        raise ValueError(f"{name} must be [planes][rows][words] with contiguous rows")
    ld = t.stride(1) if t.shape[1] > 1 else max(t.shape[2], 1)
    ps = t.stride(0) if t.shape[0] > 1 else 0
    return t.shape[0], t.shape[1], t.shape[2], ld, ps


def _coef(c: Sequence[int]):
    return (C.c_int32 * len(c))(*[int(v) for v in c])


def words_for(K: int) -> int:
    return (K + 31) // 32


def qnn_last_engine() -> int:
    return int(_lib.qnn_last_engine())


def qnn_last_engines() -> list:
    buf = (C.c_int * 32)()
    n = int(_lib.qnn_last_engines(buf, 32))
    return [int(buf[i]) for i in range(min(n, 32))]


def qnn_probe_shader_clock() -> float:
    """Shader clock in MHz right now (synchronizes: measurement helper only)."""
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    _check(_lib.qnn_probe_shader_clock(out.data_ptr(), _stream()))
    c, r, _ = out.cpu().tolist()
    return 100.0 * c / r if r else float("nan")


def qnn_stamp_clocks(out: torch.Tensor) -> None:
    """Enqueues a stamp {shader-clock counter, 100 MHz counter, die id} into out (int64[3] on the GPU)."""
    _check(_lib.qnn_stamp_clocks(_dev(out, torch.int64, "out"), _stream()))


def qnn_probe_valu_peak(sink: torch.Tensor, blocks: int, iterations: int) -> None:
    """Enqueues the register-resident xor + popcount kernel: blocks * 256 * iterations * 16 * 32 MACs."""
    if sink.numel() < blocks * 256:
        raise ValueError("sink needs blocks * 256 elements")
    _check(_lib.qnn_probe_valu_peak(_dev(sink, torch.int32, "sink"), int(blocks), int(iterations), _stream()))


def qnn_probe_mfma_fp4_peak(sink: torch.Tensor, blocks: int, iterations: int, operand_bits: int, vary: bool) -> None:
    """Enqueues the register-resident FP4 matrix-core kernel: blocks * 4 * iterations * 16 * 65536 MACs."""
    if sink.numel() < blocks * 256:
        raise ValueError("sink needs blocks * 256 elements")
    _check(_lib.qnn_probe_mfma_fp4_peak(_dev(sink, torch.float32, "sink"), int(blocks), int(iterations),
                                        int(operand_bits) & 0xFFFFFFFF, 1 if vary else 0, _stream()))


def average_shader_clock_mhz(stamp0: torch.Tensor, stamp1: torch.Tensor) -> Optional[float]:
    """Average shader clock between two stamps (None if they were taken on different dies or are degenerate)."""
    a, b = stamp0.cpu().tolist(), stamp1.cpu().tolist()
    if a[2] != b[2] or b[1] <= a[1] or b[0] <= a[0]:
        return None
    return 100.0 * (b[0] - a[0]) / (b[1] - a[1])


def qnn_version() -> str:
    return _lib.qnn_version().decode()


def qnn_pack_sign(x: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, K, ldx = _rows_ld(x, "x")
    if out is None:
        out = torch.empty((rows, words_for(K)), dtype=torch.int32, device=x.device)
    _, _, ldo = _rows_ld(out, "out")
    _check(_lib.qnn_pack_sign(_dev(x, torch.float32, "x"), rows, K, ldx, _dev(out, torch.int32, "out"), ldo, _stream()))
    return out


def qnn_pack_bitplanes(v: torch.Tensor, nbits: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, K, ldv = _rows_ld(v, "v")
    if out is None:
        out = torch.empty((nbits, rows, words_for(K)), dtype=torch.int32, device=v.device)
    P, _, _, ld, ps = _planes_ld(out, "out")
    if P != nbits:
        raise ValueError("out must have nbits planes")
    _check(_lib.qnn_pack_bitplanes(_dev(v, torch.uint8, "v"), rows, K, ldv, nbits, _dev(out, torch.int32, "out"), ld,
                                   ps, _stream()))
    return out


def qnn_linear_quant_planes(x: torch.Tensor, step: float, qmin: int, qmax: int, nbits: int,
                            out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, K, ldx = _rows_ld(x, "x")
    if out is None:
        out = torch.empty((nbits, rows, words_for(K)), dtype=torch.int32, device=x.device)
    P, _, _, ld, ps = _planes_ld(out, "out")
    if P != nbits:
        raise ValueError("out must have nbits planes")
    _check(_lib.qnn_linear_quant_planes(_dev(x, torch.float32, "x"), rows, K, ldx, step, qmin, qmax, nbits,
                                        _dev(out, torch.int32, "out"), ld, ps, _stream()))
    return out


def qnn_log_quant_planes(x: torch.Tensor, emin: int, emax: int, nbits: int, as_value: bool = False,
                         gate: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, K, ldx = _rows_ld(x, "x")
    ldg = 0
    if gate is not None:
        gr, gk, ldg = _rows_ld(gate, "gate")
        if (gr, gk) != (rows, K):
            raise ValueError("gate must have the shape of x")
    if out is None:
        out = torch.empty((nbits, rows, words_for(K)), dtype=torch.int32, device=x.device)
    P, _, _, ld, ps = _planes_ld(out, "out")
    if P != nbits:
        raise ValueError("out must have nbits planes")
    _check(_lib.qnn_log_quant_planes(_dev(x, torch.float32, "x"), _dev(gate, torch.float32, "gate"), rows, K, ldx, ldg,
                                     emin, emax, 1 if as_value else 0, nbits, _dev(out, torch.int32, "out"), ld, ps,
                                     _stream()))
    return out


def qnn_batchnorm_affine(sums: torch.Tensor, scale: torch.Tensor, shift: torch.Tensor,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, N, lds = _rows_ld(sums, "sums")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=sums.device)
    _, _, ldy = _rows_ld(out, "out")
    _check(_lib.qnn_batchnorm_affine(_dev(sums, torch.int32, "sums"), lds, M, N, _dev(scale, torch.float32, "scale"),
                                     _dev(shift, torch.float32, "shift"), _dev(out, torch.float32, "out"), ldy, _stream()))
    return out


def qnn_transpose_bits(planes: torch.Tensor, cols: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """planes: [P][rows][words] holding `cols` bits per row -> [P][cols][ceil(rows/32)]."""
    P, rows, _, ld, ps = _planes_ld(planes, "planes")
    if out is None:
        out = torch.empty((P, cols, words_for(rows)), dtype=torch.int32, device=planes.device)
    Po, _, _, ldo, pso = _planes_ld(out, "out")
    if Po != P:
        raise ValueError("out must have as many planes as the input")
    _check(_lib.qnn_transpose_bits(_dev(planes, torch.int32, "planes"), rows, cols, ld, ps, P,
                                   _dev(out, torch.int32, "out"), ldo, pso, _stream()))
    return out


def qnn_conv2d_dedup(A: torch.Tensor, coefA: Sequence[int], Cin: int, W: torch.Tensor, pad: int,
                     workspace: Optional[torch.Tensor] = None):
    """A: [Pa][B][H][W][words] bit-mode planes; W: [Cout][3][3][words] packed +-1 -> (out int32 [B][Ho][Wo][Cout],
    distinct 2-D filters per input channel int32 [Cin])."""
    if A.dim() != 5 or not A.is_contiguous() or W.dim() != 4 or not W.is_contiguous() or W.shape[1:3] != (3, 3):
        raise ValueError("A must be contiguous [Pa][B][H][W][words], W contiguous [Cout][3][3][words]")
    Pa, B, H, Wd, _ = A.shape
    Cout = W.shape[0]
    need = int(_lib.qnn_conv2d_dedup_workspace_bytes(B, H, Wd, Cin, Cout, pad))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=A.device)
    out = torch.empty((B, H + 2 * pad - 2, Wd + 2 * pad - 2, Cout), dtype=torch.int32, device=A.device)
    counts = torch.empty((Cin,), dtype=torch.int32, device=A.device)
    _check(_lib.qnn_conv2d_dedup(_dev(A, torch.int32, "A"), Pa, _coef(coefA), A.stride(0) if Pa > 1 else 0, B, H, Wd, Cin,
                                 _dev(W, torch.int32, "W"), Cout, pad, _dev(out, torch.int32, "out"),
                                 _dev(counts, torch.int32, "counts"), workspace.data_ptr(), workspace.numel(), _stream()))
    return out, counts


def qnn_binary_backward_workspace_bytes(M: int, N: int, K: int, Pg: int) -> int:
    return int(_lib.qnn_binary_backward_workspace_bytes(M, N, K, Pg))


def qnn_binary_backward(G: torch.Tensor, coefG: Sequence[int], modeG: int, N: int, W: torch.Tensor, A: torch.Tensor,
                        K: int, workspace: Optional[torch.Tensor] = None):
    """G: [Pg][M][words of N]; W: [N][words of K]; A: [M][words of K] -> (gA int32 [M][K], gW int32 [N][K])."""
    Pg, M, _, ldg, psg = _planes_ld(G, "G")
    _, _, ldw = _rows_ld(W, "W")
    _, _, lda = _rows_ld(A, "A")
    need = qnn_binary_backward_workspace_bytes(M, N, K, Pg)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=G.device)
    gA = torch.empty((M, K), dtype=torch.int32, device=G.device)
    gW = torch.empty((N, K), dtype=torch.int32, device=G.device)
    _check(_lib.qnn_binary_backward(_dev(G, torch.int32, "G"), Pg, _coef(coefG), modeG, ldg, psg,
                                    _dev(W, torch.int32, "W"), ldw, _dev(A, torch.int32, "A"), lda,
                                    _dev(gA, torch.int32, "gA"), K, _dev(gW, torch.int32, "gW"), K, M, N, K,
                                    workspace.data_ptr(), workspace.numel(), _stream()))
    return gA, gW


def qnn_binary_gemm(A: torch.Tensor, W: torch.Tensor, K: int, out: Optional[torch.Tensor] = None,
                    engine: Optional[int] = None) -> torch.Tensor:
    M, _, lda = _rows_ld(A, "A")
    N, _, ldw = _rows_ld(W, "W")
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _, _, ldc = _rows_ld(out, "out")
    a, w, c = _dev(A, torch.int32, "A"), _dev(W, torch.int32, "W"), _dev(out, torch.int32, "out")
    if engine is None:
        _check(_lib.qnn_binary_gemm(a, lda, w, ldw, c, ldc, M, N, K, _stream()))
    else:
        _check(_lib.qnn_binary_gemm_ex(a, lda, w, ldw, c, ldc, M, N, K, engine, _stream()))
    return out


def qnn_binary_gemm_sign(A: torch.Tensor, W: torch.Tensor, K: int, T: torch.Tensor,
                         flip: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                         engine: int = ENGINE_AUTO) -> torch.Tensor:
    M, _, lda = _rows_ld(A, "A")
    N, _, ldw = _rows_ld(W, "W")
    if out is None:
        out = torch.empty((M, words_for(N)), dtype=torch.int32, device=A.device)
    _, _, ldo = _rows_ld(out, "out")
    _check(_lib.qnn_binary_gemm_sign(_dev(A, torch.int32, "A"), lda, _dev(W, torch.int32, "W"), ldw,
                                     _dev(T, torch.int32, "T"), _dev(flip, torch.uint8, "flip"),
                                     _dev(out, torch.int32, "out"), ldo, M, N, K, engine, _stream()))
    return out


def qnn_bitplane_gemm(A: torch.Tensor, coefA: Sequence[int], modeA: int, W: torch.Tensor, coefW: Sequence[int],
                      modeW: int, K: int, out: Optional[torch.Tensor] = None,
                      engine: Optional[int] = None) -> torch.Tensor:
    """engine None -> qnn_bitplane_gemm; an engine -> qnn_bitplane_gemm_ex."""
    Pa, M, _, lda, sa = _planes_ld(A, "A")
    Pb, N, _, ldw, sw = _planes_ld(W, "W")
    if len(coefA) != Pa or len(coefW) != Pb:
        raise ValueError("one coefficient per plane")
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _, _, ldc = _rows_ld(out, "out")
    args = (_dev(A, torch.int32, "A"), Pa, _coef(coefA), modeA, lda, sa, _dev(W, torch.int32, "W"), Pb, _coef(coefW),
            modeW, ldw, sw, _dev(out, torch.int32, "out"), ldc, M, N, K)
    if engine is None:
        _check(_lib.qnn_bitplane_gemm(*args, _stream()))
    else:
        _check(_lib.qnn_bitplane_gemm_ex(*args, engine, _stream()))
    return out


def qnn_bitplane_gemm_sign(A: torch.Tensor, coefA: Sequence[int], modeA: int, W: torch.Tensor, coefW: Sequence[int],
                           modeW: int, K: int, T: torch.Tensor, flip: Optional[torch.Tensor] = None,
                           out: Optional[torch.Tensor] = None, engine: int = ENGINE_AUTO) -> torch.Tensor:
    Pa, M, _, lda, sa = _planes_ld(A, "A")
    Pb, N, _, ldw, sw = _planes_ld(W, "W")
    if len(coefA) != Pa or len(coefW) != Pb:
        raise ValueError("one coefficient per plane")
    if out is None:
        out = torch.empty((M, words_for(N)), dtype=torch.int32, device=A.device)
    _, _, ldo = _rows_ld(out, "out")
    _check(_lib.qnn_bitplane_gemm_sign(_dev(A, torch.int32, "A"), Pa, _coef(coefA), modeA, lda, sa,
                                       _dev(W, torch.int32, "W"), Pb, _coef(coefW), modeW, ldw, sw,
                                       _dev(T, torch.int32, "T"), _dev(flip, torch.uint8, "flip"),
                                       _dev(out, torch.int32, "out"), ldo, M, N, K, engine, _stream()))
    return out


def qnn_threshold_sign(Cm: torch.Tensor, T: torch.Tensor, flip: Optional[torch.Tensor] = None,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, N, ldc = _rows_ld(Cm, "C")
    if out is None:
        out = torch.empty((M, words_for(N)), dtype=torch.int32, device=Cm.device)
    _, _, ldo = _rows_ld(out, "out")
    _check(_lib.qnn_threshold_sign(_dev(Cm, torch.int32, "C"), ldc, M, N, _dev(T, torch.int32, "T"),
                                   _dev(flip, torch.uint8, "flip"), _dev(out, torch.int32, "out"), ldo, _stream()))
    return out


def qnn_fold_batchnorm(gamma, beta, mean, var, eps: float):
    """Host-only helper (numpy float64 arrays in, (int32 T, uint8 flip) numpy arrays out)."""
    import numpy as np

    g, b, m, v = (np.ascontiguousarray(a, dtype=np.float64) for a in (gamma, beta, mean, var))
    n = g.size
    T = np.empty(n, dtype=np.int32)
    flip = np.empty(n, dtype=np.uint8)
    _check(_lib.qnn_fold_batchnorm(g.ctypes.data, b.ctypes.data, m.ctypes.data, v.ctypes.data, float(eps), n,
                                   T.ctypes.data, flip.ctypes.data))
    return T, flip


def qnn_binary_mlp_workspace_bytes(batch: int, in_bits: int, dims: Sequence[int]) -> int:
    d = (C.c_int64 * len(dims))(*[int(v) for v in dims])
    return int(_lib.qnn_binary_mlp_workspace_bytes(batch, in_bits, len(dims) - 1, d))


def qnn_static_scratch_bytes() -> int:
    return int(_lib.qnn_static_scratch_bytes())


def qnn_binary_mlp_forward(x: torch.Tensor, in_bits: int, dims: Sequence[int], W: Sequence[torch.Tensor],
                           T: Sequence[torch.Tensor], flip: Optional[Sequence[Optional[torch.Tensor]]] = None,
                           logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           engine: Optional[int] = None, static_scratch: bool = False) -> torch.Tensor:
    """engine None and dense x -> qnn_binary_mlp_forward; an engine or a strided x -> qnn_binary_mlp_forward_ex;
    static_scratch -> qnn_binary_mlp_forward_static (no workspace: the library's built-in scratch array)."""
    batch, _, ldx = _rows_ld(x, "x")
    L = len(dims) - 1
    if len(W) != L or len(T) != L - 1:
        raise ValueError("need one W per layer and one T per hidden layer")
    for l, w in enumerate(W):
        if w.dim() != 2 or not w.is_contiguous() or tuple(w.shape) != (dims[l + 1], words_for(dims[l])):
            raise ValueError(f"W[{l}] must be dense [{dims[l + 1]}][{words_for(dims[l])}]")
    if logits is None:
        logits = torch.empty((batch, dims[-1]), dtype=torch.int32, device=x.device)
    _, _, ldl = _rows_ld(logits, "logits")
    d = (C.c_int64 * (L + 1))(*[int(v) for v in dims])
    Wp = (C.c_void_p * L)(*[_dev(w, torch.int32, "W") for w in W])
    Tp = (C.c_void_p * max(L - 1, 1))(*[_dev(t, torch.int32, "T") for t in T])
    Fp = None
    if flip is not None:
        Fp = (C.c_void_p * max(L - 1, 1))(*[_dev(f, torch.uint8, "flip") for f in flip])
    head = (_dev(x, torch.uint8, "x"), batch, ldx, in_bits, L, d, Wp, Tp, Fp, _dev(logits, torch.int32, "logits"), ldl)
    if static_scratch:
        if engine is not None or ldx != dims[0]:
            raise ValueError("the static-scratch entry point takes dense rows and no engine")
        _check(_lib.qnn_binary_mlp_forward_static(*head, _stream()))
        return logits
    if workspace is None:
        workspace = torch.empty(qnn_binary_mlp_workspace_bytes(batch, in_bits, dims), dtype=torch.uint8, device=x.device)
    ws = (_dev(workspace, torch.uint8, "workspace"), workspace.numel())
    if engine is None and ldx == dims[0]:
        _check(_lib.qnn_binary_mlp_forward(*head, *ws, _stream()))
    else:
        _check(_lib.qnn_binary_mlp_forward_ex(*head, *ws, ENGINE_AUTO if engine is None else engine, _stream()))
    return logits


def qnn_bitplane_conv2d(A: torch.Tensor, coefA: Sequence[int], modeA: int, Cin: int, W: torch.Tensor,
                        coefW: Sequence[int], modeW: int, pad: int, stride: int = 1,
                        out: Optional[torch.Tensor] = None, engine: Optional[int] = None) -> torch.Tensor:
    """A: [Pa][B][H][W][Cw] packed planes (dense); W: [Pb][Cout][KH][KW][Cw] packed planes (dense)."""
    if A.dim() != 5 or W.dim() != 5 or not A.is_contiguous() or not W.is_contiguous():
        raise ValueError("A must be dense [Pa][B][H][W][Cw] and W dense [Pb][Cout][KH][KW][Cw]")
    Pa, B, H, Wd, Cw = A.shape
    Pb, Cout, KH, KW, Cw2 = W.shape
    if Cw != words_for(Cin) or Cw2 != Cw:
        raise ValueError("channel words do not match Cin")
    Ho = (H + 2 * pad - KH) // stride + 1
    Wo = (Wd + 2 * pad - KW) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.int32, device=A.device)
    if not out.is_contiguous() or tuple(out.shape) != (B, Ho, Wo, Cout):
        raise ValueError("out must be dense [B][Ho][Wo][Cout]")
    args = (_dev(A, torch.int32, "A"), Pa, _coef(coefA), modeA, A.stride(0) if Pa > 1 else 0, B, H, Wd, Cin,
            _dev(W, torch.int32, "W"), Pb, _coef(coefW), modeW, W.stride(0) if Pb > 1 else 0, Cout, KH, KW, pad, stride,
            _dev(out, torch.int32, "out"))
    if engine is None:
        _check(_lib.qnn_bitplane_conv2d(*args, _stream()))
    else:
        _check(_lib.qnn_bitplane_conv2d_ex(*args, engine, _stream()))
    return out


def qnn_bitplane_conv2d_sign(A: torch.Tensor, coefA: Sequence[int], modeA: int, Cin: int, W: torch.Tensor,
                             coefW: Sequence[int], modeW: int, pad: int, stride: int, T: torch.Tensor,
                             flip: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                             engine: int = ENGINE_AUTO) -> torch.Tensor:
    """A: [Pa][B][H][W][Cw], W: [Pb][Cout][KH][KW][Cw] (dense) -> packed bits [B][Ho][Wo][ceil(Cout/32)]."""
    if A.dim() != 5 or W.dim() != 5 or not A.is_contiguous() or not W.is_contiguous():
        raise ValueError("A must be dense [Pa][B][H][W][Cw] and W dense [Pb][Cout][KH][KW][Cw]")
    Pa, B, H, Wd, Cw = A.shape
    Pb, Cout, KH, KW, Cw2 = W.shape
    if Cw != words_for(Cin) or Cw2 != Cw:
        raise ValueError("channel words do not match Cin")
    Ho = (H + 2 * pad - KH) // stride + 1
    Wo = (Wd + 2 * pad - KW) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, words_for(Cout)), dtype=torch.int32, device=A.device)
    if not out.is_contiguous() or tuple(out.shape) != (B, Ho, Wo, words_for(Cout)):
        raise ValueError("out must be dense [B][Ho][Wo][ceil(Cout/32)]")
    _check(_lib.qnn_bitplane_conv2d_sign(_dev(A, torch.int32, "A"), Pa, _coef(coefA), modeA, A.stride(0) if Pa > 1 else 0,
                                         B, H, Wd, Cin, _dev(W, torch.int32, "W"), Pb, _coef(coefW), modeW,
                                         W.stride(0) if Pb > 1 else 0, Cout, KH, KW, pad, stride,
                                         _dev(T, torch.int32, "T"), _dev(flip, torch.uint8, "flip"),
                                         _dev(out, torch.int32, "out"), engine, _stream()))
    return out


def _net_arrays(cout, pool, fc_out):
    co = (C.c_int64 * len(cout))(*[int(v) for v in cout])
    pl = (C.c_int32 * len(pool))(*[1 if v else 0 for v in pool])
    fo = (C.c_int64 * len(fc_out))(*[int(v) for v in fc_out])
    return co, pl, fo


def qnn_binary_convnet_workspace_bytes(B: int, H: int, Wd: int, C0: int, in_bits: int, cout: Sequence[int],
                                       pool: Sequence[int], fc_out: Sequence[int]) -> int:
    co, pl, fo = _net_arrays(cout, pool, fc_out)
    return int(_lib.qnn_binary_convnet_workspace_bytes(B, H, Wd, C0, in_bits, len(cout), co, pl, len(fc_out), fo))


def qnn_binary_convnet_forward(x: torch.Tensor, in_bits: int, cout: Sequence[int], pool: Sequence[int],
                               fc_out: Sequence[int], W: Sequence[torch.Tensor], T: Sequence[torch.Tensor],
                               flip: Optional[Sequence[Optional[torch.Tensor]]] = None,
                               logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                               engine: int = ENGINE_AUTO) -> torch.Tensor:
    """x: uint8 [B][H][W][C0] (dense); W: packed +-1 weights, convolutions [cout][3][3][Cw], fully connected [out][Kw]."""
    if x.dim() != 4 or not x.is_contiguous():
        raise ValueError("x must be dense [B][H][W][C0]")
    B, H, Wd, C0 = x.shape
    L = len(cout) + len(fc_out)
    if len(W) != L or len(T) != L - 1:
        raise ValueError("need one W per layer and one T per layer but the last")
    for w in W:
        if not w.is_contiguous():
            raise ValueError("weights must be dense")
    if logits is None:
        logits = torch.empty((B, fc_out[-1]), dtype=torch.int32, device=x.device)
    _, _, ldl = _rows_ld(logits, "logits")
    if workspace is None:
        need = qnn_binary_convnet_workspace_bytes(B, H, Wd, C0, in_bits, cout, pool, fc_out)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    co, pl, fo = _net_arrays(cout, pool, fc_out)
    Wp = (C.c_void_p * L)(*[_dev(w, torch.int32, "W") for w in W])
    Tp = (C.c_void_p * max(L - 1, 1))(*[_dev(t, torch.int32, "T") for t in T])
    Fp = None
    if flip is not None:
        Fp = (C.c_void_p * max(L - 1, 1))(*[_dev(f, torch.uint8, "flip") for f in flip])
    _check(_lib.qnn_binary_convnet_forward(_dev(x, torch.uint8, "x"), B, H, Wd, C0, in_bits, len(cout), co, pl, len(fc_out),
                                           fo, Wp, Tp, Fp, _dev(logits, torch.int32, "logits"), ldl,
                                           _dev(workspace, torch.uint8, "workspace"), workspace.numel(), engine, _stream()))
    return logits
