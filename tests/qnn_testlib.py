"""Helpers shared by the GPU parity tests: host-side packing of test inputs with numpy (a third packer, independent of
both the oracle's and the library's) and transfers to / from the device.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch


def np_pack_bits(bits01: np.ndarray, ld_words: int | None = None) -> np.ndarray:
    """[..., K] array of 0/1 -> [..., ld_words] uint32, element 32j+t at bit t of word j, tail zero."""
    K = bits01.shape[-1]
    Kw = (K + 31) // 32
    ld = Kw if ld_words is None else ld_words
    padded = np.zeros(bits01.shape[:-1] + (ld * 32,), dtype=np.uint8)
    padded[..., :K] = bits01 != 0
    return np.ascontiguousarray(np.packbits(padded, axis=-1, bitorder="little")).view("<u4")


def np_pack_pm1(s: np.ndarray, ld_words: int | None = None) -> np.ndarray:
    return np_pack_bits((s > 0).astype(np.uint8), ld_words)


def np_unpack_bits(words: np.ndarray, K: int) -> np.ndarray:
    """[..., Kw] uint32 -> [..., K] uint8 of 0/1."""
    b = np.unpackbits(np.ascontiguousarray(words).view(np.uint8), axis=-1, bitorder="little")
    return b[..., :K]


def dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def host_u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy()


# --------------------------------------------------------------------------------------------------------------------
# What the matrix-core engines take BY DESIGN (engine 2 = int8, 3 = FP4, 4 = int8 with planes merged once per workgroup
# in LDS); everything else they refuse with status 5 and AUTO sends to another engine.  The tests assert both directions:
# a supported case must run, an unsupported one must be refused - a regression in what an engine accepts cannot hide
# behind a skip.
INT8_PLANE_PAIRS = {(1, 1), (8, 1), (4, 4), (2, 1), (4, 1), (2, 2)}
INT8_PLANE_PAIRS_SIGN_OUT = {(1, 1), (8, 1)}
INT8_PLANE_PAIRS_CONV = {(1, 1), (2, 1)}
INT8_PLANE_PAIRS_CONV_SIGN_OUT = {(1, 1), (2, 1)}
LDS_PLANE_PAIRS = {(8, 1), (4, 4), (4, 1), (2, 2)}
LDS_PLANE_PAIRS_SIGN_OUT = {(8, 1)}
LDS_PLANE_PAIRS_CONV = {(2, 1)}  # both epilogues


def _code_positions(coefs):
    """Bit positions of the planes in the int8 code (coefficients = common factor x distinct powers of two up to 128:
    unsigned, two's complement, single plane), or None."""
    from math import gcd

    g = 0
    for c in coefs:
        if c == 0:
            return None
        g = gcd(g, abs(int(c)))
    mags = [abs(int(c)) // g for c in coefs]
    if not all(m <= 128 and (m & (m - 1)) == 0 for m in mags) or len(set(mags)) != len(mags):
        return None
    return sorted(m.bit_length() - 1 for m in mags)


def engine_takes(engine: int, Pa: int = 1, Pb: int = 1, coefA=(1,), coefW=(1,), conv: bool = False,
                 sign_out: bool = False, row_words: int | None = None) -> bool:
    """row_words: packed words per row (per pixel for a convolution) of the dense test operands; engine 4 needs whole
    groups of four."""
    if engine in (0, 1):
        return True
    if engine == 3:
        return Pa == 1 and Pb == 1
    pa, pw = _code_positions(coefA), _code_positions(coefW)
    if pa is None or pw is None:
        return False
    if engine == 4:
        pairs = LDS_PLANE_PAIRS_CONV if conv else (LDS_PLANE_PAIRS_SIGN_OUT if sign_out else LDS_PLANE_PAIRS)
        dense = pa == list(range(Pa)) and pw == list(range(Pb))
        return (Pa, Pb) in pairs and dense and row_words is not None and row_words % 4 == 0
    if conv:
        pairs = INT8_PLANE_PAIRS_CONV_SIGN_OUT if sign_out else INT8_PLANE_PAIRS_CONV
    else:
        pairs = INT8_PLANE_PAIRS_SIGN_OUT if sign_out else INT8_PLANE_PAIRS
    return (Pa, Pb) in pairs


def run_on_engine(fn, *a, engine: int, takes: bool = True, **kw):
    """fn(..., engine=engine): the result if the engine is documented to take the case (any refusal fails the test),
    otherwise None after checking that the refusal is exactly status 5."""
    import pytest

    if takes:
        return fn(*a, engine=engine, **kw)
    with pytest.raises(Exception) as e:
        fn(*a, engine=engine, **kw)
    assert getattr(e.value, "status", None) == 5, e.value
    return None
