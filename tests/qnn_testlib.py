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
