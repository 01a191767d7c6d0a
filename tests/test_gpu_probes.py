"""The measurement helpers do the work their figures are computed from: the vector-ALU probe counts disagreements of
register-resident words (the inner product of Sec. 6, Eq. (popc)), the matrix-core probe multiplies E2M1 operands."""
import numpy as np
import pytest
import torch

import paper_1609_07061_amd as q

pytestmark = pytest.mark.gpu


def test_valu_probe_counts_what_it_claims():
    blocks, iters = 3, 5
    sink = torch.zeros(blocks * 256, dtype=torch.int32, device="cuda")
    q.qnn_probe_valu_peak(sink, blocks, iters)
    got = sink.cpu().numpy().astype(np.int64)
    t = np.arange(256, dtype=np.uint64)[None, :]
    b = np.arange(blocks, dtype=np.uint64)[:, None]
    w = (t * np.uint64(2654435761) + b) & np.uint64(0xFFFFFFFF)
    want = np.zeros((blocks, 256), dtype=np.int64)
    for j in range(16):
        a = (w * np.uint64(2 * j + 3)) & np.uint64(0xFFFFFFFF)
        x = (a ^ w).astype(np.uint64)
        want += np.array([[bin(int(v)).count("1") for v in row] for row in x], dtype=np.int64)
    assert np.array_equal(got, (want * iters).reshape(-1))


@pytest.mark.parametrize("bits,per_product", [(0x22222222, 1.0), (0x44444444, 4.0), (0, 0.0)])
def test_mfma_probe_multiplies_e2m1_operands(bits, per_product):
    """All operand nibbles equal: every accumulator element gains 64 products per instruction, sixteen blocks of
    sixteen elements per lane are summed."""
    blocks, iters = 2, 3
    sink = torch.full((blocks * 256,), -1.0, dtype=torch.float32, device="cuda")
    q.qnn_probe_mfma_fp4_peak(sink, blocks, iters, bits, False)
    want = 16 * 16 * iters * 64 * per_product
    assert (sink.cpu().numpy() == want).all()


def test_probe_argument_errors():
    sink = torch.zeros(256, dtype=torch.int32, device="cuda")
    with pytest.raises(ValueError):
        q.qnn_probe_valu_peak(sink, 2, 1)
    with pytest.raises(q.QnnError):
        q.qnn_probe_valu_peak(sink, 0, 1)
