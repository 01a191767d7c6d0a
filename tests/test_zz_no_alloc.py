"""qnn_binary_mlp_forward_static, the entry point for callers that cannot allocate device memory: it must give, bit for
bit, what qnn_binary_mlp_forward gives with a caller workspace (and what the oracle gives), on two calls in a row that
share the library's built-in scratch array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi
from qnn_testlib import dev, host, np_pack_pm1

pytestmark = pytest.mark.gpu


def _case(seed, batch, dims, stream0):
    L = len(dims) - 1
    x = qi.uniform_int(seed, stream0, (batch, dims[0]), 0, 255, dtype=np.uint8)
    W = [qi.pm1(seed, stream0 + 1 + l, (dims[l + 1], dims[l])) for l in range(L)]
    T = [qi.uniform_int(seed, stream0 + 8 + l, (dims[l + 1],), -3000 if l == 0 else -40, 3000 if l == 0 else 40)
         for l in range(L - 1)]
    flip = [qi.bernoulli_bits(seed, stream0 + 16 + l, (dims[l + 1],)) for l in range(L - 1)]
    return x, W, T, flip


def test_static_scratch_forward_matches_workspace_forward_twice(seed):
    import paper_1609_07061_amd as q

    assert torch.cuda.is_available()
    # first call: large enough for the matrix-core kernels (several tiles, ragged batch); second: a smaller network and
    # batch that leaves most of the array holding the first call's data
    cases = [(_case(seed, 2100, [784, 1024, 512, 10], 1200), [784, 1024, 512, 10]),
             (_case(seed, 300, [100, 96, 10], 1230), [100, 96, 10])]
    for (x, W, T, flip), dims in cases:
        assert q.qnn_binary_mlp_workspace_bytes(x.shape[0], 8, dims) <= q.qnn_static_scratch_bytes()
        Wd, Td, Fd = [dev(np_pack_pm1(w)) for w in W], [dev(t) for t in T], [dev(f) for f in flip]
        xd = dev(x)
        want = host(q.qnn_binary_mlp_forward(xd, 8, dims, Wd, Td, Fd))
        engines = q.qnn_last_engines()
        got = torch.full(want.shape, -99, dtype=torch.int32, device="cuda")
        q.qnn_binary_mlp_forward(xd, 8, dims, Wd, Td, Fd, logits=got, static_scratch=True)
        assert q.qnn_last_engines() == engines
        assert np.array_equal(host(got), want)
        assert np.array_equal(want, oracle.mlp(x, W, T, flip))


def test_static_scratch_forward_refuses_what_does_not_fit(seed):
    import paper_1609_07061_amd as q

    dims = [784, 4096, 4096, 10]
    batch = 40000
    assert q.qnn_binary_mlp_workspace_bytes(batch, 8, dims) > q.qnn_static_scratch_bytes()
    x = torch.zeros((batch, 784), dtype=torch.uint8, device="cuda")
    W = [torch.zeros((dims[l + 1], (dims[l] + 31) // 32), dtype=torch.int32, device="cuda") for l in range(3)]
    T = [torch.zeros((dims[l + 1],), dtype=torch.int32, device="cuda") for l in range(2)]
    with pytest.raises(q.QnnError) as e:
        q.qnn_binary_mlp_forward(x, 8, dims, W, T, static_scratch=True)
    assert e.value.status == 6
