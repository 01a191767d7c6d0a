"""Randomised shape sweep of the multiply calls against the oracle: many small and medium shapes with ragged M, N, K,
random leading dimensions, every engine.  Seeded, so a failure names a reproducible case."""
import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi
from qnn_testlib import dev, engine_takes, host, host_u32, np_pack_bits, np_pack_pm1, run_on_engine

pytestmark = pytest.mark.gpu


def _rand_ints(seed, stream, n, lo, hi):
    return qi.uniform_int(seed, stream, (n,), lo, hi).tolist()


@pytest.mark.parametrize("engine", [0, 1, 2, 3])
def test_random_binary_gemm_shapes(seed, engine):
    import paper_1609_07061_amd as q

    Ms = _rand_ints(seed, 900, 14, 1, 700)
    Ns = _rand_ints(seed, 901, 14, 1, 700)
    Ks = _rand_ints(seed, 902, 14, 1, 3000)
    pads = _rand_ints(seed, 903, 42, 0, 5)
    for i, (M, N, K) in enumerate(zip(Ms, Ns, Ks)):
        a = qi.pm1(seed, 910 + i, (M, K))
        w = qi.pm1(seed, 930 + i, (N, K))
        Kw = (K + 31) // 32
        A = dev(np_pack_pm1(a, Kw + pads[3 * i]))[:, :Kw]
        W = dev(np_pack_pm1(w, Kw + pads[3 * i + 1]))[:, :Kw]
        out = torch.full((M, N + pads[3 * i + 2]), 12345, dtype=torch.int32, device="cuda")
        q.qnn_binary_gemm(A, W, K, out=out[:, :N], engine=engine)  # single planes: every engine takes every shape
        if engine:
            assert q.qnn_last_engine() == engine
        got = host(out)
        assert np.array_equal(got[:, :N], oracle.gemm_pm1(a, w)), (M, N, K, engine)
        assert (got[:, N:] == 12345).all(), (M, N, K, engine)


@pytest.mark.parametrize("engine", [0, 1, 2, 3])
def test_random_binary_gemm_sign_shapes(seed, engine):
    import paper_1609_07061_amd as q

    Ms = _rand_ints(seed, 950, 10, 1, 600)
    Ns = _rand_ints(seed, 951, 10, 1, 600)
    Ks = _rand_ints(seed, 952, 10, 1, 2500)
    for i, (M, N, K) in enumerate(zip(Ms, Ns, Ks)):
        a = qi.pm1(seed, 960 + i, (M, K))
        w = qi.pm1(seed, 975 + i, (N, K))
        T = qi.uniform_int(seed, 990 + i, (N,), -12, 12)
        flip = qi.bernoulli_bits(seed, 1005 + i, (N,)) if i % 2 else None
        want = oracle.pack_bits(oracle.threshold(oracle.gemm_pm1(a, w), T, flip))
        got = q.qnn_binary_gemm_sign(dev(np_pack_pm1(a)), dev(np_pack_pm1(w)), K, dev(T),
                                     dev(flip) if flip is not None else None, engine=engine)
        if engine:
            assert q.qnn_last_engine() == engine
        assert np.array_equal(host_u32(got), want), (M, N, K, engine)


@pytest.mark.parametrize("engine", [0, 1, 2])
def test_random_bitplane_shapes(seed, engine):
    import paper_1609_07061_amd as q

    cases = [(2, 1, [1, 2], [1], 0, 1), (4, 1, [1, 2, 4, -8], [1], 0, 1), (2, 2, [1, -2], [1, 2], 0, 0),
             (4, 4, [1, 2, 4, -8], [1, 2, 4, -8], 0, 0), (8, 1, [1 << p for p in range(8)], [-1], 0, 1),
             (1, 1, [-3], [5], 1, 0), (2, 1, [2, 4], [3], 1, 1), (3, 2, [1, 2, 4], [1, -2], 0, 1)]
    Ms = _rand_ints(seed, 1020, len(cases), 1, 400)
    Ns = _rand_ints(seed, 1021, len(cases), 1, 400)
    Ks = _rand_ints(seed, 1022, len(cases), 1, 1500)
    for i, ((Pa, Pb, ca, cw, ma, mw), M, N, K) in enumerate(zip(cases, Ms, Ns, Ks)):
        pa = qi.bernoulli_bits(seed, 1030 + i, (Pa, M, K))
        pw = qi.bernoulli_bits(seed, 1050 + i, (Pb, N, K))
        want = oracle.gemm_planes(pa, ca, ma, pw, cw, mw)
        got = run_on_engine(q.qnn_bitplane_gemm, dev(np_pack_bits(pa)), ca, ma, dev(np_pack_bits(pw)), cw, mw, K,
                            engine=engine, takes=engine_takes(engine, Pa, Pb, ca, cw))
        if got is None:  # refused with status 5, as documented for this (engine, case) pair
            continue
        assert np.array_equal(host(got), want), (Pa, Pb, ca, cw, ma, mw, M, N, K, engine)
