"""Parity of the quantizer front ends (Sec. 3), the affine BatchNorm of the output layer (Alg. 4), the packed-bit
transpose and the backward products of Alg. 1 against the CPU oracle: through the C ABI, element by element, bit exact.
Where a float decides an integer (a quantization code) both sides decide in the precision the definition names, so the
codes are compared for equality too."""
import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi
from qnn_testlib import dev, host, host_u32, np_pack_bits, np_pack_pm1, np_unpack_bits

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


def planes_of(codes: np.ndarray, nbits: int) -> np.ndarray:
    """Packed two's-complement planes of int32 codes, by the oracle's own split and pack."""
    low = (codes.astype(np.int64) & ((1 << nbits) - 1)).astype(np.int32)
    return np.stack([oracle.pack_bits(pl.astype(np.int8)) for pl in oracle.split_planes(low, nbits)])


def edge_floats(seed, stream, shape, scale):
    """N(0, scale^2) values with the float edge cases planted, plus exact ties and powers of two."""
    x = qi.with_special_floats(qi.normal_f32(seed, stream, shape) * np.float32(scale), seed, stream + 1)
    flat = x.reshape(-1)
    ties = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 0.125, 0.375, 1.0, 2.0, 4.0, -8.0, 2.0 ** -140, 3 * 2.0 ** -149,
                     1.41421353816986083984375, 1.414213657379150390625], dtype=np.float32)
    n = min(len(ties), flat.size)
    pos = (qi.raw_u64(seed, stream + 2, n) % np.uint64(flat.size)).astype(np.int64)
    flat[pos] = ties[:n]
    return x


@pytest.mark.parametrize("rows,K", [(1, 1), (3, 31), (5, 64), (7, 65), (4, 300), (9, 1000), (33, 4099), (5, 1024), (3, 2048),
                                     (33, 4100), (2, 6148)])
@pytest.mark.parametrize("step,qmin,qmax,nbits", [(0.25, -8, 7, 4), (1.0, 0, 3, 2), (0.1, 0, 15, 4), (1.0 / 3.0, -2, 1, 2),
                                                 (0.05, -128, 127, 8), (0.5, 0, 255, 8), (2.0, 0, 1, 1)])
def test_linear_quant_planes(seed, rows, K, step, qmin, qmax, nbits):
    x = edge_floats(seed, 2000, (rows, K), 3.0)
    want = planes_of(oracle.linear_quant(x, step, qmin, qmax), nbits)
    got = host_u32(q.qnn_linear_quant_planes(dev(x), step, qmin, qmax, nbits))
    assert np.array_equal(got, want)


def test_linear_quant_planes_feed_the_product(seed):
    """fp32 activations -> 2-bit unsigned codes -> planes -> product with +-1 weights equals the oracle's integer
    product of the oracle's codes (the path of the 2-bit activation networks of Sec. 4.3)."""
    M, N, K = 70, 40, 200
    x = np.abs(qi.normal_f32(seed, 2010, (M, K)))
    w = qi.pm1(seed, 2011, (N, K))
    codes = oracle.linear_quant(x, 0.5, 0, 3)
    planes = q.qnn_linear_quant_planes(dev(x), 0.5, 0, 3, 2)
    got = host(q.qnn_bitplane_gemm(planes, [1, 2], q.PLANE_BIT, dev(np_pack_pm1(w)[None]), [1], q.PLANE_SIGN, K))
    assert np.array_equal(got, oracle.gemm_int(codes, w.astype(np.int32)))


def test_linear_quant_planes_strided_and_padding(seed):
    rows, K, ldx = 6, 70, 96
    buf = qi.normal_f32(seed, 2020, (rows, ldx))
    out = torch.full((3, rows, 5), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_linear_quant_planes(dev(buf)[:, :K], 0.25, -4, 3, 3, out=out[:, :, :3])
    got = host_u32(out)
    assert np.array_equal(got[:, :, :3], planes_of(oracle.linear_quant(buf[:, :K], 0.25, -4, 3), 3))
    assert (got[:, :, 3:] == 0x5A5A5A5A).all()


@pytest.mark.parametrize("rows,K", [(1, 1), (3, 33), (5, 64), (4, 300), (17, 2051), (5, 1024), (9, 2052), (3, 6144)])
@pytest.mark.parametrize("emin,emax,nbits", [(-3, 2, 4), (-6, 0, 4), (-10, 4, 5), (0, 0, 2), (-126, -120, 4), (-20, 10, 6)])
def test_log_quant_planes_codes(seed, rows, K, emin, emax, nbits):
    x = edge_floats(seed, 2100, (rows, K), 2.0 ** ((emin + emax) // 2))
    want = planes_of(oracle.log_quant(x, emin, emax).astype(np.int32), nbits)
    got = host_u32(q.qnn_log_quant_planes(dev(x), emin, emax, nbits))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("rows,K", [(9, 333), (7, 2060)])  # the second shape takes the 16-byte-load kernel
@pytest.mark.parametrize("emin,emax,nbits", [(-3, 2, 8), (-6, 0, 8), (-2, 0, 4), (0, 0, 2)])
def test_log_quant_planes_values_and_gate(seed, emin, emax, nbits, rows, K):
    g = edge_floats(seed, 2200, (rows, K), 2.0 ** emax / 4)
    a = qi.with_special_floats(qi.normal_f32(seed, 2210, (rows, K)), seed, 2211)
    a.reshape(-1)[:6] = [1.0, -1.0, 1.0000001, -1.0000001, 0.0, 0.99999994]
    for gate in (None, a):
        gg = g if gate is None else oracle.ste_mask(g, gate)
        want = planes_of(oracle.log_code_value(oracle.log_quant(gg, emin, emax)), nbits)
        got = host_u32(q.qnn_log_quant_planes(dev(g), emin, emax, nbits, as_value=True,
                                              gate=None if gate is None else dev(gate)))
        assert np.array_equal(got, want)


def test_quant_argument_errors():
    x = torch.zeros((2, 40), dtype=torch.float32, device="cuda")
    for bad in (lambda: q.qnn_linear_quant_planes(x, 0.0, 0, 3, 2), lambda: q.qnn_linear_quant_planes(x, 1.0, 0, 4, 2),
                lambda: q.qnn_linear_quant_planes(x, 1.0, -3, 1, 2), lambda: q.qnn_linear_quant_planes(x, 1.0, 2, 1, 2),
                lambda: q.qnn_log_quant_planes(x, 0, 7, 4), lambda: q.qnn_log_quant_planes(x, 0, 3, 4, as_value=True),
                lambda: q.qnn_log_quant_planes(x, 3, 1, 4)):
        with pytest.raises(q.QnnError) as e:
            bad()
        assert e.value.status == 2


@pytest.mark.parametrize("M,N", [(1, 1), (5, 10), (300, 10), (64, 1000), (10000, 10)])
def test_batchnorm_affine(seed, M, N):
    s = qi.uniform_int(seed, 2300, (M, N), -200000, 200000)
    s.reshape(-1)[: min(4, s.size)] = [2 ** 24 + 1, -(2 ** 24) - 3, 2 ** 30 + 65, 0][: min(4, s.size)]
    scale = qi.normal_f32(seed, 2301, (N,)) * np.float32(0.01)
    shift = qi.normal_f32(seed, 2302, (N,))
    got = host(q.qnn_batchnorm_affine(dev(s), dev(scale), dev(shift)))
    want = oracle.bn_affine(s, scale, shift)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("rows,cols", [(1, 1), (31, 33), (64, 32), (65, 31), (100, 70), (300, 129), (1000, 257), (70, 4099)])
@pytest.mark.parametrize("P", [1, 3])
def test_transpose_bits(seed, rows, cols, P):
    bits = qi.bernoulli_bits(seed, 2400, (P, rows, cols))
    got = host_u32(q.qnn_transpose_bits(dev(np_pack_bits(bits)), cols))
    want = np.stack([oracle.pack_bits(np.ascontiguousarray(bits[p].T).astype(np.int8)) for p in range(P)])
    assert np.array_equal(got, want)


@pytest.mark.parametrize("rows,cols,ld_in,ld_out", [(1024, 1024, 32, 32), (1000, 1000, 32, 32), (600, 4000, 128, 20),
                                                    (4100, 300, 12, 132), (513, 257, 12, 20), (2050, 2050, 68, 68)])
@pytest.mark.parametrize("P", [1, 2])
def test_transpose_bits_large_padded_rows(seed, rows, cols, ld_in, ld_out, P):
    """Rows of whole 16-byte groups on both sides: the tiled kernel.  The padding words of the input hold garbage; the
    padding words of the output (beyond ceil(rows / 32)) must be left alone."""
    bits = qi.bernoulli_bits(seed, 2420, (P, rows, cols))
    cw, rw = (cols + 31) // 32, (rows + 31) // 32
    src = torch.full((P, rows, ld_in), 0x3C3C3C3C, dtype=torch.int32, device="cuda")
    src[:, :, :cw] = dev(np_pack_bits(bits))
    out = torch.full((P, cols, ld_out), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_transpose_bits(src[:, :, :cw], cols, out=out[:, :, :rw])
    got = host_u32(out)
    want = np.stack([oracle.pack_bits(np.ascontiguousarray(bits[p].T).astype(np.int8)) for p in range(P)])
    assert np.array_equal(got[:, :, :rw], want)
    assert (got[:, :, rw:] == 0x5A5A5A5A).all()


def test_transpose_bits_strided_and_padding(seed):
    rows, cols = 70, 45
    bits = qi.bernoulli_bits(seed, 2410, (2, rows, cols))
    src = torch.full((2, rows, 4), 0, dtype=torch.int32, device="cuda")
    src[:, :, :2] = dev(np_pack_bits(bits))
    out = torch.full((2, cols, 5), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    q.qnn_transpose_bits(src[:, :, :2], cols, out=out[:, :, :3])
    got = host_u32(out)
    want = np.stack([oracle.pack_bits(np.ascontiguousarray(bits[p].T).astype(np.int8)) for p in range(2)])
    assert np.array_equal(got[:, :, :3], want)
    assert (got[:, :, 3:] == 0x5A5A5A5A).all()


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 9), (64, 32, 96), (100, 70, 130), (257, 300, 513), (1000, 512, 1024)])
@pytest.mark.parametrize("emin,emax", [(-6, 0), (-2, 0)])
def test_binary_backward(seed, M, N, K, emin, emax):
    """Alg. 1 backward block for one layer: fp32 gradient, straight-through mask, LogQuant to fixed-point values,
    then g_a = g W and g_W = g^T a on packed operands; every element against the oracle's chain of the same steps."""
    nbits = emax - emin + 2
    g = qi.normal_f32(seed, 2500, (M, N)) * np.float32(0.2)
    pre = qi.normal_f32(seed, 2501, (M, N)) * np.float32(0.8)
    w = qi.pm1(seed, 2502, (N, K))
    a = qi.pm1(seed, 2503, (M, K))
    gq = oracle.log_code_value(oracle.log_quant(oracle.ste_mask(g, pre), emin, emax))
    want_ga, want_gw = oracle.backward(gq, w, a)
    G = q.qnn_log_quant_planes(dev(g), emin, emax, nbits, as_value=True, gate=dev(pre))
    coef = [1 << p for p in range(nbits - 1)] + [-(1 << (nbits - 1))]
    ga, gw = q.qnn_binary_backward(G, coef, q.PLANE_BIT, N, dev(np_pack_pm1(w)), dev(np_pack_pm1(a)), K)
    assert np.array_equal(host(ga), want_ga)
    assert np.array_equal(host(gw), want_gw)


def test_binary_backward_workspace_errors(seed):
    M, N, K = 40, 33, 70
    G = dev(np_pack_bits(qi.bernoulli_bits(seed, 2600, (2, M, N))))
    W, A = dev(np_pack_pm1(qi.pm1(seed, 2601, (N, K)))), dev(np_pack_pm1(qi.pm1(seed, 2602, (M, K))))
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(q.QnnError) as e:
        q.qnn_binary_backward(G, [1, -2], q.PLANE_BIT, N, W, A, K, workspace=small)
    assert e.value.status == 6
    with pytest.raises(q.QnnError) as e:
        q.qnn_binary_backward(G, [2 ** 30, 2 ** 30], q.PLANE_BIT, N, W, A, K)
    assert e.value.status == 4


# ---------------------------------------------------------------- repetition of binary 2-D filters (Sec. 5)
@pytest.mark.parametrize("B,H,W,cin,cout,pad,bits", [(2, 6, 5, 7, 40, 1, 2), (1, 8, 8, 3, 600, 1, 1), (3, 4, 4, 5, 9, 0, 1),
                                                    (2, 9, 7, 70, 130, 1, 2), (1, 3, 3, 33, 300, 1, 4)])
def test_conv2d_dedup(seed, B, H, W, cin, cout, pad, bits):
    """The convolution through the distinct 2-D filters equals the oracle's direct convolution on every element, and the
    per-channel counts of distinct filters equal the oracle's."""
    u = qi.uniform_int(seed, 3100, (B, H, W, cin), 0, (1 << bits) - 1)
    w = qi.pm1(seed, 3101, (cout, 3, 3, cin))
    if cout == 600:  # plant exact repeats and negations on top of the ones chance provides
        w[1] = w[0]
        w[2] = -w[0]
    A = dev(np.stack([np_pack_bits((u >> p) & 1) for p in range(bits)]))
    got, counts = q.qnn_conv2d_dedup(A, [1 << p for p in range(bits)], cin, dev(np_pack_pm1(w)), pad)
    assert np.array_equal(host(got), oracle.conv2d(u, w.astype(np.int32), pad))
    assert np.array_equal(host(counts), oracle.filter_unique(w))


def test_conv2d_dedup_in_image_chunks_and_errors(seed):
    B, H, W, cin, cout = 5, 6, 6, 40, 64
    u = qi.uniform_int(seed, 3110, (B, H, W, cin), 0, 3)
    w = qi.pm1(seed, 3111, (cout, 3, 3, cin))
    A = dev(np.stack([np_pack_bits((u >> p) & 1) for p in range(2)]))
    Wp = dev(np_pack_pm1(w))
    need = q._lib.qnn_conv2d_dedup_workspace_bytes(B, H, W, cin, cout, 1)  # room for one image: five chunks
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    got, _ = q.qnn_conv2d_dedup(A, [1, 2], cin, Wp, 1, workspace=ws)
    assert np.array_equal(host(got), oracle.conv2d(u, w.astype(np.int32), 1))
    with pytest.raises(q.QnnError) as e:
        q.qnn_conv2d_dedup(A, [1, 2], cin, Wp, 1, workspace=ws[: need - 256])
    assert e.value.status == 6
    with pytest.raises(q.QnnError) as e:
        q.qnn_conv2d_dedup(A, [4000, 2], cin, Wp, 1)
    assert e.value.status == 4
