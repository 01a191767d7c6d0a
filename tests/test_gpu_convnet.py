"""Binarized ConvNet forward (Alg. 4 on the network shape of App. A) against the oracle, logits element by element:
small networks that exercise odd sizes, channel tails, pooling with flipped channels and every engine preference,
and the CIFAR-10 ConvNet of the paper's table at a batch the oracle finishes in seconds."""
import numpy as np
import pytest
import torch

import oracle
import qnn_inputs as qi
from qnn_testlib import dev, host, np_pack_pm1

pytestmark = pytest.mark.gpu


def _case(seed, B, H, Wd, C0, couts, pools, fcs, stream0, first_span=2000, span=12):
    x = qi.uniform_int(seed, stream0, (B, H, Wd, C0), 0, 255, dtype=np.uint8)
    conv_w, cin = [], C0
    for l, co in enumerate(couts):
        conv_w.append(qi.pm1(seed, stream0 + 1 + l, (co, 3, 3, cin)))
        cin = co
    h, w = H, Wd
    for p in pools:
        if p:
            h, w = h // 2, w // 2
    fc_w, fin = [], h * w * cin
    for j, fo in enumerate(fcs):
        fc_w.append(qi.pm1(seed, stream0 + 20 + j, (fo, fin)))
        fin = fo
    widths = list(couts) + list(fcs[:-1])
    T, flip = [], []
    for l, n in enumerate(widths):
        s = first_span if l == 0 else span
        T.append(qi.uniform_int(seed, stream0 + 40 + l, (n,), -s, s))
        flip.append(qi.bernoulli_bits(seed, stream0 + 60 + l, (n,)))
    return x, conv_w, list(pools), fc_w, T, flip


def _run(q, case, couts, fcs, engine=0, with_flip=True):
    x, conv_w, pools, fc_w, T, flip = case
    W = [dev(np_pack_pm1(w)) for w in conv_w] + [dev(np_pack_pm1(w)) for w in fc_w]
    got = q.qnn_binary_convnet_forward(dev(x), 8, couts, pools, fcs, W, [dev(t) for t in T],
                                       [dev(f) for f in flip] if with_flip else None, engine=engine)
    return host(got)


@pytest.mark.parametrize("engine", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("B,H,Wd,C0,couts,pools,fcs", [
    (2, 8, 8, 3, [32, 32, 64, 64], [0, 1, 0, 1], [24, 10]),        # the table's pattern in small
    (3, 6, 10, 3, [40, 64], [1, 0], [9, 6, 4]),                    # channel tails inside the network, odd map sizes
    (2, 5, 7, 2, [6], [1], [3]),                                   # odd sizes dropped by the pooling; tiny
    (5, 12, 12, 3, [128, 128, 256], [0, 1, 1], [100, 10]),         # wide enough for the matrix-core kernels
    (3, 9, 11, 1, [70, 32], [1, 1], [10]),                         # grey images; 99 pixels per image, 70 filters
    (2, 7, 7, 4, [32, 32], [0, 1], [5]),                           # four input channels: the first layer goes through planes
    (2, 6, 6, 3, [100, 32], [0, 1], [7]),                          # first layer: four words of filters, the last ragged
])
def test_convnet_small(seed, B, H, Wd, C0, couts, pools, fcs, engine):
    import paper_1609_07061_amd as q

    if couts[-1] % 32 and not (H // 2 ** sum(pools) == 1 and Wd // 2 ** sum(pools) == 1):
        case = _case(seed, B, H, Wd, C0, couts, pools, fcs, 1500)
        with pytest.raises(q.QnnError) as e:  # documented: the last map needs whole words of channels
            _run(q, case, couts, fcs, engine)
        assert e.value.status == 5
        return
    case = _case(seed, B, H, Wd, C0, couts, pools, fcs, 1500)
    want = oracle.convnet(*case)
    assert np.array_equal(_run(q, case, couts, fcs, engine), want)


@pytest.mark.parametrize("with_flip", [True, False])
def test_convnet_ragged_shapes_on_the_panel_fed_convolution(seed, with_flip):
    """Non-square maps of 10 x 14 pixels, 420 pixels per batch (one whole tile of 256 rows and a ragged one), 256 channels
    into 200 filters (a ragged tile of filters) and 200 channels into 64 (not a multiple of 128: another kernel)."""
    import paper_1609_07061_amd as q

    couts, pools, fcs = [256, 200, 64], [0, 0, 1], [10]
    x, conv_w, pools, fc_w, T, flip = _case(seed, 3, 10, 14, 3, couts, pools, fcs, 1800)
    want = oracle.convnet(x, conv_w, pools, fc_w, T, flip if with_flip else None)
    got = _run(q, (x, conv_w, pools, fc_w, T, flip), couts, fcs, with_flip=with_flip)
    assert np.array_equal(got, want)
    engines = q.qnn_last_engines()
    assert engines[0] == 2 and engines[1] == 3 and engines[2] != 3, engines


def test_convnet_panel_fed_convolution_with_1024_channels(seed):
    """1024 channels into 40 filters: the patch's 9216 bits are nine whole groups of 1024, so every step of a tile's last
    group is multiplied (with 128, 256 or 512 channels some are padding and are left out)."""
    import paper_1609_07061_amd as q

    couts, pools, fcs = [1024, 40, 32], [0, 0, 1], [6]
    case = _case(seed, 2, 8, 16, 3, couts, pools, fcs, 1900)
    want = oracle.convnet(*case)
    assert np.array_equal(_run(q, case, couts, fcs), want)
    engines = q.qnn_last_engines()
    assert engines[0] == 2 and engines[1] == 3, engines


def test_convnet_first_convolution_over_several_turns_per_wave(seed):
    """110 images of 30 x 31 pixels: 102 300 pixels are 3197 tiles of 32 (the last one ragged), more than the 3072 waves
    the first-layer kernel launches at most, so some waves take a second tile, whose patch bytes they asked for while
    working on the first."""
    import paper_1609_07061_amd as q

    couts, pools, fcs = [32], [1], [4]
    case = _case(seed, 110, 30, 31, 3, couts, pools, fcs, 2000)
    want = oracle.convnet(*case)
    assert np.array_equal(_run(q, case, couts, fcs), want)
    assert q.qnn_last_engines()[0] == 2


def test_convnet_panel_fed_convolution_over_several_tiles_per_workgroup(seed):
    """75 images of 31 x 31 pixels and 128 channels: 72 075 pixels are 282 tiles of 256 rows (the last one ragged) for the
    256 persistent workgroups, so some of them take a second tile."""
    import paper_1609_07061_amd as q

    couts, pools, fcs = [128, 128], [0, 1], [10]
    case = _case(seed, 75, 31, 31, 3, couts, pools, fcs, 2100)
    want = oracle.convnet(*case)
    assert np.array_equal(_run(q, case, couts, fcs), want)
    assert q.qnn_last_engines()[:2] == [2, 3]


def test_convnet_without_flips(seed):
    import paper_1609_07061_amd as q

    couts, pools, fcs = [32, 64], [1, 1], [16, 5]
    x, conv_w, pools, fc_w, T, flip = _case(seed, 4, 8, 8, 3, couts, pools, fcs, 1600)
    want = oracle.convnet(x, conv_w, pools, fc_w, T, None)
    assert np.array_equal(_run(q, (x, conv_w, pools, fc_w, T, flip), couts, fcs, with_flip=False), want)


def test_convnet_cifar10_architecture(seed):
    """The CIFAR-10 ConvNet of App. A: 2 x (128C3) - MP2 - 2 x (256C3) - MP2 - 2 x (512C3) - MP2 - 1024FC - 1024FC - 10,
    32 x 32 RGB inputs, batch 64; every logit against the oracle."""
    import paper_1609_07061_amd as q

    couts, pools, fcs = [128, 128, 256, 256, 512, 512], [0, 1, 0, 1, 0, 1], [1024, 1024, 10]
    case = _case(seed, 64, 32, 32, 3, couts, pools, fcs, 1700, first_span=3000, span=40)
    want = oracle.convnet(*case)
    got = _run(q, case, couts, fcs)
    assert np.array_equal(got, want)
    engines = q.qnn_last_engines()
    # first layer: the byte kernel for images of up to three channels, reported as the matrix-core engine; the other
    # convolutions (128, 256, 512 channels in): the panel-fed FP4 kernel on the maps' sign planes
    assert len(engines) == 9 and engines[0] == 2 and all(e == 3 for e in engines[1:6]), engines
