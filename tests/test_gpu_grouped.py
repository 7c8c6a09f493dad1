"""GPU parity of the depthwise / grouped nested convolution (the layers of the lightweight CNNs of the
paper's evaluation, Sec. 4), full-bit and part-bit, against the CPU oracle.  Bar: int32 accumulators and
int8 outputs bit exact, fp32 outputs identical."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, dev, run_gconv_both
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def make_case(nq, C, K, n, l, seed):
    w_int, scale = tl.weights(C, K, inputs.he_sigma(K), n, seed)
    return Case(nq, w_int, scale, n, l)


@pytest.mark.parametrize("geom", [
    # B, H, W, C, groups, KH, stride, pad
    (2, 14, 14, 32, 32, 3, 1, 1),        # depthwise, half a channel tile
    (2, 15, 13, 64, 64, 3, 2, 1),        # stride 2, odd sizes
    (1, 9, 7, 144, 144, 3, 1, 1),        # two and a quarter channel tiles, pixel count not a multiple of 16
    (3, 7, 7, 96, 96, 3, 1, 1),          # rows shorter than a pixel tile: tiles run across rows and images
    (2, 12, 12, 16, 16, 3, 1, 0),        # no padding, a single 16-channel piece
    (1, 16, 16, 240, 240, 5, 1, 2),      # 5x5 (25 taps)
    (2, 17, 15, 96, 96, 5, 2, 2),        # 5x5, stride 2
    (2, 10, 10, 128, 32, 3, 1, 1),       # 32 groups of 4 channels
    (1, 11, 9, 64, 32, 3, 2, 1),         # groups of 2
    (1, 8, 8, 80, 20, 5, 1, 2),          # groups of 4, 5x5: K = 100, two K steps of the pages
    (1, 6, 6, 48, 48, 1, 1, 0),          # 1x1 depthwise: a per-channel scaling
    (2, 3, 3, 32, 32, 3, 1, 1),          # image smaller than a pixel tile
])
def test_geometries(nq, geom):
    B, H, W, C, groups, KH, stride, pad = geom
    gs = C // groups
    K = KH * KH * gs
    case = make_case(nq, C, K, 8, 2, seed=sum(geom))
    assert case.pages_match()
    x = inputs.uniform_activations((B, H, W, C), seed=C + H)
    for full in (True, False):
        run_gconv_both(nq, case, x, (KH, KH, stride, pad), groups, full, s_a=0.02)
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KH) // stride + 1
    bias = inputs.small_floats(C, 0.1, seed=3)
    res = inputs.uniform_activations((B, Ho, Wo, C), seed=C)
    for full in (True, False):
        run_gconv_both(nq, case, x, (KH, KH, stride, pad), groups, full, s_a=0.02, bias=bias, relu=True,
                       out_int8=True, inv_s_out=5.0)
        run_gconv_both(nq, case, x, (KH, KH, stride, pad), groups, full, s_a=0.02, bias=bias, residual=res, s_r=0.04,
                       relu=True, out_int8=True, inv_s_out=5.0)


@pytest.mark.parametrize("n,l", [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)])
def test_every_nesting(nq, n, l):
    B, H, W, C = 2, 10, 9, 96
    case = make_case(nq, C, 9, n, l, seed=n * 7 + l)
    x = inputs.uniform_activations((B, H, W, C), seed=l)
    for full in (True, False):
        run_gconv_both(nq, case, x, (3, 3, 1, 1), C, full, s_a=0.02, relu=True)
        run_gconv_both(nq, case, x, (3, 3, 1, 1), C, full, s_a=0.02, relu=True, out_int8=True, inv_s_out=4.0)


def test_extreme_values_and_compensated_format(nq):
    from oracle import nq_oracle as oracle
    from nq_testlib import host
    B, H, W, C = 1, 9, 9, 64
    # the largest sums: every activation and weight at the end of its range
    for wv in (-128, 127):
        case = Case(nq, np.full((C, 9), wv, np.int8), np.full(C, 0.001, np.float32), 8, 2)
        x = np.full((B, H, W, C), -128, np.int8)
        for full in (True, False):
            run_gconv_both(nq, case, x, (3, 3, 1, 1), C, full, s_a=0.01)
    # compensated lower part (signed l + 1 bits, round-to-nearest w_high)
    n, l, gs = 8, 3, 4
    K = 9 * gs
    w, scale = tl.weights(C, K, inputs.he_sigma(K), n, seed=21)
    W_ = nq.NestedWeight.from_int8(dev(w), dev(scale), nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1))
    hi, _ = oracle.decompose(w, n, l, "rtn")
    x = inputs.uniform_activations((2, H, W, C), seed=8)
    cs = nq.nq_conv_shape(2, H, W, C, C, 3, 3, 1, 1)
    for full in (True, False):
        w4 = (w if full else hi).astype(np.int16).reshape(C, 3, 3, gs)
        acc_ref = oracle.conv_grouped_acc(x, w4, C // gs, 1, 1)
        acc = torch.empty((2, H, W, C), dtype=torch.int32, device="cuda")
        y = torch.empty((2, H, W, C), dtype=torch.float32, device="cuda")
        (nq.nq_gconv_full if full else nq.nq_gconv_part)(dev(x), cs, C // gs, W_.desc,
                                                         nq.make_epilogue(0.02, d_acc_dump=acc), y)
        torch.cuda.synchronize()
        assert np.array_equal(host(acc), acc_ref)
        assert np.array_equal(host(y), oracle.epilogue(acc_ref, 0.02, scale, part_l_bits=0 if full else l))


def test_unsupported_shapes_are_refused(nq):
    x = torch.zeros((1, 8, 8, 64), dtype=torch.int8, device="cuda")
    y = torch.zeros((1, 8, 8, 64), dtype=torch.float32, device="cuda")
    epi = nq.make_epilogue(0.02)
    for C, groups, KH, status in ((64, 8, 3, "NQ_ERR_UNSUPPORTED"),      # groups of 8
                                  (64, 64, 7, "NQ_ERR_UNSUPPORTED"),     # 49 taps
                                  (24, 24, 3, "NQ_ERR_UNSUPPORTED"),     # channels not a multiple of 16
                                  (64, 5, 3, "NQ_ERR_SHAPE")):           # groups do not divide the channels
        gs = max(C // groups, 1)
        W_ = nq.NestedWeight(C, KH * KH * gs, nq.make_cfg(8, 2))
        cs = nq.nq_conv_shape(1, 8, 8, C, C, KH, KH, 1, KH // 2)
        with pytest.raises(nq.NQError) as e:
            nq.nq_gconv_part(x, cs, groups, W_.desc, epi, y)
        assert e.value.status == getattr(nq, status), (C, groups, KH)
