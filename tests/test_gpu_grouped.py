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


def test_shapes_that_are_refused(nq):
    x = torch.zeros((1, 8, 8, 64), dtype=torch.int8, device="cuda")
    y = torch.zeros((1, 8, 8, 64), dtype=torch.float32, device="cuda")
    epi = nq.make_epilogue(0.02)
    W_ = nq.NestedWeight(64, 9 * 12, nq.make_cfg(8, 2))
    with pytest.raises(nq.NQError) as e:       # groups do not divide the channels
        nq.nq_gconv_part(x, nq.nq_conv_shape(1, 8, 8, 64, 64, 3, 3, 1, 1), 5, W_.desc, epi, y)
    assert e.value.status == nq.NQ_ERR_SHAPE
    W_ = nq.NestedWeight(48, 9 * 16, nq.make_cfg(8, 2))
    with pytest.raises(nq.NQError) as e:       # groups divide the input channels but not the output channels
        nq.nq_gconv_part(x, nq.nq_conv_shape(1, 8, 8, 64, 48, 3, 3, 1, 1), 32, W_.desc, epi, y)
    assert e.value.status == nq.NQ_ERR_SHAPE


# Shapes the matrix-core kernel does not take and the direct kernel does: (B, H, W, Cin, Cout, groups, KH, stride, pad)
ANY_GEOMS = [
    (2, 9, 8, 64, 64, 8, 3, 1, 1),        # ResNeXt-style groups of 8
    (1, 10, 10, 128, 128, 4, 3, 2, 1),    # groups of 32, stride 2
    (2, 7, 7, 48, 120, 3, 1, 1, 0),       # ShuffleNet-style grouped 1x1, 3 groups, more output than input channels
    (2, 7, 7, 60, 24, 3, 1, 1, 0),        # ... and fewer: 20 in, 8 out per group
    (1, 9, 9, 24, 24, 24, 3, 1, 1),       # depthwise over a channel count that is not a multiple of 16
    (1, 11, 11, 32, 32, 32, 7, 1, 3),     # depthwise 7x7: 49 taps
    (2, 6, 5, 9, 6, 3, 3, 1, 1),          # groups of 3 input channels: bytes fetched one by one
    (1, 8, 8, 10, 70, 2, 3, 2, 1),        # groups of 5 in, 35 out; more than one 64-channel run of lanes
    (1, 5, 5, 16, 16, 1, 3, 1, 1),        # one group: a dense convolution
    (3, 4, 4, 12, 12, 3, 2, 1, 0),        # even filter, no padding
]


@pytest.mark.parametrize("geom", ANY_GEOMS, ids=lambda g: "x".join(str(v) for v in g))
def test_wide_groups_and_unequal_channel_counts(nq, geom):
    B, H, W, Cin, Cout, groups, KH, stride, pad = geom
    gs = Cin // groups
    K = KH * KH * gs
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KH) // stride + 1
    x = inputs.uniform_activations((B, H, W, Cin), seed=Cin + H)
    bias = inputs.small_floats(Cout, 0.1, seed=3)
    res = inputs.uniform_activations((B, Ho, Wo, Cout), seed=Cout)
    for n, l in ((8, 2), (8, 5), (6, 3)):
        case = make_case(nq, Cout, K, n, l, seed=sum(geom) + n + l)
        for full in (True, False):
            run_gconv_both(nq, case, x, (KH, KH, stride, pad), groups, full, s_a=0.02)
            run_gconv_both(nq, case, x, (KH, KH, stride, pad), groups, full, s_a=0.02, bias=bias, residual=res, s_r=0.04,
                           relu=True, out_int8=True, inv_s_out=5.0)
    assert nq.nq_profile_last_kernel()[0] == 10


def test_wide_groups_every_nesting_compensated_and_unaligned(nq):
    from oracle import nq_oracle as oracle
    B, H, W, Cin, Cout, groups, KH = 2, 8, 7, 40, 24, 2, 3
    gs = Cin // groups
    K = KH * KH * gs
    xbuf = dev(inputs.uniform_activations((B * H * W * Cin + 4,), seed=5))
    for n, l in [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]:
        for fmt in ("unsigned", "compensated"):
            case = make_case(nq, Cout, K, n, l, seed=10 * n + l)
            if fmt == "compensated":
                case.cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
                case.W = nq.NestedWeight.from_int8(dev(case.w_int), dev(case.scale), case.cfg)
                hi, _ = oracle.decompose(case.w_int, n, l, "rtn")
                case.ow_part = hi.astype(np.int16)
                case.ow_full = case.w_int.astype(np.int16)
            for first in (0, 1):            # an input tensor that starts one byte off a dword boundary
                xv = xbuf[first:first + B * H * W * Cin].view(B, H, W, Cin)
                x = xv.cpu().numpy()
                w4 = case.ow_full.reshape(Cout, KH, KH, gs)
                acc_ref = oracle.conv_grouped_acc(x, w4, groups, 1, 1)
                acc = torch.empty((B, H, W, Cout), dtype=torch.int32, device="cuda")
                y = torch.empty((B, H, W, Cout), dtype=torch.float32, device="cuda")
                nq.nq_gconv_full(xv, nq.nq_conv_shape(B, H, W, Cin, Cout, KH, KH, 1, 1), groups, case.W.desc,
                                 nq.make_epilogue(0.02, d_acc_dump=acc), y)
                torch.cuda.synchronize()
                assert np.array_equal(acc.cpu().numpy(), acc_ref), (n, l, fmt, first)
                y_ref = oracle.epilogue(acc_ref, 0.02, case.scale)
                assert np.array_equal(y.cpu().numpy(), y_ref), (n, l, fmt, first)


def test_resnext_and_shufflenet_layers_reduced_batch(nq):
    """ResNeXt-50 32x8d stage-1 grouped 3x3 (56 x 56 x 256, 32 groups of 8) and a ShuffleNet (g = 3) stage-2 pair of grouped
    1x1 layers (28 x 28: 240 -> 60 and 60 -> 240), batch 2."""
    for (B, H, W, Cin, Cout, groups, KH, stride, pad) in ((2, 56, 56, 256, 256, 32, 3, 1, 1), (2, 28, 28, 240, 60, 3, 1, 1, 0),
                                                          (2, 28, 28, 60, 240, 3, 1, 1, 0)):
        gs = Cin // groups
        K = KH * KH * gs
        case = make_case(nq, Cout, K, 8, 2, seed=Cin + Cout)
        x = inputs.uniform_activations((B, H, W, Cin), seed=Cin)
        bias = inputs.small_floats(Cout, 0.1, seed=4)
        for full in (True, False):
            run_gconv_both(nq, case, x, (KH, KH, stride, pad), groups, full, s_a=0.02, bias=bias, relu=True, out_int8=True,
                           inv_s_out=5.0)