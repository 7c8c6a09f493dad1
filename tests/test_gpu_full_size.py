"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (same entry points, same epilogue options).  The C oracle with OpenMP finishes each of these in
seconds, so every output element is compared, not a sample."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, run_conv_both, run_gemm_both
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def test_resnet18_conv_full_batch(nq):
    # batch 32, 56x56x64 -> 64, 3x3 stride 1 pad 1, INT8 nesting INT6; bias + ReLU, fp32 out (as bench.py)
    c = inputs.CONV_RESNET18
    K = 9 * c["Cin"]
    w_int, scale = tl.weights(c["Cout"], K, inputs.he_sigma(K), 8, seed=0)
    case = Case(nq, w_int, scale, 8, 2)
    x = inputs.uniform_activations((c["B"], c["H"], c["W"], c["Cin"]), seed=0)
    bias = inputs.small_floats(c["Cout"], 0.1, seed=2)
    for full in (False, True):
        run_conv_both(nq, case, x, (3, 3, 1, 1), full, s_a=0.02, bias=bias, relu=True)
    run_conv_both(nq, case, x, (3, 3, 1, 1), True, s_a=0.02, bias=bias, relu=True, out_int8=True, inv_s_out=2.5)


@pytest.mark.parametrize("l", [2, 4])
def test_resnet101_bottleneck_full_batch(nq, l):
    # batch 64, 14x14: 1x1 1024->256, 3x3 256->256, 1x1 256->1024; ReLU-clipped N(0,1) activations
    x0, s0 = tl.relu_activations((64, 14, 14, 1024), seed=7)
    for i, g in enumerate(inputs.BOTTLENECK_RESNET101):
        K = g["KH"] * g["KW"] * g["Cin"]
        w_int, scale = tl.weights(g["Cout"], K, inputs.he_sigma(K), 8, seed=10 * l + i)
        case = Case(nq, w_int, scale, 8, l)
        x = x0 if g["Cin"] == 1024 else tl.relu_activations((64, 14, 14, g["Cin"]), seed=i)[0]
        for full in (True, False):
            run_conv_both(nq, case, x, (g["KH"], g["KW"], g["stride"], g["pad"]), full, s_a=float(s0), relu=True,
                          out_int8=True, inv_s_out=6.0)
        if i == 2:   # block output: residual added, fp32 out
            run_conv_both(nq, case, x, (1, 1, 1, 0), True, s_a=float(s0), residual=x0, s_r=float(s0), relu=True)


@pytest.mark.parametrize("idx", [0, 1])
def test_vit_mlp_full_size(nq, idx):
    # M = 12608 (197 x 64), fc1 768 -> 3072 and fc2 3072 -> 768, INT8 nesting INT5 (l = 3)
    g = inputs.VIT_MLP[idx]
    w_int, scale = tl.weights(g["N"], g["K"], g["sigma"], 8, seed=idx)
    case = Case(nq, w_int, scale, 8, g["l_bits"])
    x, s_a = tl.gaussian_activations((g["M"], g["K"]), seed=idx)
    bias = inputs.small_floats(g["N"], 0.05, seed=idx)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=float(s_a), bias=bias)
    run_gemm_both(nq, case, x, True, s_a=float(s_a), bias=bias, out_int8=True, inv_s_out=20.0)


def test_resnet101_early_layers_full_resolution(nq):
    # the layers that depend on the image size, at 224 x 224 and a reduced batch: the 7x7 stride-2 stem on three
    # input channels (few-channel kernel, several units per block) and the first bottleneck's 1x1 64 -> 256
    # at 56 x 56 (register-stationary kernel with four channel tiles per block), with the residual epilogue
    K = 7 * 7 * 3
    w_int, scale = tl.weights(64, K, inputs.he_sigma(K), 8, seed=41)
    case = Case(nq, w_int, scale, 8, 2)
    x, s_x = tl.gaussian_activations((4, 224, 224, 3), seed=41)
    bias = inputs.small_floats(64, 0.1, seed=42)
    for full in (True, False):
        run_conv_both(nq, case, x, (7, 7, 2, 3), full, s_a=float(s_x), bias=bias, relu=True, out_int8=True,
                      inv_s_out=9.0)
    w_int, scale = tl.weights(256, 64, inputs.he_sigma(64), 8, seed=43)
    case = Case(nq, w_int, scale, 8, 2)
    x, s_x = tl.relu_activations((4, 56, 56, 64), seed=43)
    res = inputs.uniform_activations((4, 56, 56, 256), seed=44)
    for full in (True, False):
        run_conv_both(nq, case, x, (1, 1, 1, 0), full, s_a=float(s_x), residual=res, s_r=0.04, relu=True,
                      out_int8=True, inv_s_out=5.0)


@pytest.mark.parametrize("geom", [(112, 64, 64, 3, 2), (56, 128, 128, 3, 1), (28, 240, 240, 5, 1), (56, 128, 32, 3, 1)])
def test_depthwise_layers_full_batch(nq, geom):
    # batch 32, the sizes bench_configs.py times: MobileNet 112x112x64 stride 2 and 56x56x128, EfficientNet-B0
    # 5x5 28x28x240, ResNeXt 32x4d 56x56x128 in 32 groups; int8 in and out, bias + ReLU, INT(8|5)
    from nq_testlib import run_gconv_both
    hw, C, groups, k, stride = geom
    K = k * k * (C // groups)
    w_int, scale = tl.weights(C, K, inputs.he_sigma(K), 8, seed=hw + C)
    case = Case(nq, w_int, scale, 8, 3)
    x = inputs.uniform_activations((32, hw, hw, C), seed=hw)
    bias = inputs.small_floats(C, 0.1, seed=1)
    for full in (True, False):
        run_gconv_both(nq, case, x, (k, k, stride, k // 2), groups, full, s_a=0.02, bias=bias, relu=True,
                       out_int8=True, inv_s_out=3.0)


def test_quantiser_full_size(nq):
    # 4096 x 4096 fp32 weights (the size bench_configs.py times), INT(8|6): scales and pages bit exact
    from nq_testlib import dev, host
    from oracle import nq_oracle as oracle
    N = K = 4096
    w = inputs.float_weights(N, K, 0.02, seed=3)
    wi_ref, s_ref = oracle.quantize(w, 8)
    ph_ref, pl_ref = oracle.decompose_pack(wi_ref, 8, 2)
    d_s = torch.empty(N, dtype=torch.float32, device="cuda")
    ph = torch.zeros(ph_ref.size, dtype=torch.uint8, device="cuda")
    pl = torch.zeros(pl_ref.size, dtype=torch.uint8, device="cuda")
    nq.nq_quantize_decompose_pack(dev(w), N, K, nq.make_cfg(8, 2), d_s, ph, pl)
    torch.cuda.synchronize()
    assert np.array_equal(host(d_s).view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(host(ph), ph_ref) and np.array_equal(host(pl), pl_ref)


@pytest.mark.parametrize("M,l", [(16, 2), (64, 4), (33, 3)])
def test_weight_bound_linear_long_rows(nq, M, l):
    # few rows against a long reduction (the weight-bound stand-in of the linear configuration: the packed
    # pages are the traffic); N small enough that every block has a compute unit to itself
    N, K = 2048, 8192
    w_int, scale = tl.weights(N, K, 0.02, 8, seed=50 + l)
    case = Case(nq, w_int, scale, 8, l)
    x = inputs.uniform_activations((M, K), seed=51 + l)
    bias = inputs.small_floats(N, 0.05, seed=l)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.02, bias=bias)
    run_gemm_both(nq, case, x, True, s_a=0.02, bias=bias, relu=True, out_int8=True, inv_s_out=4.0)
