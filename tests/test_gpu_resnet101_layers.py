"""GPU parity of every distinct layer shape of the ResNet-101 plan at batch 128, the batch the benchmark's
forward runs at, through nq_conv_full / nq_conv_part with the epilogue the network walker uses (bias, ReLU,
residual where the block adds one, int8 output).  The kernel and its tile shape are the library's own choice
for the shape, i.e. the instantiations the benchmark times.  Every output element is compared (bit exact):
the C oracle with OpenMP needs well under a second per layer."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, dev, host
from oracle import nq_oracle as oracle
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

BATCH = 128


def layer_shapes():
    """(H, W, Cin, Cout, k, stride, pad, relu, has_residual) of the plan's convolutions, each once."""
    from paper_2506_17870_amd import network
    hw, seen = {0: (224, 224)}, []
    for op in network.resnet101_plan():
        h, w = hw[op["src"]]
        if op["op"] == "conv":
            key = (h, w, op["cin"], op["cout"], op["k"], op["stride"], op["pad"], op["relu"],
                   op["residual"] is not None)
            if key not in seen:
                seen.append(key)
            hw[op["dst"]] = network.out_hw(h, w, op["k"], op["stride"], op["pad"])
        elif op["op"] == "maxpool":
            hw[op["dst"]] = network.out_hw(h, w, op["k"], op["stride"], op["pad"])
        else:
            hw[op["dst"]] = (1, 1)
    return seen


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def test_plan_has_the_expected_shapes():
    assert len(layer_shapes()) == 24


@pytest.mark.parametrize("shape", layer_shapes(), ids=lambda s: "x".join(str(int(v)) for v in s))
def test_layer_at_batch_128(nq, shape):
    H, W, Cin, Cout, k, stride, pad, relu, has_res = shape
    K = k * k * Cin
    seed = H + Cin + Cout + k + stride
    w_int, scale = tl.weights(Cout, K, inputs.he_sigma(K), 8, seed=seed)
    case = Case(nq, w_int, scale, 8, 2)
    assert case.pages_match()
    x = inputs.uniform_activations((BATCH, H, W, Cin), seed=seed)
    if Cin > 3:
        x = np.maximum(x, 0)                      # the network's activations follow a ReLU
    bias = inputs.small_floats(Cout, 0.02, seed=seed)
    Ho, Wo = oracle.conv_out_hw(H, W, k, k, stride, pad)
    res = inputs.uniform_activations((BATCH, Ho, Wo, Cout), seed=seed + 1) if has_res else None
    s_a, s_r = 0.02, 0.03
    cs = nq.nq_conv_shape(BATCH, H, W, Cin, Cout, k, k, stride, pad)
    dx, d_bias = dev(x), dev(bias)
    d_res = dev(res) if has_res else None
    for full in (True, False):
        w4 = (case.ow_full if full else case.ow_part).reshape(Cout, k, k, Cin)
        acc = oracle.conv_acc(x, w4, stride, pad)
        okw = dict(s_a=s_a, s_w=scale, part_l_bits=0 if full else 2, bias=bias, residual=res, s_r=s_r, relu=relu)
        # an output step that spreads the codes over the int8 range without saturating most of them
        yf = oracle.epilogue(acc[:2], **{**okw, "residual": None if res is None else res[:2]})
        inv_s_out = float(40.0 / max(float(np.abs(yf).std()), 1e-6))
        y_ref = oracle.epilogue(acc, out_int8=True, inv_s_out=inv_s_out, **okw)
        del acc
        y = torch.full((BATCH, Ho, Wo, Cout), 77, dtype=torch.int8, device="cuda")
        epi = nq.make_epilogue(s_a, d_bias, d_res, s_r, relu, True, inv_s_out)
        (nq.nq_conv_full if full else nq.nq_conv_part)(dx, cs, case.W.desc, epi, y)
        torch.cuda.synchronize()
        got = host(y)
        assert np.array_equal(got, y_ref), f"int8 outputs differ ({'full' if full else 'part'}-bit)"
        assert np.unique(y_ref).size > 50          # the comparison is not one of saturated codes
