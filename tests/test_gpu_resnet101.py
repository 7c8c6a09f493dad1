"""Whole-network parity: ResNet-101-shaped CNN (104 convolutions + fc), random He-normal weights, every layer
INT8 nesting INT6, int8 activations with per-layer steps calibrated once by the CPU oracle.  Full-bit forward,
then part-bit forward after paging every lower-bit page out, then full-bit again after paging them back in.
Every intermediate int8 tensor and the fp32 logits are compared with the oracle's (bit exact / 1e-5)."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import dev, host, oracle_cnn_forward
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

# Large enough that the rows of the layers (8 * Ho * Wo) span several block tiles and that the large-GEMM kernel's
# choice of the tile height differs between layers (25088 rows at 56 x 56 down to 392 at 7 x 7).
BATCH = 8


def test_resnet101_full_part_full():
    import paper_2506_17870_amd as nq
    from paper_2506_17870_amd import network
    n_bits, l_bits = 8, 2
    ops = network.resnet101_plan()
    assert sum(1 for op in ops if op["op"] == "conv") == 104
    weights = tl.plan_weights(ops, n_bits, seed=0)
    assert sum(w[0].size for w in weights if w is not None) == 44_442_816   # conv + fc weights of ResNet-101
    x, s_x = tl.gaussian_activations((BATCH, 224, 224, 3), seed=0)

    logits_o, tens_o, scales = oracle_cnn_forward(ops, weights, x, s_x, n_bits, l_bits, full=True)
    logits_op, tens_op, _ = oracle_cnn_forward(ops, weights, x, s_x, n_bits, l_bits, full=False, scales=scales)

    # the network quantises the same float draws on the device (nq_quantize); the oracle's codes came from its own
    model = network.NestedCNN(ops, network.plan_float_weights(ops, seed=0), n_bits, l_bits)
    # the walker's own calibration (fp32-output pass + nq_tensor_scale per layer) finds the oracle's steps
    model.calibrate(dev(x), s_x)
    for t, s in scales.items():
        assert model.out_scale[t] == s, f"calibrated step of tensor {t} differs: {model.out_scale[t]} vs {s}"

    def check(full, logits_ref, tens_ref, branch_stream=None):
        keep = {}
        logits = model.forward(dev(x), s_x, full=full, keep=keep, branch_stream=branch_stream)
        torch.cuda.synchronize()
        for op in ops:
            if op["op"] == "fc":
                continue
            got, want = host(keep[op["dst"]]), tens_ref[op["dst"]]
            assert np.array_equal(got, want), f"tensor {op['dst']} after {op} differs ({'full' if full else 'part'})"
        got = host(logits)
        assert np.all(np.abs(got - logits_ref) <= 1e-5 * np.maximum(np.abs(logits_ref), 1e-30))
        assert np.array_equal(got, logits_ref)

    check(True, logits_o, tens_o)
    model.page_out_low()                                    # downgrade the whole model
    with pytest.raises(nq.NQError):
        model.forward(dev(x), s_x, full=True)
    check(False, logits_op, tens_op)
    side = torch.cuda.Stream()
    model.page_in_low(side)                                 # upgrade: 104 + 1 pages over a second stream
    check(True, logits_o, tens_o)
    # the projection shortcuts issued on a second stream beside their blocks' main paths: the same tensors
    assert len(model.branch_ops) == 4
    branch = torch.cuda.Stream()
    for buf in model.buf.values():
        buf.zero_()
    check(True, logits_o, tens_o, branch_stream=branch)
    check(False, logits_op, tens_op, branch_stream=branch)
    # the part-bit model is a different, coarser model: its logits differ from the full-bit ones
    assert not np.array_equal(logits_o, logits_op)
