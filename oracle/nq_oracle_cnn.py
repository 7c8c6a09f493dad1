"""Walks a CNN layer table (a list of ops as paper_2506_17870_amd.network.resnet101_plan() makes it: plain
dicts, no code) on the CPU oracle: every convolution / fc through the oracle's own decompose, pack,
unpack, integer convolution and fp32 epilogue, pooling through its pooling routines.  Test
infrastructure like the rest of oracle/: used by the GPU parity tests and by the CPU-baseline leg of the
benchmark, never by the library."""
import numpy as np

from . import nq_oracle as oracle


def oracle_cnn_forward(ops, weights, x, in_scale, n_bits, l_bits, full, scales=None, cache=None):
    """Walks a plan of paper_2506_17870_amd.network on the CPU oracle.  With scales=None every conv is first
    dequantised to fp32 to fix its int8 step (Eq. 1 per tensor: absmax / 127 in fp32, by the oracle's
    quantiser), which is returned for the other runs.  cache, if a dict, keeps each layer's weights as the
    oracle decomposed, packed and unpacked them, so that a second walk (a timed one) does the inference only."""
    calibrate = scales is None
    scales = {} if calibrate else dict(scales)
    scales[0] = float(in_scale)
    tensors = {0: x}
    logits = None
    for op, w in zip(ops, weights):
        src = tensors[op["src"]]
        s_in = scales[op["src"]]
        if op["op"] == "maxpool":
            tensors[op["dst"]] = oracle.maxpool(src, op["k"], op["stride"], op["pad"])
            scales[op["dst"]] = s_in
        elif op["op"] == "avgpool":
            if calibrate:
                scales[op["dst"]] = s_in
            y = oracle.avgpool(src, s_in, 1.0 / scales[op["dst"]])
            tensors[op["dst"]] = y.reshape(y.shape[0], 1, 1, y.shape[1])
        else:
            w_int, scale, bias = w
            N, K = w_int.shape
            if cache is not None and (id(w_int), full) in cache:
                wq = cache[(id(w_int), full)]
            else:
                ph, pl = oracle.decompose_pack(w_int, n_bits, l_bits)
                wq = oracle.weights_from_pages(ph, pl if full else None, N, K, n_bits, l_bits)
                if cache is not None:
                    cache[(id(w_int), full)] = wq
            part_l = 0 if full else l_bits
            if op["op"] == "fc":
                acc = oracle.gemm_acc(src.reshape(src.shape[0], -1), wq)
                logits = oracle.epilogue(acc, s_in, scale, part_l_bits=part_l, bias=bias)
                continue
            k = op["k"]
            acc = oracle.conv_acc(src, wq.reshape(N, k, k, op["cin"]), op["stride"], op["pad"])
            res, s_r = None, 0.0
            if op["residual"] is not None:
                res, s_r = tensors[op["residual"]], scales[op["residual"]]
            if calibrate:
                yf = oracle.epilogue(acc, s_in, scale, part_l_bits=part_l, bias=bias, residual=res, s_r=s_r,
                                     relu=op["relu"])
                scales[op["dst"]] = float(oracle.quantize(yf.reshape(1, -1), 8)[1][0])
            tensors[op["dst"]] = oracle.epilogue(acc, s_in, scale, part_l_bits=part_l, bias=bias, residual=res,
                                                 s_r=s_r, relu=op["relu"], out_int8=True,
                                                 inv_s_out=1.0 / scales[op["dst"]])
    return logits, tensors, scales
