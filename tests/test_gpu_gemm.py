"""GPU parity of the nested GEMM / convolution, full-bit and part-bit, against the CPU oracle.
Bar: int32 accumulators and int8 outputs bit exact; fp32 outputs within 1e-5 relative (and, since both
sides take the same fp32 steps in the same order, identical)."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, dev, host, run_conv_both, run_gemm_both
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

ALL_NL = [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def make_case(nq, N, K, n, l, sigma=0.02, seed=0):
    w_int, scale = tl.weights(N, K, sigma, n, seed)
    return Case(nq, w_int, scale, n, l)


def test_linear_config_small(nq):
    # M=64 x K=512 activations uniform int8, 512x512 weights N(0,0.02), INT8 nesting INT6, seed 0
    c = inputs.LINEAR_SMALL
    case = make_case(nq, c["N"], c["K"], c["n_bits"], c["l_bits"], c["sigma"], seed=0)
    assert case.pages_match()
    x = inputs.uniform_activations((c["M"], c["K"]), seed=0)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.0123)


@pytest.mark.parametrize("n,l", ALL_NL)
def test_every_nesting(nq, n, l):
    case = make_case(nq, 96, 192, n, l, seed=n * 10 + l)
    assert case.pages_match()
    x = inputs.uniform_activations((70, 192), seed=l)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.05)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 33, 70), (3, 64, 16), (300, 100, 192), (130, 257, 320),
                                   (257, 64, 1024), (64, 300, 64), (513, 40, 100), (200, 520, 48),
                                   # few rows: K split over the waves of a block (K steps 5, 17 and 36 + a tail)
                                   (7, 96, 320), (33, 130, 1088), (64, 48, 2320), (1, 32, 4096)])
def test_ragged_shapes(nq, M, N, K):
    # several tiles plus ragged tails in every dimension; K not a multiple of 16 takes the byte-gather path
    case = make_case(nq, N, K, 8, 2, seed=M + N + K)
    x = inputs.uniform_activations((M, K), seed=M)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.02)


def test_extreme_values(nq):
    # all activations -128 against all weights -128 / 127: the largest accumulators K * 2^14
    N, K, M = 64, 4608, 40
    for wv in (-128, 127):
        case = Case(nq, np.full((N, K), wv, np.int8), np.full(N, 0.001, np.float32), 8, 2)
        x = np.full((M, K), -128, np.int8)
        for full in (True, False):
            run_gemm_both(nq, case, x, full, s_a=0.01)


def test_epilogue_options(nq):
    N, K, M = 160, 256, 150
    case = make_case(nq, N, K, 8, 3, seed=5)
    x, s_a = tl.gaussian_activations((M, K), seed=5)
    bias = inputs.small_floats(N, 0.5, seed=1)
    res = inputs.uniform_activations((M, N), seed=9)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=float(s_a), bias=bias)
        run_gemm_both(nq, case, x, full, s_a=float(s_a), bias=bias, residual=res, s_r=0.031, relu=True)
        run_gemm_both(nq, case, x, full, s_a=float(s_a), bias=bias, residual=res, s_r=0.031, relu=True,
                      out_int8=True, inv_s_out=9.7)
        run_gemm_both(nq, case, x, full, s_a=float(s_a), out_int8=True, inv_s_out=30.0)


@pytest.mark.parametrize("geom", [
    # B, H, W, Cin, Cout, KH, KW, stride, pad
    (2, 9, 8, 16, 24, 3, 3, 1, 1), (2, 9, 8, 16, 24, 3, 3, 2, 1), (1, 12, 12, 32, 40, 1, 1, 1, 0),
    (2, 11, 10, 64, 64, 3, 3, 1, 1), (1, 14, 14, 64, 96, 1, 1, 2, 0), (2, 20, 20, 3, 64, 7, 7, 2, 3),
    (1, 7, 7, 48, 33, 3, 3, 1, 0), (3, 6, 6, 5, 7, 3, 3, 1, 1), (1, 5, 5, 128, 300, 3, 3, 1, 1),
    # implicit GEMM on the large-GEMM kernel: several row tiles, ragged rows, K not a multiple of 256 or 64
    (2, 14, 14, 256, 256, 3, 3, 1, 1), (3, 15, 13, 32, 96, 3, 3, 2, 1), (1, 9, 9, 16, 130, 5, 5, 1, 2),
    (2, 12, 12, 128, 272, 1, 1, 2, 0),
    # its pixel table holds one bit per filter row and column: the largest filter it takes (15 x 16), one row too
    # many (goes to another kernel), a 1 x 7 filter whose padding puts whole output rows outside the image
    (1, 10, 12, 16, 72, 15, 16, 1, 7), (1, 20, 9, 16, 40, 16, 3, 1, 1), (2, 8, 30, 32, 96, 1, 7, 2, 3),
    # strided 1x1 on the register-stationary kernel (fetches only the pixels it needs): odd sizes, stride 3,
    # several units per image, every K-step count of that kernel
    (2, 13, 11, 64, 64, 1, 1, 2, 0), (1, 57, 57, 256, 96, 1, 1, 2, 0), (2, 9, 10, 512, 40, 1, 1, 3, 0),
    (3, 28, 28, 128, 160, 1, 1, 2, 0),
    # few input channels: one matrix-core step per filter row, several units, ragged last unit
    (2, 64, 64, 3, 64, 7, 7, 2, 3), (1, 37, 36, 3, 48, 7, 7, 2, 3), (2, 12, 12, 4, 40, 3, 3, 1, 1),
    (1, 30, 28, 1, 32, 3, 3, 2, 0),
])
def test_conv_geometries(nq, geom):
    B, H, W, Cin, Cout, KH, KW, stride, pad = geom
    K = KH * KW * Cin
    case = make_case(nq, Cout, K, 8, 2, sigma=inputs.he_sigma(K), seed=sum(geom))
    x = inputs.uniform_activations((B, H, W, Cin), seed=Cin)
    for full in (True, False):
        run_conv_both(nq, case, x, (KH, KW, stride, pad), full, s_a=0.02)
    if Cout % 16 == 0:   # the 16-byte epilogue of int8 outputs, with a residual
        res = inputs.uniform_activations((B, (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1, Cout),
                                         seed=Cout)
        run_conv_both(nq, case, x, (KH, KW, stride, pad), True, s_a=0.02, residual=res, s_r=0.05, relu=True,
                      out_int8=True, inv_s_out=6.0)


def test_conv_resnet18_layer_reduced_batch(nq):
    # the benchmark's 3x3 convolution 56x56x64 -> 64 at batch 2 (full batch: sampled check in test_gpu_bench_size)
    c = inputs.CONV_RESNET18
    K = 9 * c["Cin"]
    case = make_case(nq, c["Cout"], K, 8, 2, sigma=inputs.he_sigma(K), seed=0)
    x = inputs.uniform_activations((2, c["H"], c["W"], c["Cin"]), seed=0)
    bias = inputs.small_floats(c["Cout"], 0.1, seed=2)
    for full in (True, False):
        run_conv_both(nq, case, x, (3, 3, 1, 1), full, s_a=0.02, bias=bias, relu=True)
        run_conv_both(nq, case, x, (3, 3, 1, 1), full, s_a=0.02, bias=bias, relu=True, out_int8=True, inv_s_out=3.0)


def test_bottleneck_block_chain(nq):
    # ResNet-101 stage-3 bottleneck at reduced batch: 1x1 1024->256, 3x3 256->256, 1x1 256->1024 with int8
    # requantisation between the layers and the residual added in the last epilogue; l = 2 and l = 4
    B = 4
    for l in (2, 4):
        x0, s0 = tl.relu_activations((B, 14, 14, 1024), seed=l)
        act, s_in = x0, float(s0)
        from oracle import nq_oracle as oracle
        for i, g in enumerate(inputs.BOTTLENECK_RESNET101):
            K = g["KH"] * g["KW"] * g["Cin"]
            case = make_case(nq, g["Cout"], K, 8, l, sigma=inputs.he_sigma(K), seed=100 * l + i)
            last = i == 2
            kw = dict(s_a=s_in, relu=True, out_int8=True, inv_s_out=8.0 if not last else 4.0)
            if last:
                kw.update(residual=x0, s_r=float(s0))
            for full in (True, False):
                run_conv_both(nq, case, act, (g["KH"], g["KW"], g["stride"], g["pad"]), full, **kw)
            # feed the next layer with the oracle's full-bit output so that errors cannot compound
            w4 = case.ow_full.reshape(g["Cout"], g["KH"], g["KW"], g["Cin"])
            acc = oracle.conv_acc(act, w4, g["stride"], g["pad"])
            okw = dict(s_a=s_in, s_w=case.scale, relu=True, out_int8=True, inv_s_out=kw["inv_s_out"])
            if last:
                okw.update(residual=x0, s_r=float(s0))
            act = oracle.epilogue(acc, **okw)
            s_in = 1.0 / kw["inv_s_out"]


def test_switching(nq):
    # downgrade: page the lower-bit part out -> only part-bit runs; upgrade: page it in -> full-bit again
    N, K, M = 128, 256, 90
    case = make_case(nq, N, K, 8, 2, seed=3)
    x = inputs.uniform_activations((M, K), seed=3)
    W = case.W
    run_gemm_both(nq, case, x, True, s_a=0.02)
    nq.nq_page_out_low(W.desc)
    assert W.desc.low_resident == 0
    W.low.fill_(0x5A)                                   # the device slot is no longer ours to read
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_full(dev(x), M, W.desc, nq.make_epilogue(0.02), y)
    assert e.value.status == nq.NQ_ERR_NOT_RESIDENT
    run_gemm_both(nq, case, x, False, s_a=0.02)          # part-bit never reads the page
    copy_stream = torch.cuda.Stream()
    nq.nq_page_in_low(W.desc, copy_stream)               # upgrade, on a second stream
    assert W.desc.low_resident == 1
    run_gemm_both(nq, case, x, True, s_a=0.02)           # the full-bit call waits for the copy itself
    assert case.pages_match()


def test_linearity_of_the_nesting(nq):
    # Eq. 4: acc_full = 2^l * acc_part + sum_k x * w_low, checked on GPU outputs alone
    N, K, M, l = 64, 128, 33, 3
    case = make_case(nq, N, K, 8, l, seed=8)
    x = inputs.uniform_activations((M, K), seed=8)
    accs = {}
    for full in (True, False):
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        epi = nq.make_epilogue(1.0, d_acc_dump=acc)
        (nq.nq_gemm_full if full else nq.nq_gemm_part)(dev(x), M, case.W.desc, epi, y)
        accs[full] = host(acc).astype(np.int64)
    low = (case.w_int.astype(np.int64) & ((1 << l) - 1))
    assert np.array_equal(accs[True], (accs[False] << l) + x.astype(np.int64) @ low.T)


def test_glue_kernels(nq, oracle):
    x = inputs.uniform_activations((3, 17, 15, 64), seed=4)
    y = torch.empty((3, 9, 8, 64), dtype=torch.int8, device="cuda")
    nq.nq_maxpool_i8(dev(x), 3, 17, 15, 64, 3, 2, 1, y)
    assert np.array_equal(host(y), oracle.maxpool(x, 3, 2, 1))
    # both max-pool kernels (16 channels per thread; one channel per thread for any C), windows that hang over
    # every border, all-minimum inputs
    for (B, H, W, C, k, s_, p_) in [(2, 9, 11, 48, 3, 2, 1), (2, 9, 11, 20, 3, 2, 1), (1, 5, 5, 16, 2, 2, 0),
                                    (3, 8, 6, 32, 3, 1, 1), (1, 4, 4, 16, 5, 3, 2), (2, 7, 7, 10, 2, 1, 0)]:
        for mode in ("uniform", "min"):
            x = inputs.uniform_activations((B, H, W, C), seed=B + C)
            if mode == "min":
                x[:] = -128
            Ho, Wo = (H + 2 * p_ - k) // s_ + 1, (W + 2 * p_ - k) // s_ + 1
            y = torch.full((B, Ho, Wo, C), 77, dtype=torch.int8, device="cuda")
            nq.nq_maxpool_i8(dev(x), B, H, W, C, k, s_, p_, y)
            assert np.array_equal(host(y), oracle.maxpool(x, k, s_, p_)), (B, H, W, C, k, s_, p_, mode)
    x = inputs.uniform_activations((5, 7, 7, 200), seed=6)
    y = torch.empty((5, 200), dtype=torch.int8, device="cuda")
    nq.nq_avgpool_i8(dev(x), 5, 49, 200, 0.05, 11.0, y)
    assert np.array_equal(host(y), oracle.avgpool(x, 0.05, 11.0))


@pytest.mark.parametrize("fmt", ["unsigned", "compensated"])
def test_large_kernel_every_tile_height(nq, fmt):
    # The large-GEMM kernel is built for 64, 96, 128 and 160 rows per block and picks one from the shape.
    # run_*_both force each height in turn (kernel choices "4/tm2" .. "4/tm5"): a GEMM and a 3x3 implicit
    # GEMM with ragged row tiles, full-bit and part-bit, fp32, int8 and int8 + residual outputs.
    from oracle import nq_oracle as oracle
    n, l = 8, 2
    low_format = nq.NQ_LOW_SIGNED_L1 if fmt == "compensated" else nq.NQ_LOW_UNSIGNED_L

    def case_for(N, K, sigma, seed):
        w_int, scale = tl.weights(N, K, sigma, n, seed)
        c = Case(nq, w_int, scale, n, l)
        if fmt == "compensated":
            # same weights in the compensated format: w_high rounded to nearest, signed (l+1)-bit lower part
            c.cfg = nq.make_cfg(n, l, low_format)
            c.W = nq.NestedWeight.from_int8(dev(w_int), dev(scale), c.cfg)
            hi, _ = oracle.decompose(w_int, n, l, "rtn")
            c.ow_part = hi.astype(np.int16)
            c.ow_full = w_int.astype(np.int16)
        return c

    M, N, K = 700, 320, 512
    case = case_for(N, K, 0.02, seed=77)
    x = inputs.uniform_activations((M, K), seed=77)
    res = inputs.uniform_activations((M, N), seed=78)
    bias = inputs.small_floats(N, 0.3, seed=79)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.02, bias=bias)
        run_gemm_both(nq, case, x, full, s_a=0.02, bias=bias, relu=True, out_int8=True, inv_s_out=7.0)
        run_gemm_both(nq, case, x, full, s_a=0.02, bias=bias, residual=res, s_r=0.04, relu=True, out_int8=True,
                      inv_s_out=7.0)
    B, H, W, Cin, Cout = 3, 15, 14, 64, 160
    K = 9 * Cin
    case = case_for(Cout, K, inputs.he_sigma(K), seed=80)
    x = inputs.uniform_activations((B, H, W, Cin), seed=80)
    for stride in (1, 2):
        Ho, Wo = (H + 2 - 3) // stride + 1, (W + 2 - 3) // stride + 1
        res = inputs.uniform_activations((B, Ho, Wo, Cout), seed=81)
        bias = inputs.small_floats(Cout, 0.3, seed=82)
        for full in (True, False):
            run_conv_both(nq, case, x, (3, 3, stride, 1), full, s_a=0.02, bias=bias)
            run_conv_both(nq, case, x, (3, 3, stride, 1), full, s_a=0.02, bias=bias, relu=True, out_int8=True,
                          inv_s_out=5.0)
            run_conv_both(nq, case, x, (3, 3, stride, 1), full, s_a=0.02, bias=bias, residual=res, s_r=0.04,
                          relu=True, out_int8=True, inv_s_out=5.0)


def test_failed_call_enqueues_nothing_and_keeps_the_timing_events(nq):
    # a call that fails its checks must leave the one-shot profiling events for the next launch
    N, K, M = 64, 256, 40
    case = make_case(nq, N, K, 8, 2, seed=12)
    x = dev(inputs.uniform_activations((M, K), seed=12))
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    ev0, ev1 = nq.nq_event_create(), nq.nq_event_create()
    nq.nq_profile_next_launch(ev0, ev1)
    short = nq.NestedWeight(N, K, case.cfg)
    short.desc.high_bytes = 16
    with pytest.raises(nq.NQError):
        nq.nq_gemm_part(x, M, short.desc, nq.make_epilogue(0.02), y)
    nq.nq_gemm_part(x, M, case.W.desc, nq.make_epilogue(0.02), y)
    torch.cuda.synchronize()
    assert nq.nq_event_elapsed_ms(ev0, ev1) > 0.0
    nq.nq_event_destroy(ev0)
    nq.nq_event_destroy(ev1)
