"""GPU parity of the stationary-weights GEMM (short reductions: K = 64, 128, 256; 1x1 convolutions at any
stride) against the CPU oracle: every nesting, every block shape (64, 128 or 256 columns per block), tiles
that straddle images and the end of M, many tiles per block, strided pixel gathers, all epilogues, the
compensated format.  Bar as everywhere: int32 accumulators and int8 codes bit exact, fp32 identical."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, dev, run_conv_both, run_gemm_both
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

ALL_NL = [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def make_case(nq, N, K, n, l, seed, compensated=False):
    from oracle import nq_oracle as oracle
    w_int, scale = tl.weights(N, K, inputs.he_sigma(K), n, seed)
    c = Case(nq, w_int, scale, n, l)
    if compensated:
        c.cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
        c.W = nq.NestedWeight.from_int8(dev(w_int), dev(scale), c.cfg)
        c.ow_part = oracle.decompose(w_int, n, l, "rtn")[0].astype(np.int16)
        c.ow_full = w_int.astype(np.int16)
    return c


@pytest.mark.parametrize("n,l", ALL_NL)
@pytest.mark.parametrize("K", [64, 128, 256])
def test_every_nesting_and_reduction_length(nq, n, l, K):
    N, M = 96, 333                      # 128-column blocks, five row tiles with a ragged last one
    case = make_case(nq, N, K, n, l, seed=n * 100 + l * 10 + K)
    x = inputs.uniform_activations((M, K), seed=K + l) >> (8 - n)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.03)


@pytest.mark.parametrize("M,N,K", [(65, 64, 64), (1000, 48, 256), (257, 128, 128), (129, 130, 256), (700, 272, 64),
                                   (4097, 320, 128), (70000, 64, 64), (40000, 512, 256), (90, 1040, 256)])
def test_block_shapes_and_many_tiles(nq, M, N, K):
    # 64 / 128 / 256 columns per block, column tiles past N, one to many row tiles per block, M = 1 mod tile
    case = make_case(nq, N, K, 8, 2, seed=M % 97 + N + K)
    x = inputs.uniform_activations((M, K), seed=N)
    bias = inputs.small_floats(N, 0.2, seed=K)
    res = inputs.uniform_activations((M, N), seed=K + 1)
    big = M * N > 4_000_000
    for full in (True, False):
        if not big:
            run_gemm_both(nq, case, x, full, s_a=0.02, bias=bias)
        if N % 16 == 0:
            run_gemm_both(nq, case, x, full, s_a=0.02, bias=bias, residual=res, s_r=0.05, relu=True, out_int8=True,
                          inv_s_out=4.0)
        if not big:
            run_gemm_both(nq, case, x, full, s_a=0.02, out_int8=True, inv_s_out=4.0)


@pytest.mark.parametrize("geom", [
    # B, H, W, Cin, Cout, stride: images smaller than a row tile, odd sizes, strides 2 and 3, one pixel out
    (5, 7, 7, 256, 96, 1), (9, 7, 7, 64, 64, 2), (3, 13, 11, 128, 160, 2), (2, 57, 55, 256, 272, 2),
    (4, 9, 10, 64, 320, 3), (70, 2, 2, 128, 64, 2), (2, 56, 56, 64, 256, 1), (130, 1, 1, 256, 144, 1),
])
def test_pixel_rows_of_1x1_convolutions(nq, geom):
    B, H, W, Cin, Cout, stride = geom
    case = make_case(nq, Cout, Cin, 8, 3, seed=sum(geom))
    x = inputs.uniform_activations((B, H, W, Cin), seed=Cin + H)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    res = inputs.uniform_activations((B, Ho, Wo, Cout), seed=Cout)
    bias = inputs.small_floats(Cout, 0.2, seed=3)
    for full in (True, False):
        run_conv_both(nq, case, x, (1, 1, stride, 0), full, s_a=0.02, bias=bias, relu=True)
        run_conv_both(nq, case, x, (1, 1, stride, 0), full, s_a=0.02, bias=bias, residual=res, s_r=0.04, relu=True,
                      out_int8=True, inv_s_out=5.0)


@pytest.mark.parametrize("n,l", [(8, 2), (8, 4), (6, 3)])
def test_compensated_format(nq, n, l):
    M, N, K = 300, 160, 256
    case = make_case(nq, N, K, n, l, seed=l, compensated=True)
    x = inputs.uniform_activations((M, K), seed=l) >> (8 - n)
    res = inputs.uniform_activations((M, N), seed=5)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, s_a=0.02)
        run_gemm_both(nq, case, x, full, s_a=0.02, residual=res, s_r=0.04, relu=True, out_int8=True, inv_s_out=5.0)


def test_consecutive_row_runs(nq):
    # the other way of splitting the rows over the blocks (NQ_TUNE_STAT_ROWS = 1): runs that end inside a tile
    try:
        nq.nq_set_tuning(nq.NQ_TUNE_STAT_ROWS, 1)
        for M, N, K in ((4097, 320, 128), (70000, 64, 64), (333, 96, 256)):
            case = make_case(nq, N, K, 8, 2, seed=M % 89)
            x = inputs.uniform_activations((M, K), seed=N)
            res = inputs.uniform_activations((M, N), seed=K)
            for full in (True, False):
                run_gemm_both(nq, case, x, full, s_a=0.02, residual=res, s_r=0.05, relu=True, out_int8=True,
                              inv_s_out=4.0)
    finally:
        nq.nq_set_tuning(nq.NQ_TUNE_STAT_ROWS, 0)


def test_library_picks_this_kernel(nq):
    # the shapes this kernel is meant for are routed to it without any override
    case = make_case(nq, 256, 64, 8, 2, seed=1)
    x = dev(inputs.uniform_activations((500, 64), seed=1))
    y = torch.empty((500, 256), dtype=torch.float32, device="cuda")
    nq.nq_gemm_part(x, 500, case.W.desc, nq.make_epilogue(0.02), y)
    assert nq.nq_profile_last_kernel()[0] == 9
