"""Seeded random shapes through every inference entry point, against the CPU oracle: sizes, strides, paddings,
nestings, lower-part formats and epilogue options drawn together, so that combinations nobody wrote down by
hand (and whichever kernel the library picks for them) are covered.  Bar as everywhere: int32 accumulators
and int8 outputs bit exact, fp32 outputs identical."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, run_conv_both, run_gconv_both, run_gemm_both
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

NESTINGS = [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def epilogue_options(rng, out_shape, N):
    kw = dict(s_a=float(rng.uniform(0.005, 0.05)))
    if rng.random() < 0.6:
        kw["bias"] = inputs.small_floats(N, 0.3, seed=int(rng.integers(1 << 20)))
    if rng.random() < 0.4:
        kw["residual"] = inputs.uniform_activations(tuple(out_shape) + (N,), seed=int(rng.integers(1 << 20)))
        kw["s_r"] = float(rng.uniform(0.01, 0.08))
    kw["relu"] = bool(rng.random() < 0.5)
    if rng.random() < 0.5:
        kw["out_int8"] = True
        kw["inv_s_out"] = float(rng.uniform(2.0, 12.0))
    return kw


@pytest.mark.parametrize("seed", range(24))
def test_random_gemm(nq, seed):
    rng = np.random.default_rng(1000 + seed)
    n, l = NESTINGS[int(rng.integers(len(NESTINGS)))]
    M = int(rng.choice([1, 7, 16, 33, 64, 65, 100, 200, 333, 700]))
    N = int(rng.choice([1, 16, 31, 32, 48, 64, 96, 130, 256, 272, 400]))
    K = int(rng.choice([1, 16, 63, 64, 100, 128, 256, 320, 512, 768, 1000, 1024]))
    w_int, scale = tl.weights(N, K, 0.02, n, seed)
    case = Case(nq, w_int, scale, n, l)
    x = inputs.uniform_activations((M, K), seed=seed) >> (8 - n)
    kw = epilogue_options(rng, (M,), N)
    for full in (True, False):
        run_gemm_both(nq, case, x, full, **kw)


@pytest.mark.parametrize("seed", range(24))
def test_random_convolution(nq, seed):
    rng = np.random.default_rng(2000 + seed)
    n, l = NESTINGS[int(rng.integers(len(NESTINGS)))]
    KH = int(rng.choice([1, 1, 3, 3, 3, 5, 7]))
    stride = int(rng.choice([1, 1, 2]))
    pad = int(rng.choice([0, KH // 2]))
    Cin = int(rng.choice([1, 3, 4, 8, 16, 24, 32, 64, 64, 128, 256])) if KH <= 3 else int(rng.choice([1, 3, 4, 16]))
    Cout = int(rng.choice([8, 16, 32, 33, 64, 64, 96, 128, 160]))
    H = int(rng.integers(max(KH, 4), 21))
    W = int(rng.integers(max(KH, 4), 21))
    B = int(rng.integers(1, 4))
    K = KH * KH * Cin
    w_int, scale = tl.weights(Cout, K, inputs.he_sigma(K), n, seed)
    case = Case(nq, w_int, scale, n, l)
    x = inputs.uniform_activations((B, H, W, Cin), seed=seed) >> (8 - n)
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KH) // stride + 1
    kw = epilogue_options(rng, (B, Ho, Wo), Cout)
    for full in (True, False):
        run_conv_both(nq, case, x, (KH, KH, stride, pad), full, **kw)


@pytest.mark.parametrize("seed", range(16))
def test_random_grouped_convolution(nq, seed):
    rng = np.random.default_rng(3000 + seed)
    n, l = NESTINGS[int(rng.integers(len(NESTINGS)))]
    gs = int(rng.choice([1, 1, 2, 4]))
    KH = int(rng.choice([1, 3, 3, 5]))
    stride = int(rng.choice([1, 2]))
    pad = int(rng.choice([0, KH // 2]))
    C = 16 * int(rng.integers(1, 13))
    H = int(rng.integers(max(KH, 3), 24))
    W = int(rng.integers(max(KH, 3), 24))
    B = int(rng.integers(1, 4))
    K = KH * KH * gs
    w_int, scale = tl.weights(C, K, inputs.he_sigma(K), n, seed)
    case = Case(nq, w_int, scale, n, l)
    x = inputs.uniform_activations((B, H, W, C), seed=seed) >> (8 - n)
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KH) // stride + 1
    kw = epilogue_options(rng, (B, Ho, Wo), C)
    for full in (True, False):
        run_gconv_both(nq, case, x, (KH, KH, stride, pad), C // gs, full, **kw)
