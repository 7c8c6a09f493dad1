"""GPU parity of the GEMM that reads the paper's own pages (Sec. 3.3.4: 64 // k fields per unsigned 64-bit word)
directly, full-bit (Eq. 4) and part-bit (Eq. 8), for every nesting and both lower-bit formats.  The pages the
kernel reads are the ORACLE's (packed on the CPU), so the test is that of a model file written as the paper
describes.  Bar: int32 accumulators bit exact, fp32 outputs identical, int8 outputs identical."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import check_outputs, dev, host
from oracle import nq_oracle as oracle
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

ALL_NL = [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def oracle_side(w_int, n, l, signed):
    """(word page of w_high, word page of w_low, full-bit weights, higher-bit part) from the CPU oracle."""
    h = n - l
    if signed:
        hi, res = oracle.decompose(w_int, n, l, "rtn")
        lo = oracle.low_encode(res, l, oracle.LOW_SIGNED_L1)
        lf = l + 1
    else:
        hi, res = oracle.decompose(w_int, n, l, "bitshift")
        lo = oracle.low_encode(res, l, oracle.LOW_UNSIGNED_L)
        lf = l
    ph = oracle.pack_paper(hi, h)
    pl = oracle.pack_paper(lo, lf)
    N, K = w_int.shape
    # what the pages hold, read back by the oracle's own unpacker
    hi_back = oracle.unpack_paper(ph, N, K, h, True)
    lo_back = oracle.unpack_paper(pl, N, K, lf, signed)
    full = oracle.compose(hi_back, lo_back, l)
    assert np.array_equal(full, w_int.astype(np.int16))
    return ph, pl, full, hi_back.astype(np.int16)


def weight_from_pages(nq, ph, pl, scale, N, K, n, l, signed):
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1 if signed else nq.NQ_LOW_UNSIGNED_L, nq.NQ_LAYOUT_PAPER_U64)
    W = nq.NestedWeight(N, K, cfg)
    assert ph.nbytes == nq.nq_packed_bytes(N, K, n - l, nq.NQ_LAYOUT_PAPER_U64)
    assert pl.nbytes == nq.nq_packed_bytes(N, K, l + (1 if signed else 0), nq.NQ_LAYOUT_PAPER_U64)
    W.fill_from_pages(ph.view(np.uint8).ravel(), pl.view(np.uint8).ravel(), scale)
    return W


def run_both(nq, W, x, w_ref, scale, l, full, out_int8=False, bias=None, residual=None, s_r=0.0, relu=False,
             s_a=0.043, inv_s_out=1.0):
    M, N = x.shape[0], w_ref.shape[0]
    acc_ref = oracle.gemm_acc(x, w_ref)
    y_ref = oracle.epilogue(acc_ref, s_a=s_a, s_w=scale, part_l_bits=0 if full else l, bias=bias, residual=residual,
                            s_r=s_r, relu=relu, out_int8=out_int8, inv_s_out=inv_s_out)
    fn = nq.nq_gemm_full if full else nq.nq_gemm_part
    dx = dev(x)
    for dump in (True, False):
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda") if dump else None
        d_bias = dev(bias) if bias is not None else None
        d_res = dev(residual) if residual is not None else None
        epi = nq.make_epilogue(s_a, d_bias, d_res, s_r, relu, out_int8, inv_s_out, acc)
        y = torch.full((M, N), 77, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
        fn(dx, M, W.desc, epi, y)
        torch.cuda.synchronize()
        check_outputs(host(y), host(acc) if dump else None, y_ref, acc_ref, out_int8)


# (M, N, K): ragged in every dimension; K below one word, K a whole number of words, several row tiles
SHAPES = [(1, 1, 1), (16, 70, 333), (45, 33, 64), (3, 32, 7), (33, 96, 1000), (16, 40, 1024)]


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("n,l", ALL_NL)
def test_words_gemm_all_nestings(nq, n, l, signed):
    for si, (M, N, K) in enumerate(SHAPES):
        seed = 1000 * n + 100 * l + 10 * si + int(signed)
        w_int, scale = tl.weights(N, K, 0.05, n, seed=seed)
        x = inputs.uniform_activations((M, K), seed=seed + 1)
        ph, pl, w_full, w_high = oracle_side(w_int, n, l, signed)
        W = weight_from_pages(nq, ph, pl, scale, N, K, n, l, signed)
        run_both(nq, W, x, w_full, scale, l, True)
        run_both(nq, W, x, w_high, scale, l, False)


@pytest.mark.parametrize("n,l,signed", [(8, 3, False), (8, 3, True), (8, 4, False), (6, 2, True), (8, 1, False)])
def test_words_gemm_epilogues(nq, n, l, signed):
    M, N, K = 37, 80, 520
    rng = np.random.default_rng(7 * n + l)
    w_int, scale = tl.weights(N, K, 0.05, n, seed=5 + l)
    x = inputs.uniform_activations((M, K), seed=6 + l)
    bias = rng.normal(0, 0.5, N).astype(np.float32)
    residual = rng.integers(-128, 128, (M, N)).astype(np.int8)
    ph, pl, w_full, w_high = oracle_side(w_int, n, l, signed)
    W = weight_from_pages(nq, ph, pl, scale, N, K, n, l, signed)
    for full, w_ref in ((True, w_full), (False, w_high)):
        run_both(nq, W, x, w_ref, scale, l, full, bias=bias, relu=True)
        run_both(nq, W, x, w_ref, scale, l, full, bias=bias, residual=residual, s_r=0.02, relu=True, out_int8=True,
                 inv_s_out=1.0 / 0.05)
        run_both(nq, W, x, w_ref, scale, l, full, out_int8=True, inv_s_out=1.0 / 0.11)


def test_extreme_values_and_spare_bits(nq):
    """All-minimum weights against all-minimum activations (the largest accumulator of a row), and words whose
    spare top bits are set: the format leaves them undefined, the kernel must not read them as fields."""
    for n, l in ((8, 3), (8, 1), (6, 3), (8, 5)):
        h = n - l
        M, N, K = 5, 34, 2000
        w_int = np.full((N, K), -(1 << (n - 1)), dtype=np.int8)
        w_int[1::2] = (1 << (n - 1)) - 1
        scale = np.full(N, 0.01, dtype=np.float32)
        x = np.full((M, K), -128, dtype=np.int8)
        x[1::2] = 127
        ph, pl, w_full, w_high = oracle_side(w_int, n, l, False)
        for k, page in ((h, ph), (l, pl)):
            spare = 64 - (64 // k) * k
            if spare:
                page |= np.uint64(((1 << spare) - 1) << (64 - spare))
        W = weight_from_pages(nq, ph, pl, scale, N, K, n, l, False)
        run_both(nq, W, x, w_full, scale, l, True)
        run_both(nq, W, x, w_high, scale, l, False)


def test_gpu_packed_word_pages_feed_the_gemm(nq):
    """Pages packed by nq_decompose_pack in the word layout equal the oracle's and run through the same GEMM."""
    n, l = 8, 3
    M, N, K = 16, 64, 700
    w_int, scale = tl.weights(N, K, 0.05, n, seed=3)
    x = inputs.uniform_activations((M, K), seed=4)
    ph, pl, w_full, w_high = oracle_side(w_int, n, l, False)
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_UNSIGNED_L, nq.NQ_LAYOUT_PAPER_U64)
    W = nq.NestedWeight.from_int8(dev(w_int), dev(scale), cfg)
    assert np.array_equal(host(W.high)[:ph.nbytes], ph.view(np.uint8).ravel())
    assert np.array_equal(host(W.low)[:pl.nbytes], pl.view(np.uint8).ravel())
    run_both(nq, W, x, w_full, scale, l, True)
    run_both(nq, W, x, w_high, scale, l, False)


def test_word_pages_argument_checks(nq):
    n, l = 8, 2
    N, K, M = 32, 128, 4
    w_int, scale = tl.weights(N, K, 0.05, n, seed=1)
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_UNSIGNED_L, nq.NQ_LAYOUT_PAPER_U64)
    W = nq.NestedWeight.from_int8(dev(w_int), dev(scale), cfg)
    epi = nq.make_epilogue(1.0)
    y = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    xb = torch.zeros(M * K + 4, dtype=torch.int8, device="cuda")
    # activations that do not start on a dword
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_full(xb[1:1 + M * K], M, W.desc, epi, y)
    assert e.value.status == nq.NQ_ERR_ALIGN
    # a convolution whose input does not start on a dword
    cs = nq.nq_conv_shape(1, 4, 4, 8, N, 4, 4, 1, 0)
    with pytest.raises(nq.NQError) as e:
        nq.nq_conv_full(xb[1:1 + 128], cs, W.desc, epi, y)
    assert e.value.status == nq.NQ_ERR_ALIGN
    # grouped convolutions read the dense pages only
    Wg = nq.NestedWeight.from_int8(dev(w_int[:, :18].copy()), dev(scale), cfg)
    with pytest.raises(nq.NQError) as e:
        nq.nq_gconv_full(xb, nq.nq_conv_shape(1, 4, 4, 32, 32, 3, 3, 1, 1), 16, Wg.desc, epi,
                         torch.zeros((4, 4, 32), dtype=torch.float32, device="cuda"))
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    # nothing to do
    nq.nq_gemm_full(xb, 0, W.desc, epi, y)
    torch.cuda.synchronize()


@pytest.mark.parametrize("l,signed", [(3, False), (2, True)])
def test_words_gemm_at_the_measured_size(nq, l, signed):
    """16 x 8192 -> 8192, the size the word-page tables are measured at; every output compared."""
    n, M, N, K = 8, 16, 8192, 8192
    w_int, scale = tl.weights(N, K, 0.02, n, seed=40 + l)
    x = inputs.uniform_activations((M, K), seed=41 + l)
    ph, pl, w_full, w_high = oracle_side(w_int, n, l, signed)
    W = weight_from_pages(nq, ph, pl, scale, N, K, n, l, signed)
    run_both(nq, W, x, w_full, scale, l, True, s_a=0.02)
    run_both(nq, W, x, w_high, scale, l, False, s_a=0.02)


# Convolutions straight from the word pages: (B, H, W, Cin, Cout, KH, KW, stride, pad).  Channel counts that are and
# are not multiples of four (dword and byte gathers), the 7x7 stem over 3 channels, strides, padding wider than the
# filter needs, 1x1 with a stride (gathered) and without (the plain GEMM over the pixels), K of one word and less,
# ragged pixel tiles and channel tiles.
CONV_GEOMS = [
    (2, 9, 8, 16, 40, 3, 3, 1, 1),
    (1, 12, 11, 3, 24, 7, 7, 2, 3),
    (3, 7, 7, 20, 33, 3, 3, 2, 1),
    (2, 6, 5, 6, 16, 1, 1, 2, 0),
    (2, 6, 5, 6, 16, 1, 1, 1, 0),
    (1, 5, 5, 5, 8, 5, 5, 1, 2),
    (2, 10, 9, 64, 70, 3, 3, 1, 1),
    (1, 4, 4, 1, 3, 2, 2, 1, 1),
    (4, 8, 8, 32, 64, 1, 3, 1, 1),
]


def run_conv_both(nq, W, x, geom, w_ref, scale, l, full, **opt):
    B, H, Wd, Cin, Cout, KH, KW, stride, pad = geom
    s_a = opt.get("s_a", 0.031)
    acc_ref = oracle.conv_acc(x, w_ref.reshape(Cout, KH, KW, Cin), stride, pad)
    Ho, Wo = acc_ref.shape[1:3]
    y_ref = oracle.epilogue(acc_ref, s_a=s_a, s_w=scale, part_l_bits=0 if full else l, bias=opt.get("bias"),
                            residual=opt.get("residual"), s_r=opt.get("s_r", 0.0), relu=opt.get("relu", False),
                            out_int8=opt.get("out_int8", False), inv_s_out=opt.get("inv_s_out", 1.0))
    fn = nq.nq_conv_full if full else nq.nq_conv_part
    cs = nq.nq_conv_shape(B, H, Wd, Cin, Cout, KH, KW, stride, pad)
    dx = dev(x)
    for dump in (True, False):
        acc = torch.empty((B, Ho, Wo, Cout), dtype=torch.int32, device="cuda") if dump else None
        d_bias = dev(opt["bias"]) if opt.get("bias") is not None else None
        d_res = dev(opt["residual"]) if opt.get("residual") is not None else None
        epi = nq.make_epilogue(s_a, d_bias, d_res, opt.get("s_r", 0.0), opt.get("relu", False), opt.get("out_int8", False),
                               opt.get("inv_s_out", 1.0), acc)
        y = torch.full((B, Ho, Wo, Cout), 77, dtype=torch.int8 if opt.get("out_int8") else torch.float32, device="cuda")
        fn(dx, cs, W.desc, epi, y)
        torch.cuda.synchronize()
        check_outputs(host(y), host(acc) if dump else None, y_ref, acc_ref, opt.get("out_int8", False))


@pytest.mark.parametrize("geom", CONV_GEOMS, ids=lambda g: "x".join(str(v) for v in g))
def test_words_conv_geometries(nq, geom):
    B, H, Wd, Cin, Cout, KH, KW, stride, pad = geom
    K = KH * KW * Cin
    for n, l, signed in ((8, 2, False), (8, 3, True), (6, 2, False), (8, 5, False)):
        seed = sum(geom) + 10 * n + l
        w_int, scale = tl.weights(Cout, K, inputs.he_sigma(K), n, seed=seed)
        x = inputs.uniform_activations((B, H, Wd, Cin), seed=seed + 1)
        ph, pl, w_full, w_high = oracle_side(w_int, n, l, signed)
        W = weight_from_pages(nq, ph, pl, scale, Cout, K, n, l, signed)
        run_conv_both(nq, W, x, geom, w_full, scale, l, True)
        run_conv_both(nq, W, x, geom, w_high, scale, l, False)


@pytest.mark.parametrize("n,l", ALL_NL)
def test_words_conv_all_nestings_with_epilogues(nq, n, l):
    geom = (2, 9, 7, 12, 48, 3, 3, 1, 1)
    B, H, Wd, Cin, Cout, KH, KW, stride, pad = geom
    K = KH * KW * Cin
    rng = np.random.default_rng(31 * n + l)
    w_int, scale = tl.weights(Cout, K, inputs.he_sigma(K), n, seed=70 + n + l)
    x = inputs.uniform_activations((B, H, Wd, Cin), seed=71 + n + l)
    bias = rng.normal(0, 0.5, Cout).astype(np.float32)
    residual = rng.integers(-128, 128, (B, H, Wd, Cout)).astype(np.int8)
    for signed in (False, True):
        ph, pl, w_full, w_high = oracle_side(w_int, n, l, signed)
        W = weight_from_pages(nq, ph, pl, scale, Cout, K, n, l, signed)
        for full, w_ref in ((True, w_full), (False, w_high)):
            run_conv_both(nq, W, x, geom, w_ref, scale, l, full, bias=bias, relu=True)
            run_conv_both(nq, W, x, geom, w_ref, scale, l, full, bias=bias, residual=residual, s_r=0.02, relu=True,
                          out_int8=True, inv_s_out=1.0 / 0.07)


def test_words_conv_resnet_layer_shapes(nq):
    """A 3x3 bottleneck convolution (14 x 14 x 256 -> 256) and the 7x7 stem at a reduced batch: several row tiles, long rows."""
    n, l = 8, 2
    for geom in ((2, 14, 14, 256, 256, 3, 3, 1, 1), (1, 56, 56, 3, 64, 7, 7, 2, 3)):
        B, H, Wd, Cin, Cout, KH, KW, stride, pad = geom
        K = KH * KW * Cin
        w_int, scale = tl.weights(Cout, K, inputs.he_sigma(K), n, seed=90 + Cin)
        x = inputs.uniform_activations((B, H, Wd, Cin), seed=91 + Cin)
        ph, pl, w_full, w_high = oracle_side(w_int, n, l, False)
        W = weight_from_pages(nq, ph, pl, scale, Cout, K, n, l, False)
        run_conv_both(nq, W, x, geom, w_full, scale, l, True, relu=True, out_int8=True, inv_s_out=1.0 / 0.2)
        run_conv_both(nq, W, x, geom, w_high, scale, l, False, relu=True, out_int8=True, inv_s_out=1.0 / 0.2)
