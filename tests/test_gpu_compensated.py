"""GPU parity of the paper's compensated format (Sec. 3.3.3): w_high from a rounding other than the shift,
signed w_low of l + 1 bits, recomposition by shift-add (Eq. 4).  Bar: parts, pages and int32 accumulators bit
exact against the CPU oracle; fp32 outputs identical."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import check_outputs, dev, each_kernel, host
from oracle import nq_oracle as oracle
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu

ALL_NL = [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def all_values(n_bits, N=40, K=100, seed=0):
    """Every INT-n value many times, in a ragged tensor (tiles plus tails in both dimensions)."""
    rng = np.random.default_rng(seed)
    lo, hi = -(1 << (n_bits - 1)), (1 << (n_bits - 1)) - 1
    w = rng.integers(lo, hi + 1, size=(N, K)).astype(np.int8)
    w.ravel()[:hi - lo + 1] = np.arange(lo, hi + 1, dtype=np.int8)
    return w


@pytest.mark.parametrize("n,l", ALL_NL)
def test_decompose_and_pages(nq, n, l):
    h = n - l
    w = all_values(n, seed=n * 10 + l)
    N, K = w.shape
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
    hi_ref, res = oracle.decompose(w, n, l, "rtn")
    lo_ref = oracle.low_encode(res, l, oracle.LOW_SIGNED_L1)
    assert np.array_equal(oracle.compose(hi_ref, lo_ref, l), w.astype(np.int16))       # Eq. 4, exact
    assert lo_ref.min() >= -(1 << l) + 1 and lo_ref.max() <= (1 << l) - 1
    # unpacked parts
    d_hi = torch.empty((N, K), dtype=torch.int8, device="cuda")
    d_lo = torch.empty((N, K), dtype=torch.int8, device="cuda")
    nq.nq_decompose(dev(w), N, K, cfg, d_hi, d_lo)
    torch.cuda.synchronize()
    assert np.array_equal(host(d_hi), hi_ref) and np.array_equal(host(d_lo), lo_ref)
    # dense pages, from w_int (fused) and from the parts, and back
    ph_ref = oracle.pack_dense(hi_ref, h, oracle.KIND_CARRIER)
    pl_ref = oracle.pack_dense(lo_ref, l + 1, oracle.KIND_BITSTRING)
    assert pl_ref.size == nq.nq_packed_bytes(N, K, l + 1)
    for src in ("w_int", "parts"):
        ph = torch.zeros(ph_ref.size, dtype=torch.uint8, device="cuda")
        pl = torch.zeros(pl_ref.size, dtype=torch.uint8, device="cuda")
        if src == "w_int":
            nq.nq_decompose_pack(dev(w), N, K, cfg, ph, pl)
        else:
            nq.nq_pack(dev(hi_ref), dev(lo_ref), N, K, cfg, ph, pl)
        torch.cuda.synchronize()
        assert np.array_equal(host(ph), ph_ref), f"higher-bit page differs ({src})"
        assert np.array_equal(host(pl), pl_ref), f"lower-bit page differs ({src})"
    u_hi, u_lo = torch.empty_like(d_hi), torch.empty_like(d_lo)
    nq.nq_unpack(ph, pl, N, K, cfg, u_hi, u_lo)
    torch.cuda.synchronize()
    assert np.array_equal(host(u_hi), hi_ref) and np.array_equal(host(u_lo), lo_ref)
    # the paper's word pages: 64 // k fields per word, k = h and l + 1
    cw = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1, nq.NQ_LAYOUT_PAPER_U64)
    wh_ref = oracle.pack_paper(hi_ref, h).view(np.uint8).ravel()
    wl_ref = oracle.pack_paper(lo_ref, l + 1).view(np.uint8).ravel()
    wh = torch.zeros(wh_ref.size, dtype=torch.uint8, device="cuda")
    wl = torch.zeros(wl_ref.size, dtype=torch.uint8, device="cuda")
    nq.nq_decompose_pack(dev(w), N, K, cw, wh, wl)
    torch.cuda.synchronize()
    assert np.array_equal(host(wh), wh_ref) and np.array_equal(host(wl), wl_ref)
    nq.nq_unpack(wh, wl, N, K, cw, u_hi, u_lo)
    torch.cuda.synchronize()
    assert np.array_equal(host(u_hi), hi_ref) and np.array_equal(host(u_lo), lo_ref)


def run_both_modes(nq, W, x, hi, w_full, scale, l, conv=None, out_int8=False):
    """Full-bit (= the original INT-n weights) and part-bit (= the supplied w_high) against the oracle."""
    inv_s_out = 9.0 if out_int8 else 1.0
    for full in (True, False):
        w_ref = (w_full if full else hi).astype(np.int16)
        if conv is None:
            acc_ref = oracle.gemm_acc(x, w_ref)
            shape = (x.shape[0],)
        else:
            KH, KW, stride, pad = conv
            acc_ref = oracle.conv_acc(x, w_ref.reshape(W.N, KH, KW, x.shape[3]), stride, pad)
            shape = acc_ref.shape[:3]
        y_ref = oracle.epilogue(acc_ref, 0.02, scale, part_l_bits=0 if full else l, relu=True,
                                out_int8=out_int8, inv_s_out=inv_s_out)
        for dump in (True, False):
            for kernel in each_kernel():
                acc = torch.empty(shape + (W.N,), dtype=torch.int32, device="cuda") if dump else None
                y = torch.full(shape + (W.N,), 77, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
                epi = nq.make_epilogue(0.02, relu=True, out_int8=out_int8, inv_out_scale=inv_s_out, d_acc_dump=acc)
                if conv is None:
                    (nq.nq_gemm_full if full else nq.nq_gemm_part)(dev(x), x.shape[0], W.desc, epi, y)
                else:
                    cs = nq.nq_conv_shape(x.shape[0], x.shape[1], x.shape[2], x.shape[3], W.N, KH, KW, stride, pad)
                    (nq.nq_conv_full if full else nq.nq_conv_part)(dev(x), cs, W.desc, epi, y)
                torch.cuda.synchronize()
                try:
                    check_outputs(host(y), host(acc) if dump else None, y_ref, acc_ref, out_int8)
                except AssertionError as e:
                    raise AssertionError(f"{e} (full={full}, kernel choice '{kernel}', dump {dump})") from None


@pytest.mark.parametrize("n,l", ALL_NL)
def test_gemm_with_round_to_nearest_high(nq, n, l):
    N, K, M = 96, 320, 70
    w, scale = tl.weights(N, K, 0.02, n, seed=n + l)
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
    W = nq.NestedWeight.from_int8(dev(w), dev(scale), cfg)
    hi, _ = oracle.decompose(w, n, l, "rtn")
    x = inputs.uniform_activations((M, K), seed=l) >> (8 - n)
    run_both_modes(nq, W, x, hi, w, scale, l)


# shapes that reach the specialised kernels: large GEMM (K a multiple of 256, several row tiles), few
# rows (one and two 32-row tiles), each with fp32 and int8 outputs
@pytest.mark.parametrize("n,l", [(8, 4), (8, 2), (8, 1), (6, 3), (6, 1)])
@pytest.mark.parametrize("M,N,K", [(200, 160, 512), (330, 96, 768), (40, 96, 512), (16, 128, 1024)])
def test_gemm_shapes_of_the_specialised_kernels(nq, n, l, M, N, K):
    w, scale = tl.weights(N, K, 0.02, n, seed=M + n + l)
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
    W = nq.NestedWeight.from_int8(dev(w), dev(scale), cfg)
    hi, _ = oracle.decompose(w, n, l, "rtn")
    x = inputs.uniform_activations((M, K), seed=K + l)
    for out_int8 in (False, True):
        run_both_modes(nq, W, x, hi, w, scale, l, out_int8=out_int8)


# convolutions that reach the register-stationary kernel (1x1 and 3x3 over 64 channels, 1x1 over 256),
# the large implicit GEMM (3x3 over 128 channels) and the few-channel kernel (7x7 and 3x3 over 3 channels)
@pytest.mark.parametrize("n,l", [(8, 4), (8, 2), (6, 2)])
@pytest.mark.parametrize("Cin,Cout,KH,stride,pad,HW", [(64, 64, 1, 1, 0, 20), (64, 96, 3, 1, 1, 14),
                                                      (256, 64, 1, 1, 0, 12), (128, 128, 3, 1, 1, 12),
                                                      (512, 128, 1, 1, 0, 9), (3, 64, 7, 2, 3, 40),
                                                      (3, 32, 3, 2, 1, 33)])
def test_convolution_shapes_of_the_specialised_kernels(nq, n, l, Cin, Cout, KH, stride, pad, HW):
    B = 2
    K = KH * KH * Cin
    w, scale = tl.weights(Cout, K, inputs.he_sigma(K), n, seed=Cin + KH + n + l)
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
    W = nq.NestedWeight.from_int8(dev(w), dev(scale), cfg)
    hi, _ = oracle.decompose(w, n, l, "rtn")
    x = inputs.uniform_activations((B, HW, HW - 1, Cin), seed=HW + l)
    for out_int8 in (False, True):
        run_both_modes(nq, W, x, hi, w, scale, l, conv=(KH, KH, stride, pad), out_int8=out_int8)


@pytest.mark.parametrize("rounding", ["up", "down", "rtn"])
def test_externally_supplied_high(nq, rounding):
    # w_high by the caller's own rule (here the oracle's roundings stand in for an adaptive one), with its
    # residual: full-bit must give back the original weights, part-bit must use exactly that w_high
    n, l = 8, 3
    N, K, M = 130, 448, 150
    w, scale = tl.weights(N, K, 0.02, n, seed=7)
    hi, res = oracle.decompose(w, n, l, rounding)
    lo = oracle.low_encode(res, l, oracle.LOW_SIGNED_L1)
    assert np.array_equal(oracle.compose(hi, lo, l), w.astype(np.int16))
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
    W = nq.NestedWeight(N, K, cfg).fill_from_parts(dev(hi), dev(lo), dev(scale))
    x = inputs.uniform_activations((M, K), seed=3)
    run_both_modes(nq, W, x, hi, w, scale, l)


def test_convolution_and_switching(nq):
    n, l = 8, 2
    B, H, Wd, Cin, Cout = 2, 12, 11, 64, 96
    K = 9 * Cin
    w, scale = tl.weights(Cout, K, inputs.he_sigma(K), n, seed=11)
    cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
    W = nq.NestedWeight.from_int8(dev(w), dev(scale), cfg)
    hi, _ = oracle.decompose(w, n, l, "rtn")
    x = inputs.uniform_activations((B, H, Wd, Cin), seed=5)
    run_both_modes(nq, W, x, hi, w, scale, l, conv=(3, 3, 1, 1))
    # downgrade: full-bit is refused, part-bit still runs; upgrade brings the (l+1)-bit page back
    nq.nq_page_out_low(W.desc)
    W.low.zero_()
    y = torch.empty((B, H, Wd, Cout), dtype=torch.float32, device="cuda")
    cs = nq.nq_conv_shape(B, H, Wd, Cin, Cout, 3, 3, 1, 1)
    with pytest.raises(nq.NQError) as e:
        nq.nq_conv_full(dev(x), cs, W.desc, nq.make_epilogue(0.02), y)
    assert e.value.status == nq.NQ_ERR_NOT_RESIDENT
    nq.nq_page_in_low(W.desc, torch.cuda.Stream())
    run_both_modes(nq, W, x, hi, w, scale, l, conv=(3, 3, 1, 1))
