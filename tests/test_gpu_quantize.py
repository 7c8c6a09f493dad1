"""GPU parity of the per-channel quantiser (Eq. 1) and of its fusion with decomposition and packing
(Alg. 1 steps 1-3).  Both sides take the quotient and the rounding in fp32; bar: scales, codes and pages
bit exact against the CPU oracle."""
import numpy as np
import pytest
import torch

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


def awkward_weights(N, K, seed):
    """Gaussian rows plus the rows a quantiser gets wrong first: all zero, a single non-zero, exact ties
    (absmax = qmax so the step is 1 and x.5 values sit on rounding boundaries), very small and very large
    magnitudes, and a row whose extreme value is negative."""
    w = inputs.float_weights(N, K, 0.02, seed)
    rng = np.random.default_rng(seed + 17)
    if N > 6:
        w[0] = 0.0
        w[1] = 0.0
        w[1, K // 2] = -3.25
        w[2] = rng.integers(-254, 255, size=K).astype(np.float32) / 2.0       # multiples of 0.5 ...
        w[2, 0] = 127.0                                                       # ... on a grid of step 1
        w[3] *= 1e-20
        w[4] *= 1e20
        w[5] = -np.abs(w[5])
        w[6] = rng.integers(-62, 63, size=K).astype(np.float32) / 2.0
        w[6, K - 1] = 31.0                                                    # step 1 for 6-bit codes
    return w


@pytest.mark.parametrize("n_bits", [8, 6, 4, 2])
@pytest.mark.parametrize("N,K", [(96, 320), (33, 70), (130, 1028), (7, 3), (64, 4608), (1, 1), (40, 2049)])
def test_scales_and_codes(nq, n_bits, N, K):
    w = awkward_weights(N, K, seed=N + K + n_bits)
    wi_ref, s_ref = oracle.quantize(w, n_bits)
    for offset in (0, 1):            # 1: the tensor starts off a 16-byte boundary (no vector loads)
        buf = torch.zeros(N * K + 1, dtype=torch.float32, device="cuda")
        d_w = buf[offset:offset + N * K]
        d_w.copy_(torch.from_numpy(w.ravel()))
        d_wi = torch.full((N * K,), 99, dtype=torch.int8, device="cuda")
        d_s = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        nq.nq_quantize(d_w, N, K, n_bits, d_wi, d_s)
        torch.cuda.synchronize()
        assert np.array_equal(host(d_s).view(np.uint32), s_ref.view(np.uint32)), "channel scales differ"
        assert np.array_equal(host(d_wi).reshape(N, K), wi_ref), "codes differ"


@pytest.mark.parametrize("n,l", ALL_NL)
@pytest.mark.parametrize("fmt", ["unsigned", "signed"])
def test_fused_pages(nq, n, l, fmt):
    h = n - l
    for (N, K) in [(96, 320), (45, 203), (130, 1028)]:
        w = awkward_weights(N, K, seed=N + n + l)
        wi_ref, s_ref = oracle.quantize(w, n)
        if fmt == "unsigned":
            cfg = nq.make_cfg(n, l)
            ph_ref, pl_ref = oracle.decompose_pack(wi_ref, n, l)
            lf = l
        else:
            cfg = nq.make_cfg(n, l, nq.NQ_LOW_SIGNED_L1)
            hi_ref, res = oracle.decompose(wi_ref, n, l, "rtn")
            lo_ref = oracle.low_encode(res, l, oracle.LOW_SIGNED_L1)
            ph_ref = oracle.pack_dense(hi_ref, h, oracle.KIND_CARRIER)
            pl_ref = oracle.pack_dense(lo_ref, l + 1, oracle.KIND_BITSTRING)
            lf = l + 1
        assert ph_ref.size == nq.nq_packed_bytes(N, K, h) and pl_ref.size == nq.nq_packed_bytes(N, K, lf)
        ph = torch.full((ph_ref.size,), 0xA5, dtype=torch.uint8, device="cuda")
        pl = torch.full((pl_ref.size,), 0xA5, dtype=torch.uint8, device="cuda")
        d_s = torch.zeros(N, dtype=torch.float32, device="cuda")
        nq.nq_quantize_decompose_pack(dev(w), N, K, cfg, d_s, ph, pl)
        torch.cuda.synchronize()
        assert np.array_equal(host(d_s).view(np.uint32), s_ref.view(np.uint32)), "channel scales differ"
        assert np.array_equal(host(ph), ph_ref), f"higher-bit page differs ({N}x{K})"
        assert np.array_equal(host(pl), pl_ref), f"lower-bit page differs ({N}x{K})"
        # the same pages as the two-call route on the device
        d_wi = torch.empty((N, K), dtype=torch.int8, device="cuda")
        d_s2 = torch.empty(N, dtype=torch.float32, device="cuda")
        ph2, pl2 = torch.zeros_like(ph), torch.zeros_like(pl)
        nq.nq_quantize(dev(w), N, K, n, d_wi, d_s2)
        nq.nq_decompose_pack(d_wi, N, K, cfg, ph2, pl2)
        torch.cuda.synchronize()
        assert torch.equal(ph, ph2) and torch.equal(pl, pl2) and torch.equal(d_s, d_s2)
        # one page only
        ph3 = torch.zeros_like(ph)
        nq.nq_quantize_decompose_pack(dev(w), N, K, cfg, d_s, ph3, None)
        torch.cuda.synchronize()
        assert torch.equal(ph3, ph)


def test_float_weights_to_outputs(nq):
    """fp32 weights -> pages on the device -> both modes of the GEMM, against the oracle run from the same
    fp32 weights (Eq. 1, Eq. 5, Eq. 2 / Eq. 8)."""
    n, l = 8, 3
    N, K, M = 160, 512, 200
    w = inputs.float_weights(N, K, 0.02, seed=5)
    W = nq.NestedWeight.from_float(dev(w), nq.make_cfg(n, l))
    wi_ref, s_ref = oracle.quantize(w, n)
    hi_ref, _ = oracle.decompose(wi_ref, n, l, "bitshift")
    x = inputs.uniform_activations((M, K), seed=9)
    for full in (True, False):
        acc_ref = oracle.gemm_acc(x, (wi_ref if full else hi_ref).astype(np.int16))
        y_ref = oracle.epilogue(acc_ref, 0.02, s_ref, part_l_bits=0 if full else l)
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        (nq.nq_gemm_full if full else nq.nq_gemm_part)(dev(x), M, W.desc, nq.make_epilogue(0.02, d_acc_dump=acc), y)
        torch.cuda.synchronize()
        check_outputs(host(y), host(acc), y_ref, acc_ref, False)


@pytest.mark.parametrize("count", [1, 3, 255, 4096, 100_003, 3_000_000])
def test_tensor_scale(nq, count):
    # Eq. 1's step for a whole tensor (per-tensor activation quantisation): absmax / 127 in fp32, 1 for zeros
    rng = np.random.default_rng(count)
    for variant in ("gauss", "zeros", "peak_last", "unaligned"):
        v = rng.normal(0.0, 3.0, size=count + 1).astype(np.float32)
        first = 1 if variant == "unaligned" else 0          # a tensor that starts 4 bytes off a 16-byte boundary
        if variant == "zeros":
            v[:] = 0.0
        if variant == "peak_last":
            v[first + count - 1] = -1e20
        src = dev(v)[first:first + count]
        out = torch.full((1,), 77.0, dtype=torch.float32, device="cuda")
        nq.nq_tensor_scale(src, count, 8, out)
        torch.cuda.synchronize()
        _, s_ref = oracle.quantize(v[first:first + count].reshape(1, -1), 8)
        assert host(out).view(np.uint32)[0] == s_ref.view(np.uint32)[0], (variant, count)


@pytest.mark.parametrize("count", [1, 3, 1023, 1025, 4096, 100_003, 3_000_000])
def test_quantize_tensor(nq, count):
    # Eq. 1 for a whole tensor: the step of nq_tensor_scale and the codes, ties to even, clipped, both bit exact
    rng = np.random.default_rng(1000 + count)
    for variant, n_bits in (("gauss", 8), ("gauss", 6), ("zeros", 8), ("ties", 8), ("unaligned", 8)):
        v = rng.normal(0.0, 3.0, size=count + 1).astype(np.float32)
        first = 1 if variant == "unaligned" else 0
        if variant == "zeros":
            v[:] = 0.0
        if variant == "ties":
            # absmax 127 makes the step 1: halves must round to even, values beyond the range must clip
            v[:] = rng.integers(-140, 141, size=count + 1).astype(np.float32) + 0.5
            v[first] = 127.0
            v = np.clip(v, -127.0, 127.0) if count > 1 else v
        src = dev(v)[first:first + count]
        codes = torch.full((count + 8,), 55, dtype=torch.int8, device="cuda")
        step = torch.full((1,), 77.0, dtype=torch.float32, device="cuda")
        nq.nq_quantize_tensor(src, count, n_bits, codes, step)
        torch.cuda.synchronize()
        c_ref, s_ref = oracle.quantize(v[first:first + count].reshape(1, -1), n_bits)
        assert host(step).view(np.uint32)[0] == s_ref.view(np.uint32)[0], (variant, count)
        assert np.array_equal(host(codes)[:count], c_ref.reshape(-1)), (variant, count)
        assert np.all(host(codes)[count:] == 55), "wrote past the end"
