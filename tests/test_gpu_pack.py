"""GPU parity of decomposition and packing (through the C ABI) against the CPU oracle: bit exact."""
import numpy as np
import pytest
import torch

from nq_testlib import dev, host

pytestmark = pytest.mark.gpu

ALL_NL = [(8, l) for l in range(1, 7)] + [(6, l) for l in range(1, 5)]


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def rand_w(n_bits, shape, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(-(1 << (n_bits - 1)), 1 << (n_bits - 1), size=shape).astype(np.int8)


@pytest.mark.parametrize("n,l", ALL_NL)
def test_decompose_matches_oracle(nq, oracle, n, l):
    for shape in [(1, 256 if n == 8 else 64), (7, 37), (64, 512), (3, 16)]:
        w = rand_w(n, shape, seed=l)
        if shape[0] == 1:
            w = np.arange(-(1 << (n - 1)), 1 << (n - 1), dtype=np.int8).reshape(1, -1)   # every INT-n value
        N, K = w.shape
        hi = torch.empty((N, K), dtype=torch.int8, device="cuda")
        lo = torch.empty((N, K), dtype=torch.int8, device="cuda")
        nq.nq_decompose(dev(w), N, K, nq.make_cfg(n, l), hi, lo)
        o_hi, res = oracle.decompose(w, n, l, "bitshift")
        o_lo = oracle.low_encode(res, l, oracle.LOW_UNSIGNED_L)
        assert np.array_equal(host(hi), o_hi) and np.array_equal(host(lo), o_lo)


@pytest.mark.parametrize("n,l", ALL_NL)
@pytest.mark.parametrize("shape", [(1, 1), (33, 65), (70, 200), (64, 128), (96, 576), (5, 48)])
def test_dense_pages_match_oracle(nq, oracle, n, l, shape):
    h = n - l
    w = rand_w(n, shape, seed=10 * n + l)
    N, K = shape
    cfg = nq.make_cfg(n, l)
    hb, lb = nq.nq_packed_bytes(N, K, h), nq.nq_packed_bytes(N, K, l)
    assert hb == oracle.dense_bytes(N, K, h) and lb == oracle.dense_bytes(N, K, l)
    ph = torch.full((hb,), 0xAA, dtype=torch.uint8, device="cuda")
    pl = torch.full((lb,), 0xAA, dtype=torch.uint8, device="cuda")
    nq.nq_decompose_pack(dev(w), N, K, cfg, ph, pl)
    o_ph, o_pl = oracle.decompose_pack(w, n, l)
    assert np.array_equal(host(ph), o_ph), "higher-bit page"
    assert np.array_equal(host(pl), o_pl), "lower-bit page"
    # the two-step route gives the same pages
    hi = torch.empty((N, K), dtype=torch.int8, device="cuda")
    lo = torch.empty((N, K), dtype=torch.int8, device="cuda")
    nq.nq_decompose(dev(w), N, K, cfg, hi, lo)
    ph2, pl2 = torch.zeros_like(ph), torch.zeros_like(pl)
    nq.nq_pack(hi, lo, N, K, cfg, ph2, pl2)
    assert torch.equal(ph, ph2) and torch.equal(pl, pl2)
    # one page at a time
    ph3 = torch.zeros_like(ph)
    nq.nq_pack(hi, None, N, K, cfg, ph3, None)
    pl3 = torch.zeros_like(pl)
    nq.nq_pack(None, lo, N, K, cfg, None, pl3)
    assert torch.equal(ph, ph3) and torch.equal(pl, pl3)
    # and back
    hi2, lo2 = torch.zeros_like(hi), torch.zeros_like(lo)
    nq.nq_unpack(ph, pl, N, K, cfg, hi2, lo2)
    assert torch.equal(hi, hi2) and torch.equal(lo, lo2)


@pytest.mark.parametrize("n,l", [(8, 2), (8, 3), (8, 4), (8, 5), (6, 2), (6, 1)])
def test_paper_word_pages_match_oracle(nq, oracle, n, l):
    h = n - l
    N, K = 9, 131
    w = rand_w(n, (N, K), seed=n + l)
    cfg = nq.make_cfg(n, l, layout=nq.NQ_LAYOUT_PAPER_U64)
    ph = torch.zeros(nq.nq_packed_bytes(N, K, h, nq.NQ_LAYOUT_PAPER_U64), dtype=torch.uint8, device="cuda")
    pl = torch.zeros(nq.nq_packed_bytes(N, K, l, nq.NQ_LAYOUT_PAPER_U64), dtype=torch.uint8, device="cuda")
    nq.nq_decompose_pack(dev(w), N, K, cfg, ph, pl)
    o_ph, o_pl = oracle.decompose_pack(w, n, l, layout="paper")
    assert np.array_equal(host(ph), o_ph) and np.array_equal(host(pl), o_pl)
    hi = torch.empty((N, K), dtype=torch.int8, device="cuda")
    lo = torch.empty((N, K), dtype=torch.int8, device="cuda")
    nq.nq_unpack(ph, pl, N, K, cfg, hi, lo)
    o_hi, res = oracle.decompose(w, n, l, "bitshift")
    assert np.array_equal(host(hi), o_hi) and np.array_equal(host(lo), oracle.low_encode(res, l, 0))
    # recomposition on the host of what the device unpacked (Eq. 4) gives the weights back
    assert np.array_equal(host(hi).astype(np.int16) * (1 << l) + host(lo), w)


def test_benchmark_sized_pages(nq, oracle):
    # the ResNet-18 layer of the benchmark, and one wide ragged matrix
    for (N, K, n, l) in [(64, 576, 8, 2), (1000, 2048, 8, 2), (3072, 768, 8, 3)]:
        w = rand_w(n, (N, K), seed=N)
        cfg = nq.make_cfg(n, l)
        ph = torch.empty(nq.nq_packed_bytes(N, K, n - l), dtype=torch.uint8, device="cuda")
        pl = torch.empty(nq.nq_packed_bytes(N, K, l), dtype=torch.uint8, device="cuda")
        nq.nq_decompose_pack(dev(w), N, K, cfg, ph, pl)
        o_ph, o_pl = oracle.decompose_pack(w, n, l)
        assert np.array_equal(host(ph), o_ph) and np.array_equal(host(pl), o_pl)


@pytest.mark.parametrize("n,l,fmt", [(8, 2, 0), (8, 5, 0), (6, 3, 0), (8, 3, 1)])
def test_batched_decompose_pack(nq, oracle, n, l, fmt):
    # 150 tensors of mixed shapes (more than one launch's worth of jobs, ragged tiles, an empty one, a large one)
    rng = np.random.default_rng(n * 10 + l)
    shapes = [(int(rng.integers(1, 130)), int(rng.integers(1, 300))) for _ in range(147)] + [(0, 16), (512, 4608), (64, 576)]
    cfg = nq.make_cfg(n, l, fmt)
    lf = l + fmt
    jobs, refs = [], []
    for i, (N, K) in enumerate(shapes):
        w = rng.integers(-(1 << (n - 1)), 1 << (n - 1), size=(N, K)).astype(np.int8)
        ph = torch.full((max(nq.nq_packed_bytes(N, K, n - l), 16),), 0x5A, dtype=torch.uint8, device="cuda")
        pl = torch.full((max(nq.nq_packed_bytes(N, K, lf), 16),), 0x5A, dtype=torch.uint8, device="cuda")
        jobs.append((torch.from_numpy(w).cuda() if N else torch.empty(16, dtype=torch.int8, device="cuda"), N, K, ph, pl))
        refs.append(w)
    nq.nq_decompose_pack_batch(jobs, cfg)
    torch.cuda.synchronize()
    for (d_w, N, K, ph, pl), w in zip(jobs, refs):
        if N == 0:
            continue
        ph1, pl1 = torch.zeros_like(ph), torch.zeros_like(pl)
        nq.nq_decompose_pack(d_w, N, K, cfg, ph1, pl1)      # itself checked against the oracle above
        torch.cuda.synchronize()
        hb, lb = nq.nq_packed_bytes(N, K, n - l), nq.nq_packed_bytes(N, K, lf)
        assert torch.equal(ph[:hb], ph1[:hb]) and torch.equal(pl[:lb], pl1[:lb]), (N, K)
    # and directly against the oracle for a few of them
    if fmt == 0:
        for idx in (0, 5, 148, 149):
            d_w, N, K, ph, pl = jobs[idx]
            oh, ol = oracle.decompose_pack(refs[idx], n, l)
            assert np.array_equal(ph.cpu().numpy()[:oh.size], oh) and np.array_equal(pl.cpu().numpy()[:ol.size], ol)
