"""GPU parity of nq_gemm_batch (many few-row GEMMs in one launch) against the CPU oracle, problem by problem:
layers of different N, K and M in one table, both modes, fp32 and int8 outputs, long and short reductions mixed,
empty problems, the refused cases."""
import numpy as np
import pytest
import torch

import nq_testlib as tl
from nq_testlib import Case, check_outputs, dev, host
from oracle import nq_oracle as oracle
from paper_2506_17870_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nq():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    return nq


def make_jobs(nq, shapes, n, l, out_int8, seed=0, fmt=None):
    """One nested layer + activations per (M, N, K); returns the job list and what the oracle needs."""
    jobs, refs = [], []
    for i, (M, N, K) in enumerate(shapes):
        w_int, scale = tl.weights(N, K, 0.02, n, seed + i)
        case = Case(nq, w_int, scale, n, l)
        x = inputs.uniform_activations((M, K), seed=seed + 100 + i) >> (8 - n)
        bias = inputs.small_floats(N, 0.1, seed=i)
        res = inputs.uniform_activations((M, N), seed=seed + 200 + i) if out_int8 else None
        y = torch.full((M, N), 77, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
        keep = dict(x=dev(x), bias=dev(bias), res=dev(res) if res is not None else None, y=y, case=case)
        epi = nq.make_epilogue(0.02, keep["bias"], keep["res"], 0.03, out_int8, out_int8, 5.0)
        jobs.append((keep["x"], M, case.W.desc, epi, y))
        refs.append(dict(keep=keep, x=x, bias=bias, res=res, case=case))
    return jobs, refs


def check_jobs(refs, full, out_int8):
    for i, r in enumerate(refs):
        case = r["case"]
        if r["x"].shape[0] == 0 or case.N == 0:
            continue
        acc = oracle.gemm_acc(r["x"], case.ow_full if full else case.ow_part)
        y_ref = oracle.epilogue(acc, s_a=0.02, s_w=case.scale, part_l_bits=0 if full else case.l, bias=r["bias"],
                                residual=r["res"], s_r=0.03, relu=out_int8, out_int8=out_int8, inv_s_out=5.0)
        try:
            check_outputs(host(r["keep"]["y"]), None, y_ref, acc, out_int8)
        except AssertionError as e:
            raise AssertionError(f"{e} (problem {i}, {'full' if full else 'part'}-bit)") from None


SHAPES = [(64, 512, 512), (16, 96, 320), (1, 32, 4096), (33, 144, 1088), (64, 48, 2304), (7, 992, 64), (40, 16, 16),
          (64, 2048, 256)]


@pytest.mark.parametrize("n,l", [(8, 2), (8, 4), (6, 3)])
@pytest.mark.parametrize("out_int8", [False, True])
def test_batch_matches_the_oracle(nq, n, l, out_int8):
    jobs, refs = make_jobs(nq, SHAPES, n, l, out_int8, seed=n + l)
    ws = torch.empty(nq.nq_gemm_batch_workspace_bytes(len(jobs)), dtype=torch.uint8, device="cuda")
    for full in (True, False):
        for r in refs:
            r["keep"]["y"].fill_(77)
        nq.nq_gemm_batch(jobs, full, ws)
        torch.cuda.synchronize()
        check_jobs(refs, full, out_int8)


def test_short_reductions_only_and_one_row_tile(nq):
    # no problem above 32 rows, none with K >= 2048: the other two instantiations of the batch kernel
    shapes = [(32, 64, 64), (5, 160, 512), (20, 96, 1024), (1, 32, 16)]
    jobs, refs = make_jobs(nq, shapes, 8, 3, False, seed=9)
    ws = torch.empty(nq.nq_gemm_batch_workspace_bytes(len(jobs)), dtype=torch.uint8, device="cuda")
    for full in (True, False):
        nq.nq_gemm_batch(jobs, full, ws)
        torch.cuda.synchronize()
        check_jobs(refs, full, False)
    shapes = [(64, 64, 64), (40, 160, 512)]
    jobs, refs = make_jobs(nq, shapes, 8, 3, True, seed=10)
    nq.nq_gemm_batch(jobs, True, ws)
    torch.cuda.synchronize()
    check_jobs(refs, True, True)


def test_a_stack_of_layers(nq):
    # the weight-bound configuration as a stack: 48 distinct 64 x 512 -> 512 layers in one launch
    shapes = [(64, 512, 512)] * 48
    jobs, refs = make_jobs(nq, shapes, 8, 2, False, seed=3)
    ws = torch.empty(nq.nq_gemm_batch_workspace_bytes(len(jobs)), dtype=torch.uint8, device="cuda")
    for full in (True, False):
        nq.nq_gemm_batch(jobs, full, ws)
        torch.cuda.synchronize()
        check_jobs(refs, full, False)


def test_empty_problems_and_refusals(nq):
    jobs, refs = make_jobs(nq, [(0, 64, 64), (12, 64, 64)], 8, 2, False, seed=1)
    ws = torch.empty(nq.nq_gemm_batch_workspace_bytes(4), dtype=torch.uint8, device="cuda")
    nq.nq_gemm_batch(jobs, False, ws)
    torch.cuda.synchronize()
    check_jobs(refs, False, False)
    nq.nq_gemm_batch([], False, ws)                                  # nothing to do
    big, _ = make_jobs(nq, [(65, 64, 64)], 8, 2, False)              # more than 64 rows
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_batch(big, False, ws)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    mixed = make_jobs(nq, [(8, 64, 64)], 8, 2, False)[0] + make_jobs(nq, [(8, 64, 64)], 8, 3, False)[0]
    with pytest.raises(nq.NQError) as e:                              # two nestings in one table
        nq.nq_gemm_batch(mixed, False, ws)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    kinds = make_jobs(nq, [(8, 64, 64)], 8, 2, False)[0] + make_jobs(nq, [(8, 64, 64)], 8, 2, True)[0]
    with pytest.raises(nq.NQError) as e:                              # fp32 and int8 outputs in one table
        nq.nq_gemm_batch(kinds, False, ws)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_batch(jobs, False, small)
    assert e.value.status == nq.NQ_ERR_RANGE
    nq.nq_page_out_low(jobs[1][2])
    with pytest.raises(nq.NQError) as e:                              # full-bit with a page paged out
        nq.nq_gemm_batch(jobs, True, ws)
    assert e.value.status == nq.NQ_ERR_NOT_RESIDENT
