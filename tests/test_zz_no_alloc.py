"""nq_gemm_batch_static (the entry point that allocates nothing: its job table lives in a device array of the
library) against nq_gemm_batch on the same problems, bit for bit, on two calls in a row, the second with a
smaller table (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from nq_testlib import host
from test_gpu_batch import make_jobs

pytestmark = pytest.mark.gpu


def test_static_table_matches_the_workspace_call():
    import paper_2506_17870_amd as nq
    assert torch.cuda.is_available()
    first = [(64, 512, 512), (16, 96, 320), (1, 32, 4096), (33, 144, 1088), (7, 992, 64), (64, 2048, 256)]
    second = [(20, 160, 256), (64, 64, 64)]
    for out_int8 in (False, True):
        for shapes in (first, second):                 # two calls in a row, the second one smaller
            jobs, refs = make_jobs(nq, shapes, 8, 2, out_int8, seed=len(shapes))
            ws = torch.empty(nq.nq_gemm_batch_workspace_bytes(len(jobs)), dtype=torch.uint8, device="cuda")
            for full in (True, False):
                nq.nq_gemm_batch(jobs, full, ws)
                torch.cuda.synchronize()
                want = [host(r["keep"]["y"]).copy() for r in refs]
                for r in refs:
                    r["keep"]["y"].fill_(77)
                nq.nq_gemm_batch_static(jobs, full)
                torch.cuda.synchronize()
                for i, r in enumerate(refs):
                    got = host(r["keep"]["y"])
                    assert np.array_equal(got.view(np.uint8), want[i].view(np.uint8)), (out_int8, full, i)
                    assert not np.all(got == 77)
    too_many = [jobs[0]] * (nq.NQ_GEMM_BATCH_STATIC_MAX + 1)
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_batch_static(too_many, False)
    assert e.value.status == nq.NQ_ERR_SHAPE
