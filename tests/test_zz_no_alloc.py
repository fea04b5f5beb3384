"""vlq_search_noalloc (the entry point for callers that cannot allocate) against vlq_search, through
the C ABI: two calls in a row on the same index, the second with a smaller batch, must give the rows
of the allocating entry point, and the device's free memory must not move across the calls."""
import numpy as np
import pytest
import torch

from test_gpu_parity import CASES, DEV, dev, make_index
from util import problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vlq():
    import paper_1901_00275_amd as vlq

    vlq.lib()
    return vlq


@pytest.mark.parametrize("name", ["sift_ragged", "deep_m16"])
def test_noalloc_search_matches_search(vlq, name):
    kw, w1, w2, K = CASES[name]
    pr = problem(**kw)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        Yd = dev(pr.Y)
        for nq in (len(pr.Y), 20):  # the second call is smaller: whatever the first left in the scratch must not matter
            want_d = torch.empty(nq, K, device=DEV)
            want_i = torch.empty(nq, K, dtype=torch.int32, device=DEV)
            vlq.vlq_search(idx, Yd[:nq].contiguous(), nq, w1, w2, K, want_d, want_i)
            got_d = torch.full((nq, K), -1.0, device=DEV)
            got_i = torch.full((nq, K), -7, dtype=torch.int32, device=DEV)
            q = Yd[len(pr.Y) - nq:].contiguous() if nq < len(pr.Y) else Yd
            want2_d = torch.empty(nq, K, device=DEV)
            want2_i = torch.empty(nq, K, dtype=torch.int32, device=DEV)
            vlq.vlq_search(idx, q, nq, w1, w2, K, want2_d, want2_i)
            torch.cuda.synchronize()
            free0 = torch.cuda.mem_get_info()[0]
            vlq.vlq_search_noalloc(idx, q, nq, w1, w2, K, got_d, got_i)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free0
            assert torch.equal(got_i, want2_i) and torch.equal(got_d, want2_d)
            assert (got_i >= 0).all()
    finally:
        vlq.vlq_index_free(idx)


def test_noalloc_search_rejects_what_does_not_fit(vlq):
    kw, w1, w2, K = CASES["sift_ragged"]
    pr = problem(**kw)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        nq = 300000  # far beyond 32 MiB of scratch at 16 bytes per visited sub-region
        Y = torch.zeros(nq, pr.D, device=DEV)
        od = torch.full((nq, K), -1.0, device=DEV)
        oi = torch.full((nq, K), -7, dtype=torch.int32, device=DEV)
        with pytest.raises(vlq.VlqError) as ei:
            vlq.vlq_search_noalloc(idx, Y, nq, w1, w2, K, od, oi)
        assert ei.value.code == vlq.VLQ_EINVAL and "scratch" in str(ei.value)
        torch.cuda.synchronize()
        assert (oi == -7).all()  # nothing was written
        # bad arguments are rejected like vlq_search's
        with pytest.raises(vlq.VlqError):
            vlq.vlq_search_noalloc(idx, Y, 10, 0, w2, K, od, oi)
    finally:
        vlq.vlq_index_free(idx)
