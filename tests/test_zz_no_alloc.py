"""The entry point that allocates nothing (static scratch array) against ivf_search (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1802_02422_amd as ivf
import parity


def test_noalloc_search_matches_the_allocating_entry_point(tiny):
    """Two calls in a row through the C ABI, the second with a smaller batch and other parameters
    (the static array keeps the first call's contents): ids and distances are bit-identical to
    ivf_search's.  A batch whose scratch does not fit the array is rejected before any launch."""
    spec, ix, Q, X = tiny
    print("case: ivf_search_noalloc tiny", flush=True)
    handle = ivf.ivf_load_index(parity.to_device(ix))
    Qd = torch.from_numpy(Q).cuda()
    for nq, nprobe, tau, k in ((len(Q), spec.nprobe, spec.prune_frac, spec.k), (7, 5, 1.0, 3), (70, 33, 0.3, 50)):
        print("  batch", nq, nprobe, tau, k, flush=True)
        q = Qd[:nq].contiguous()
        ref_ids, ref_d = ivf.ivf_search(handle, q, nprobe, tau, k)
        ids = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
        d = torch.full((nq, k), -7.0, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ivf.ivf_search_noalloc(handle, q, nprobe, tau, k, ids, d)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(ids, ref_ids) and torch.equal(d, ref_d), (nq, nprobe, tau, k)
    # K = 1024: 64 MiB of scratch hold about 12 000 queries' distance rows; 40 000 do not fit
    big = Qd.repeat(400, 1).contiguous()
    ids = torch.empty((big.shape[0], 3), dtype=torch.int32, device="cuda")
    d = torch.empty((big.shape[0], 3), dtype=torch.float32, device="cuda")
    with pytest.raises(ivf.IvfError):
        ivf.ivf_search_noalloc(handle, big, 4, 0.5, 3, ids, d)
    assert "scratch" in ivf.ivf_last_error()
    ivf.ivf_free_index(handle)
