"""The cache lookup that allocates nothing (``ralm_cache_lookup_static``: merge slots in an
array inside the library) against the ordinary entry point called with a caller workspace.
Two calls in a row on the same GPU, the second with a smaller input, so that slots left over
from the first call would show; then the size limit."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2401_14021_amd import binding
    binding.lib()
    return binding


def _case(B, ds, N, R, C, strides, seed):
    from paper_2401_14021_amd import inputs
    off = inputs.stride_offsets(strides)
    Q = int(off[-1])
    rows = inputs.pick_rows(N, Q, seed=seed)
    Qm = inputs.queries_near_rows(ds.exact, rows.cuda(), seed=seed + 1)
    cids, clen = inputs.speculation_caches(N, R, C, off, rows, None, seed=seed + 2)
    return cids.cuda(), clen.cuda(), Qm, off.cuda()


def test_static_scratch_lookup_equals_workspace_lookup(B, oracle):
    from paper_2401_14021_amd import inputs
    N, d = 50_000, 768
    X, _ = inputs.clustered_datastore(N, d, 128, seed=77, device="cuda")
    ds = B.Datastore(X)
    # few requests with large caches: every cache is split over several workgroups that merge
    # through the scratch slots (the path that needs scratch at all)
    for R, C, strides, seed in ((6, 2048, [8, 3, 1, 5, 8, 2], 1), (2, 700, [2, 1], 9)):
        cids, clen, Qm, off = _case(B, ds, N, R, C, strides, seed)
        Qt = Qm.shape[0]
        want_i, want_s = B.ralm_cache_lookup(cids, clen, Qm, off, ds,
                                             workspace=torch.empty(Qt, dtype=torch.int64, device="cuda"))
        got_i = torch.full((Qt,), -7, dtype=torch.int32, device="cuda")
        got_s = torch.full((Qt,), float("nan"), dtype=torch.float32, device="cuda")
        B.ralm_cache_lookup_static(cids, clen, Qm, off, ds, got_i, got_s)
        torch.cuda.synchronize()
        assert torch.equal(got_i, want_i) and torch.equal(got_s, want_s)
        # and both are the oracle's answer
        oi, osc = oracle.cache_lookup(cids.cpu().numpy(), clen.cpu().numpy(), Qm.cpu().numpy(), off.cpu().numpy(),
                                      X.cpu().numpy())
        assert np.array_equal(got_i.cpu().numpy(), oi) and np.array_equal(got_s.cpu().numpy(), osc)


def test_static_scratch_lookup_rejects_sizes_beyond_its_limit(B):
    from paper_2401_14021_amd import inputs
    X, _ = inputs.clustered_datastore(1000, 64, 8, seed=3, device="cuda")
    ds = B.Datastore(X)
    P = X.data_ptr()
    rc = B.lib().ralm_cache_lookup_static(P, P, 4, 1, P, 65537, P, ctypes.byref(ds.desc), P, P, None)
    assert rc == 7 and b"65536" in B.lib().ralm_last_error()
