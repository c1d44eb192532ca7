"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times.  The oracle cannot rank 21M x 768 (or 100M x 1024) rows for thousands of
queries in test time, so it is run, by streaming the very same bytes back from the device in
row chunks, for a seeded sample of the queries; integer stages are checked on everything."""
import numpy as np
import pytest
import torch

from parity import check_topk

pytestmark = pytest.mark.gpu
CHUNK = 1 << 20


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2401_14021_amd import binding
    binding.lib()
    return binding


def _stream_chunks(exact):
    N = exact.shape[0]
    for r0 in range(0, N, CHUNK):
        yield r0, exact[r0:min(N, r0 + CHUNK)].cpu().numpy()


def _oracle_sampled(oracle, exact, queries_np, k):
    return oracle.retrieve_topk_stream(queries_np, _stream_chunks(exact), k)


def _score_of_rows(oracle, exact, queries_np):
    def f(i, ids):
        rows = exact[torch.as_tensor(np.asarray(ids, dtype=np.int64), device=exact.device)].cpu().numpy()
        return oracle.scores(queries_np[i], rows)
    return f


def test_medium_batched_verification_every_query(B, oracle):
    """1M x 768, 16 requests x stride {1,2,4,8}, k = 5, 1024-entry caches: every query checked."""
    from paper_2401_14021_amd import inputs
    w = inputs.WORKLOADS["medium"]
    X = torch.empty(w.N, w.d, dtype=torch.float32, device="cuda")
    _, assign = inputs.clustered_datastore(w.N, w.d, w.n_clusters, w.seed, device="cuda", out=X)
    ds = B.Datastore.from_fp32(X)
    Xnp = X.cpu().numpy()
    for s in (1, 2, 4, 8):
        off = inputs.stride_offsets([s] * 16)
        Q = 16 * s
        rows = inputs.pick_rows(w.N, Q, seed=w.seed + s)
        Qm = inputs.queries_near_rows(X, rows.cuda(), seed=w.seed + 10 + s)
        cids, clen = inputs.speculation_caches(w.N, 16, w.cache_C, off, rows, assign.cpu(), seed=w.seed + 20 + s)
        spec, spec_sc = B.ralm_cache_lookup(cids.cuda(), clen.cuda(), Qm, off.cuda(), ds)
        ws = B.alloc_workspace(Q, ds, w.k, w.k_prime)
        mg = torch.empty(Q, device="cuda")
        ids, sc = B.ralm_retrieve_topk_ex(Qm, ds, w.k, w.k_prime, workspace=ws, out_margin=mg)
        m = B.ralm_verify(spec, ids, off.cuda(), true_stride=w.k)
        assert B.ralm_workspace_overflows(ws) == 0
        qnp = Qm.cpu().numpy()
        wi, wsc = oracle.retrieve_topk(qnp, Xnp, w.k)
        exact, subs, total = check_topk(ids.cpu().numpy(), sc.cpu().numpy(), wi, wsc,
                                        lambda i, g: oracle.scores(qnp[i], Xnp[np.asarray(g, dtype=np.int64)]))
        assert exact >= total - 2
        ci, csc = oracle.cache_lookup(cids.numpy(), clen.numpy(), qnp, off.numpy(), Xnp)
        assert np.array_equal(spec.cpu().numpy(), ci) and np.array_equal(spec_sc.cpu().numpy(), csc)
        assert np.array_equal(m.cpu().numpy(), oracle.verify(ci, ids.cpu().numpy().reshape(-1), off.numpy(), w.k))
        hit = (ci == wi[:, 0]).mean()
        assert 0.05 < hit < 0.95, hit          # the cache hit rate is neither trivial nor perfect
        assert float(mg.min()) > 0             # every query's top-k is separated from the k'-th scan score


@pytest.fixture(scope="module")
def dense21m(B):
    from paper_2401_14021_amd import inputs
    w = inputs.WORKLOADS["dense21m"]
    X = torch.empty(w.N, w.d, dtype=torch.float32, device="cuda")
    _, assign = inputs.clustered_datastore(w.N, w.d, w.n_clusters, w.seed, device="cuda", out=X)
    ds = B.Datastore.from_fp32(X)
    torch.cuda.synchronize()
    yield w, X, assign, ds
    del ds, X
    torch.cuda.empty_cache()


def test_dense21m_sampled_queries(B, oracle, dense21m):
    """21M x 768 bf16 scan + fp32 re-score, Q in {1, 8, 64, 256, 1024}, k in {1, 20}: the oracle
    ranks all 21M rows for a seeded sample of queries; every batch size must agree with it."""
    from paper_2401_14021_amd import inputs
    w, X, assign, ds = dense21m
    Qmax = 1024
    rows = inputs.pick_rows(w.N, Qmax, seed=w.seed + 1)
    Qm = inputs.queries_near_rows(X, rows.cuda(), seed=w.seed + 2)
    sample = [0, 5, 63, 700]
    qs = Qm[sample].cpu().numpy()
    wi, wsc = _oracle_sampled(oracle, X, qs, 20)
    score_of = _score_of_rows(oracle, X, qs)
    # the source row (or a better one) must be found: a sanity check on the oracle's streaming
    assert all(wsc[j, 0] >= 0.5 for j in range(len(sample)))
    for Q in (1, 8, 64, 256, 1024):
        for k in (1, 20):
            ws = B.alloc_workspace(Q, ds, k, w.k_prime)
            ids, sc = B.ralm_retrieve_topk_ex(Qm[:Q].contiguous(), ds, k, w.k_prime, workspace=ws)
            assert B.ralm_workspace_overflows(ws) == 0
            here = [j for j, i in enumerate(sample) if i < Q]
            gi = ids.cpu().numpy()[[sample[j] for j in here]]
            gs = sc.cpu().numpy()[[sample[j] for j in here]]
            exact, subs, total = check_topk(gi, gs, wi[here][:, :k], wsc[here][:, :k],
                                            lambda i, g: score_of(here[i], g))
            assert subs <= 1
            # properties that hold for every query at any size
            assert int(ids.min()) >= 0 and int(ids.max()) < w.N
            assert bool((sc[:, :-1] >= sc[:, 1:]).all()) if k > 1 else True


def test_specloop_steps_full_size(B, oracle, dense21m):
    """Speculation loop stress shape: 512 requests with their own 4096-entry caches, strides
    uniform in 1..8 (about 2300 queries), per step a cache top-1 lookup, one batched exact top-1
    retrieval and the first-mismatch compare; queries drift between steps."""
    from paper_2401_14021_amd import inputs
    w, X, assign, ds = dense21m
    c = inputs.WORKLOADS["specloop"]
    R = 512
    strides = inputs.uniform_strides(R, 1, 8, seed=c.seed)
    off = inputs.stride_offsets(strides)
    Q = int(off[-1])
    rows = inputs.pick_rows(c.N, Q, seed=c.seed + 1)
    Qm = X[rows.cuda()].contiguous()
    cids, clen = inputs.speculation_caches(c.N, R, c.cache_C, off, rows, None, seed=c.seed + 2)
    cids_d, clen_d, off_d = cids.cuda(), clen.cuda(), off.cuda()
    ws = B.alloc_workspace(Q, ds, 1, c.k_prime)
    sample_q = [0, 1000, Q - 1]
    sample_r = [0, 17, 511]
    for step in range(3):
        Qm = inputs.drift_queries(Qm, seed=c.seed + 100 + step)
        spec, spec_sc = B.ralm_cache_lookup(cids_d, clen_d, Qm, off_d, ds)
        ids, sc = B.ralm_retrieve_topk_ex(Qm, ds, 1, c.k_prime, workspace=ws)
        m = B.ralm_verify(spec, ids, off_d, true_stride=1)
        assert B.ralm_workspace_overflows(ws) == 0
        # integer stage: exact on everything
        want_m = oracle.verify(spec.cpu().numpy(), ids.cpu().numpy().reshape(-1), off.numpy(), 1)
        assert np.array_equal(m.cpu().numpy(), want_m)
        # cache lookup: sampled requests, all of their queries, oracle over the gathered cached rows
        qnp = Qm.cpu().numpy()
        for r in sample_r:
            n = int(clen[r])
            ids_r = cids[r, :n].numpy()
            uniq, inv = np.unique(ids_r, return_inverse=True)
            sub = X[torch.from_numpy(uniq).cuda().long()].cpu().numpy()
            lo, hi = int(off[r]), int(off[r + 1])
            ci, csc = oracle.cache_lookup(inv.astype(np.int32)[None, :], np.array([n], dtype=np.int32),
                                          qnp[lo:hi], np.array([0, hi - lo], dtype=np.int64), sub)
            assert np.array_equal(uniq[ci], spec.cpu().numpy()[lo:hi])
            assert np.array_equal(csc, spec_sc.cpu().numpy()[lo:hi])
        if step == 0:
            wi, wsc = _oracle_sampled(oracle, X, qnp[sample_q], 1)
            score_of = _score_of_rows(oracle, X, qnp[sample_q])
            check_topk(ids.cpu().numpy()[sample_q], sc.cpu().numpy()[sample_q], wi, wsc, score_of)
        # rank preservation on every query (Section 3): a cached true top-1 is the cache's top-1
        t = ids[:, 0]
        same = spec == t
        req_of = torch.repeat_interleave(torch.arange(R, device="cuda"), torch.tensor(strides, device="cuda"))
        cached = (cids_d[req_of] == t[:, None]).any(dim=1)
        assert bool((same | ~cached).all())
        assert bool((spec_sc[same] == sc[same, 0]).all())
