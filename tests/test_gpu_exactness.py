"""Inputs built to break a low-precision scan: the exact top-k must come out anyway.

The scan keeps the k' rows with the best bf16/fp16 scores; the answer is exact only if the true
top-k rows are among them.  Here they are not, or not reliably: rows that differ below the scan
dtype's resolution (identical scan scores, different exact scores), and more than k rows packed
within 2^-9 relative of the rank-k score with k' = k.  The library has to notice (its margin
check) and answer such queries by its exact pass; ids must equal the CPU oracle's."""
import numpy as np
import pytest
import torch

from parity import check_topk

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2401_14021_amd import binding
    binding.lib()
    return binding


def _score_fn(oracle, Qm, Xnp, metric="ip"):
    def f(i, ids):
        return oracle.scores(Qm[i], Xnp[np.asarray(ids, dtype=np.int64)], metric)
    return f


def _scaled_copies(base, n, rel, gen):
    """n rows base * (1 + a_j * rel), a_j distinct and evenly spread over (-1, 1), shuffled."""
    a = (torch.arange(n, dtype=torch.float64) + 0.5) / n * 2 - 1
    a = a[torch.randperm(n, generator=gen)]
    return (base.double()[None, :] * (1 + a[:, None] * rel)).float()


def _run(B, ds, Qm, k, k_prime):
    ws = B.alloc_workspace(Qm.shape[0], ds, k, k_prime)
    mg = torch.empty(Qm.shape[0], dtype=torch.float32, device="cuda")
    ids, sc = B.ralm_retrieve_topk_ex(Qm.cuda(), ds, k, k_prime, workspace=ws, out_margin=mg)
    return ids.cpu().numpy(), sc.cpu().numpy(), B.ralm_workspace_counters(ws), mg.cpu().numpy()


@pytest.mark.parametrize("scan_dtype,rel", [(torch.bfloat16, 2.0 ** -10), (torch.float16, 2.0 ** -13)])
@pytest.mark.parametrize("k_prime", [0, 20])
def test_rows_that_differ_below_the_scan_resolution(B, oracle, scan_dtype, rel, k_prime):
    """100 rows are one vector scaled by factors within +-rel: in the scan dtype they are the SAME
    row (every component rounds back to the base value), so their scan scores are equal and the scan
    keeps the 64 (or 20) with the lowest ids; their exact scores differ by up to 2 * rel relative,
    far more than the 1e-5 that the acceptance rule forgives."""
    from paper_2401_14021_amd import inputs
    g = torch.Generator().manual_seed(5)
    N, d, k = 30000, 256, 20
    X, _ = inputs.clustered_datastore(N, d, 32, seed=41)
    base = X[123].to(scan_dtype).float()                 # representable in the scan dtype
    where = torch.randperm(N, generator=g)[:100]
    X[where] = _scaled_copies(base, 100, rel, g)
    assert bool((X[where].to(scan_dtype).float() == base[None, :]).all())
    Qm = torch.stack([base, base * 0.7 + 0.01 * torch.randn(d, generator=g), X[5]])
    ds = B.Datastore.from_fp32(X.cuda(), scan_dtype)
    ids, sc, c, mg = _run(B, ds, Qm, k, k_prime)
    wi, wsc = oracle.retrieve_topk(Qm.numpy(), X.numpy(), k)
    # the scaled copies are the best rows of queries 0 and 1, in the order of their factors
    assert set(wi[0].tolist()) <= set(where.tolist()) and set(wi[1].tolist()) <= set(where.tolist())
    assert np.array_equal(ids, wi), (ids[:2], wi[:2], c)
    assert np.array_equal(sc, wsc)
    assert c["exact_pass"] >= 2 and c["unanswered"] == 0 and c["soft_certified"] + c["exact_pass"] == 3, c


@pytest.mark.parametrize("scan_dtype", [torch.bfloat16, torch.float16])
def test_more_than_k_rows_near_the_rank_k_score_with_k_prime_equal_k(B, oracle, scan_dtype):
    """k' = k = 20 and, per query, 60 rows whose exact scores lie within 2^-9 relative of each other
    around rank 20, each with its own rounding error in the scan: the scan's top 20 are not the
    exact top 20.  With k' = k the margin is zero by construction, so every query takes the exact
    pass; the same data with the default k' must agree with the oracle as well."""
    from paper_2401_14021_amd import inputs
    g = torch.Generator().manual_seed(17)
    N, d, k, Q = 40000, 768, 20, 9
    X, _ = inputs.clustered_datastore(N, d, 64, seed=43)
    rows = inputs.pick_rows(N, Q, seed=2)
    Qm = inputs.queries_near_rows(X, rows, seed=3)
    for i in range(Q):
        base = X[rows[i]].clone()
        where = torch.randperm(N, generator=g)[:60]
        near = _scaled_copies(base, 60, 2.0 ** -10, g) + 1e-3 * torch.randn(60, d, generator=g) / d ** 0.5
        X[where] = near
    ds = B.Datastore.from_fp32(X.cuda(), scan_dtype)
    wi, wsc = oracle.retrieve_topk(Qm.numpy(), X.numpy(), k)
    spread = (wsc[:, 0] - wsc[:, -1]) / np.abs(wsc[:, 0])
    assert (spread < 2.0 ** -9).all()                       # the top 20 ARE packed that closely
    score_of = _score_fn(oracle, Qm.numpy(), X.numpy())
    for k_prime in (k, 0):
        ids, sc, c, mg = _run(B, ds, Qm, k, k_prime)
        exact, subs, total = check_topk(ids, sc, wi, wsc, score_of)
        assert c["unanswered"] == 0 and c["soft_certified"] + c["exact_pass"] == Q, c
        if k_prime == k:
            assert c["exact_pass"] == Q, c
            # the exact pass decides in the oracle's own precision: no substitutions at all
            assert np.array_equal(ids, wi) and np.array_equal(sc, wsc)


def test_squared_distance_metric_takes_the_exact_pass_too(B, oracle):
    from paper_2401_14021_amd import inputs
    g = torch.Generator().manual_seed(23)
    N, d, k = 20000, 128, 10
    X, _ = inputs.clustered_datastore(N, d, 16, seed=47, normalise=False)
    base = X[77].to(torch.bfloat16).float()
    where = torch.randperm(N, generator=g)[:80]
    X[where] = _scaled_copies(base, 80, 2.0 ** -10, g)
    Qm = torch.stack([base * 1.0005, X[9] + 0.05 * torch.randn(d, generator=g)])
    ds = B.Datastore.for_l2(X.cuda(), torch.bfloat16)
    ids, sc, c, mg = _run(B, ds, Qm, k, k)
    wi, wsc = oracle.retrieve_topk(Qm.numpy(), X.numpy(), k, metric="l2")
    assert np.array_equal(ids, wi) and np.array_equal(sc, wsc), (ids, wi, c)
    assert c["exact_pass"] == 2 and c["unanswered"] == 0, c


def test_fp16_keys_as_their_own_scan_copy(B, oracle):
    """KNN-LM style store (fp16 keys are the truth, only the query is rounded by the scan), k' = k:
    the exact pass reads fp16 rows."""
    from paper_2401_14021_amd import inputs
    N, d, Q, k = 30000, 1024, 5, 64
    keys, _ = inputs.knnlm_datastore(N, d, 16, seed=4)
    Qm = inputs.queries_near_rows(keys, inputs.pick_rows(N, Q, seed=8), seed=9, sigma=0.5)
    ds = B.Datastore(keys.cuda(), None)
    ids, sc, c, mg = _run(B, ds, Qm, k, k)
    wi, wsc = oracle.retrieve_topk(Qm.numpy(), keys.numpy(), k)
    assert c["exact_pass"] == Q and c["unanswered"] == 0, c
    assert np.array_equal(ids, wi) and np.array_equal(sc, wsc)


@pytest.mark.parametrize("store,d", [("f32", 64), ("f32", 200), ("f32", 384), ("f32", 96), ("f32", 2048),
                                     ("f16", 128), ("f16", 192), ("f16", 2048)])
def test_exact_pass_row_lengths_on_the_matrix_cores_and_beside_them(B, oracle, store, d):
    """k' = k sends every query to the exact pass: it runs on the fp64 matrix cores when a row is a
    whole number of 256-byte steps (d % 64 == 0 in fp32, d % 128 == 0 in fp16, up to 2048 elements)
    and on the vector units otherwise; 20 queries are more than one pass of 16 (or of 8) serves.
    Ids and scores must be the oracle's either way."""
    from paper_2401_14021_amd import inputs
    N, Q, k = 20000, 20, 10
    if store == "f16":
        X, _ = inputs.knnlm_datastore(N, d, 16, seed=d)
        ds = B.Datastore(X.cuda(), None)
        sigma = 0.5
    else:
        X, _ = inputs.clustered_datastore(N, d, 16, seed=d)
        ds = B.Datastore.from_fp32(X.cuda())
        sigma = 0.05
    Qm = inputs.queries_near_rows(X, inputs.pick_rows(N, Q, seed=3), seed=4, sigma=sigma)
    ids, sc, c, mg = _run(B, ds, Qm, k, k)
    wi, wsc = oracle.retrieve_topk(Qm.numpy(), X.numpy(), k)
    assert c["exact_pass"] == Q and c["unanswered"] == 0, c
    assert np.array_equal(ids, wi) and np.array_equal(sc, wsc)


def test_more_rows_reach_the_bound_than_a_list_holds(B, oracle):
    """100000 copies of one vector below the scan's resolution: the exact pass would have to
    collect far more than the 16384 rows a list holds.  Such a query is not answered wrongly: it
    comes back as id -1 / score NaN and is counted; the other query of the batch is unaffected."""
    from paper_2401_14021_amd import inputs
    g = torch.Generator().manual_seed(29)
    N, d, k, n_copies = 120000, 64, 20, 100000
    X, _ = inputs.clustered_datastore(N, d, 16, seed=53)
    base = X[11].to(torch.bfloat16).float()
    where = torch.randperm(N, generator=g)[:n_copies]
    X[where] = _scaled_copies(base, n_copies, 2.0 ** -10, g)
    free = torch.ones(N, dtype=torch.bool)
    free[where] = False
    other = int(torch.nonzero(free)[7])
    Qm = torch.stack([base, X[other] * 3 - base])
    wi, wsc = oracle.retrieve_topk(Qm.numpy(), X.numpy(), k)
    # precondition: all copies get the same scan score, so the scan keeps the 64 with the lowest
    # ids; count the rows that reach the exact rank-20 score among those 64
    kept = np.sort(where.numpy())[:64]
    s_all = oracle.scores(Qm[0].numpy(), X.numpy())
    bound = np.sort(s_all[kept])[::-1][k - 1]
    assert int((s_all >= bound).sum()) > 20000
    ds = B.Datastore.from_fp32(X.cuda())
    ids, sc, c, mg = _run(B, ds, Qm, k, 0)
    assert c["unanswered"] == 1 and c["exact_pass"] >= 1, c
    assert (ids[0] == -1).all() and np.isnan(sc[0]).all()
    score_of = _score_fn(oracle, Qm.numpy(), X.numpy())
    check_topk(ids[1:], sc[1:], wi[1:], wsc[1:], lambda i, r: score_of(i + 1, r))
    # the simple form reports it as an error instead of returning a wrong answer
    with pytest.raises(B.RalmError) as err:
        B.ralm_retrieve_topk(Qm.cuda(), X.cuda(), k)
    assert err.value.status == 9
    B.ralm_release_buffers()
