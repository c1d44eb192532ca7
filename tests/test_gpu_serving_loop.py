"""The whole of Alg. 1 on the library's entry points, against plain iterative retrieval.

The paper's central claim (Section 1, Section 3) is that speculation with batched verification and
rollback preserves the outputs: the documents a request ends up using are exactly those that
retrieval at every step would have given.  Here a deterministic stand-in for the language model
(the next query depends on the document used, so a wrong speculation really derails the context)
is driven twice: once retrieving at every step, once by the speculative loop - prefetch, cache
top-1 per step, batched verification, first mismatch, rollback, top-k cache update, stride from
the OS^3 scheduler - and the two document sequences must be identical."""
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


def _noise(r, t, d, dev):
    g = torch.Generator(device="cpu").manual_seed(1000003 * r + t)
    return torch.randn(d, generator=g).to(dev)


def _advance(q, doc_row, r, t):
    """Stand-in for one decoding step: the new context embedding depends on the document used."""
    v = q + 0.15 * doc_row + 0.04 * _noise(r, t, q.shape[0], q.device)
    return v / v.norm()


@pytest.mark.parametrize("baseline", ["oracle", "library"])
@pytest.mark.parametrize("asynchronous", [False, True])
def test_speculative_loop_preserves_the_document_sequence(B, oracle, asynchronous, baseline):
    """baseline = "oracle": the reference document sequence comes from the CPU oracle's retrieval
    at every step (parity evidence); "library": from the library's own retrieval at every step
    (the paper's output-preservation claim on the library alone)."""
    from paper_2401_14021_amd import inputs
    N, d, R, T, C, k, s_max = 20000, 64, 6, 20, 64, 5, 6
    X, _ = inputs.clustered_datastore(N, d, 24, seed=131)
    Xd = X.cuda()
    ds = B.Datastore.from_fp32(Xd)
    q0 = inputs.queries_near_rows(X, inputs.pick_rows(N, R, seed=132), seed=133).cuda()
    q0 = q0 / q0.norm(dim=1, keepdim=True)

    # ---- retrieval at every step ------------------------------------------------------------
    base_docs = np.zeros((R, T), dtype=np.int64)
    q = q0.clone()
    Xnp = X.numpy()
    for t in range(T):
        if baseline == "oracle":
            oi, _ = oracle.retrieve_topk(q.cpu().numpy(), Xnp, 1)
            ids = torch.from_numpy(oi).cuda()
        else:
            ids, _ = B.ralm_retrieve_topk_ex(q.contiguous(), ds, 1)
        base_docs[:, t] = ids[:, 0].cpu().numpy()
        q = torch.stack([_advance(q[r], Xd[ids[r, 0].long()], r, t) for r in range(R)])

    # ---- the speculative loop ---------------------------------------------------------------
    cache = torch.full((R, C), -1, dtype=torch.int32, device="cuda")
    clen = torch.zeros(R, dtype=torch.int32, device="cuda")
    head = torch.zeros(R, dtype=torch.int32, device="cuda")
    one = torch.arange(R + 1, dtype=torch.int64, device="cuda")
    ids, _ = B.ralm_retrieve_topk_ex(q0.contiguous(), ds, k)                  # prefetch (Alg. 1, before the loop)
    B.ralm_cache_insert(cache, clen, head, ids, one, N, p=k)
    state = [q0[r].clone() for r in range(R)]        # context at the next step to decode
    done = [[] for _ in range(R)]                     # documents used so far
    hist = [([], []) for _ in range(R)]               # (strides, matched) of recent verifications
    kb_calls = 1
    rounds = 0
    while min(len(x) for x in done) < T:
        rounds += 1
        strides = [B.ralm_os3_next_stride(hist[r][0][-5:], hist[r][1][-5:], [1.0], [4.0], s_max, 0.6, asynchronous)
                   for r in range(R)]
        # speculation: s_r steps per request from its cache, remembering query and context
        spec_q = [[] for _ in range(R)]
        spec_d = [[] for _ in range(R)]
        ctx = [state[r] for r in range(R)]
        for i in range(max(strides)):
            qs = torch.stack(ctx).contiguous()
            sid, _ = B.ralm_cache_lookup(cache, clen, qs, one, ds)
            for r in range(R):
                if i < strides[r]:
                    spec_q[r].append(ctx[r])
                    doc = int(sid[r])
                    spec_d[r].append(doc)
                    t = len(done[r]) + i
                    ctx[r] = _advance(ctx[r], Xd[doc], r, t) if doc >= 0 else ctx[r]
        # batched verification of all recorded queries, first mismatch per request
        off = torch.tensor(np.concatenate([[0], np.cumsum(strides)]), dtype=torch.int64, device="cuda")
        allq = torch.stack([v for r in range(R) for v in spec_q[r]]).contiguous()
        spec = torch.tensor([v for r in range(R) for v in spec_d[r]], dtype=torch.int32, device="cuda")
        true_ids, _ = B.ralm_retrieve_topk_ex(allq, ds, k)
        kb_calls += 1
        fm = B.ralm_verify(spec, true_ids, off, true_stride=k)
        B.ralm_cache_insert(cache, clen, head, true_ids, off, N, p=k, first_mismatch=fm)
        fm_h, true_h, off_h = fm.cpu().numpy(), true_ids[:, 0].cpu().numpy(), off.cpu().numpy()
        for r in range(R):
            m, s = int(fm_h[r]), strides[r]
            t0 = len(done[r])
            done[r] += spec_d[r][:m]                               # the matched prefix stands
            if m < s:                                              # roll back to step m, redo it with the true document
                doc = int(true_h[off_h[r] + m])
                done[r].append(doc)
                state[r] = _advance(spec_q[r][m], Xd[doc], r, t0 + m)
            else:
                state[r] = ctx[r]
            hist[r][0].append(s)
            hist[r][1].append(m)
    got = np.array([x[:T] for x in done])
    assert np.array_equal(got, base_docs)
    # speculation paid off: far fewer knowledge-base calls than steps, and strides grew beyond 1
    assert kb_calls < T
    assert max(max(h[0]) for h in hist) > 1
