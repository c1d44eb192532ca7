"""Seeded synthetic inputs shaped like the paper's retrieval workloads.

This module only *draws* inputs (datastores, queries, speculation caches,
stride mixes).  It contains none of the method's arithmetic: no inner-product
scoring, no selection, no compare.  Both the HIP path and the CPU oracle are
handed the bytes produced here; neither regenerates them on its own.

The paper evaluates on a Wikipedia passage index with dense passage-retriever
embeddings and on a WikiText-103 KNN-LM datastore (Section 5.1 "Datasets" and
"Retrievers"); those corpora are not available offline, so clustered Gaussian
datastores of the same shapes stand in for them:

* dense-retriever style: ``n_clusters`` centres ~ N(0, I); each row is its
  centre plus N(0, 0.3^2 I), L2-normalised; queries are a datastore row plus
  N(0, 0.05^2 I) noise (not renormalised unless a drift step says so);
* KNN-LM style: keys are a centre ~ N(0, I) plus N(0, 0.5^2 I), stored in
  fp16, not normalised; values are token ids in [0, 50000).

Everything is a pure function of (shape, seed, chunk size); generation runs on
whatever torch device is asked for, in fixed-size row chunks so that a
21M x 768 or 100M x 1024 datastore never needs a second full-size temporary.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import torch

ROW_CHUNK = 1 << 18  # rows drawn per generator call; part of the recipe


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def cluster_centres(n_clusters: int, d: int, seed: int, device="cpu") -> torch.Tensor:
    """Centres ~ N(0, I), fp32 [n_clusters, d]."""
    return torch.randn(n_clusters, d, generator=_gen(device, seed), device=device,
                       dtype=torch.float32)


ROW_ORDERS = ("iid", "cluster", "corpus")
CORPUS_RUN = 32  # mean length of a run of rows that share a cluster in "corpus" order


def _assignments(n: int, r0: int, N: int, n_clusters: int, order: str, g: torch.Generator, device) -> torch.Tensor:
    """Cluster of each of the rows r0 .. r0+n-1 (int64) for the given row order."""
    if order == "iid":
        return torch.randint(0, n_clusters, (n,), generator=g, device=device)
    if order == "cluster":
        # rows sorted by cluster, clusters of (nearly) equal size
        j = torch.arange(r0, r0 + n, device=device, dtype=torch.int64)
        return (j * n_clusters) // N
    if order == "corpus":
        # runs of geometric length (mean CORPUS_RUN) of one cluster each, as consecutive passages
        # of a document or consecutive tokens of a text are near each other
        start = torch.rand(n, generator=g, device=device) < (1.0 / CORPUS_RUN)
        start[0] = True
        run = torch.cumsum(start.to(torch.int64), 0) - 1
        of_run = torch.randint(0, n_clusters, (int(run[-1]) + 1,), generator=g, device=device)
        return of_run[run]
    raise ValueError(f"row order {order!r} not in {ROW_ORDERS}")


def clustered_datastore(N: int, d: int, n_clusters: int, seed: int, *, sigma: float = 0.3,
                        normalise: bool = True, device="cpu",
                        out: Optional[torch.Tensor] = None,
                        dtype: torch.dtype = torch.float32, order: str = "iid"
                        ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Rows = centre[assign] + N(0, sigma^2 I), optionally L2-normalised.

    Returns (X [N, d] of ``dtype``, assign [N] int32).  ``order``: "iid" - rows in
    random cluster order (assign is iid uniform), so any prefix or strided subset of
    the datastore is an unbiased sample of it; "cluster" - rows sorted by cluster;
    "corpus" - runs of about 32 consecutive rows share a cluster (spatial locality of
    a datastore stored in corpus order, which the paper's next-n cache update for
    KNN-LM relies on, Section 5.3).
    """
    centres = cluster_centres(n_clusters, d, seed, device)
    if out is None:
        out = torch.empty(N, d, dtype=dtype, device=device)
    assert out.shape == (N, d) and out.dtype == dtype
    assign = torch.empty(N, dtype=torch.int32, device=device)
    for ci, r0 in enumerate(range(0, N, ROW_CHUNK)):
        r1 = min(N, r0 + ROW_CHUNK)
        g = _gen(device, seed * 1000003 + 17 + ci)
        a = _assignments(r1 - r0, r0, N, n_clusters, order, g, device)
        x = torch.randn(r1 - r0, d, generator=g, device=device, dtype=torch.float32)
        x.mul_(sigma).add_(centres[a])
        if normalise:
            x.div_(x.norm(dim=1, keepdim=True).clamp_min_(1e-30))
        out[r0:r1].copy_(x)
        assign[r0:r1] = a.to(torch.int32)
    return out, assign


def queries_near_rows(X: torch.Tensor, rows: torch.Tensor, seed: int, *,
                      sigma: float = 0.05) -> torch.Tensor:
    """q_i = fp32(X[rows[i]]) + N(0, sigma^2 I); fp32 [len(rows), d]."""
    dev = X.device
    base = X[rows.to(dev).long()].to(torch.float32)
    noise = torch.randn(base.shape, generator=_gen(dev, seed), device=dev, dtype=torch.float32)
    return (base + sigma * noise).contiguous()


def drift_queries(q: torch.Tensor, seed: int, *, sigma: float = 0.02) -> torch.Tensor:
    """One step of the stress loop's query drift: normalise(q + N(0, sigma^2 I))."""
    noise = torch.randn(q.shape, generator=_gen(q.device, seed), device=q.device,
                        dtype=torch.float32)
    qn = q + sigma * noise
    return (qn / qn.norm(dim=1, keepdim=True).clamp_min(1e-30)).contiguous()


def pick_rows(N: int, n: int, seed: int, device="cpu") -> torch.Tensor:
    """n row ids iid uniform in [0, N), int64."""
    return torch.randint(0, N, (n,), generator=_gen(device, seed), device=device)


def stride_offsets(strides: List[int]) -> torch.Tensor:
    """CSR offsets (int64 [R+1]) of a list of per-request speculation strides."""
    off = [0]
    for s in strides:
        off.append(off[-1] + int(s))
    return torch.tensor(off, dtype=torch.int64)


def uniform_strides(R: int, lo: int, hi: int, seed: int) -> List[int]:
    """Per-request strides iid uniform in {lo..hi}, drawn once per request."""
    return torch.randint(lo, hi + 1, (R,), generator=_gen("cpu", seed)).tolist()


def speculation_caches(N: int, R: int, C: int, q_offsets: torch.Tensor,
                       source_rows: torch.Tensor, assign: Optional[torch.Tensor],
                       seed: int, *, p_hit: float = 0.5, fill: Optional[int] = None
                       ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per-request caches of datastore row ids (CPU tensors).

    A cache sampled uniformly from a large datastore would almost never contain
    a query's true top-1, so each request's cache is built as: for each of the
    request's queries, its source row id with probability ``p_hit``; then
    filler ids up to ``fill`` entries (default: the capacity C), half drawn
    from rows sharing a cluster with one of the request's source rows (when
    ``assign`` is given and such rows are cheap to find) and half uniformly
    from the whole datastore.  Duplicates are allowed (the lookup is
    id-based, so they are harmless).

    Returns (cache_ids int32 [R, C] padded with -1, cache_len int32 [R]).
    """
    g = _gen("cpu", seed)
    fill = C if fill is None else min(fill, C)
    ids = torch.full((R, C), -1, dtype=torch.int32)
    lens = torch.zeros(R, dtype=torch.int32)
    src = source_rows.cpu().long()
    off = q_offsets.cpu().long()
    assign_cpu = assign.cpu() if assign is not None else None
    for r in range(R):
        mine = src[off[r]:off[r + 1]]
        keep = torch.rand(len(mine), generator=g) < p_hit
        entries = [mine[keep]]
        n_have = int(keep.sum())
        n_fill = max(0, fill - n_have)
        n_near = n_fill // 2 if (assign_cpu is not None and len(mine) > 0) else 0
        if n_near > 0:
            # neighbours in id space that share the cluster of a source row: scan a
            # window of ids after the source row (cheap; no global index needed)
            pool = []
            for m in mine.tolist():
                lo = (m + 1) % N
                hi = min(N, lo + 64 * n_near)
                win = torch.arange(lo, hi)
                same = win[assign_cpu[lo:hi] == assign_cpu[m]]
                pool.append(same)
            pool = torch.cat(pool) if pool else torch.empty(0, dtype=torch.long)
            if len(pool) > n_near:
                sel = torch.randperm(len(pool), generator=g)[:n_near]
                pool = pool[sel]
            entries.append(pool)
            n_have += len(pool)
        n_uni = max(0, fill - n_have)
        entries.append(torch.randint(0, N, (n_uni,), generator=g))
        e = torch.cat(entries)[:C]
        e = e[torch.randperm(len(e), generator=g)]
        ids[r, :len(e)] = e.to(torch.int32)
        lens[r] = len(e)
    return ids, lens


def knnlm_datastore(N: int, d: int, n_clusters: int, seed: int, *, sigma: float = 0.5,
                    vocab: int = 50000, device="cpu",
                    out: Optional[torch.Tensor] = None, order: str = "iid"
                    ) -> Tuple[torch.Tensor, torch.Tensor]:
    """KNN-LM style datastore: fp16 keys [N, d] (centre + N(0, sigma^2 I), raw, not
    normalised) and int32 values [N] in [0, vocab)."""
    keys, _ = clustered_datastore(N, d, n_clusters, seed, sigma=sigma, normalise=False,
                                  device=device, out=out, dtype=torch.float16, order=order)
    vals = torch.randint(0, vocab, (N,), generator=_gen(device, seed + 99), device=device,
                         dtype=torch.int32)
    return keys, vals


@dataclasses.dataclass
class Workload:
    """One named configuration (shapes only; tensors are drawn by the functions above)."""
    name: str
    N: int
    d: int
    n_clusters: int
    k: int
    k_prime: int
    scan_dtype: str        # "bf16" | "f16" | "f32"
    exact_dtype: str       # "f32" | "f16"
    cache_C: int = 0
    seed: int = 0


WORKLOADS = {
    # tiny exact retrieval: 1 request, stride 3, k=1, 64-entry cache
    "tiny": Workload("tiny", 100_000, 768, 256, 1, 64, "bf16", "f32", 64, 0xC1),
    # medium batched verification: 16 requests x stride {1,2,4,8}, k=5, 1024-entry caches
    "medium": Workload("medium", 1_000_000, 768, 4096, 5, 64, "bf16", "f32", 1024, 0xC2),
    # dense-retriever scale: Q swept {1,8,64,256,1024}, k in {1,20}, k'=64
    "dense21m": Workload("dense21m", 21_000_000, 768, 65536, 20, 64, "bf16", "f32", 0, 0xC3),
    # KNN-LM datastore: fp16 keys are the truth, k=1024
    "knnlm100m": Workload("knnlm100m", 100_000_000, 1024, 8192, 1024, 2048, "f16", "f16", 0, 0xC4),
    # speculation loop stress: 512 requests, 4096-entry caches, stride U{1..8}
    "specloop": Workload("specloop", 21_000_000, 768, 65536, 1, 64, "bf16", "f32", 4096, 0xC5),
}
