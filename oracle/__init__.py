"""Python face of the CPU oracle (``ralm_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the HIP package
and shares no code with it.  All arrays are numpy, on the host.

What each function computes is stated in the C file; this wrapper only checks
shapes, builds the shared object with gcc when it is missing, and provides the
chunk-streaming form of the same brute-force retrieval for datastores that do
not fit in host memory at once (scores of every row of every chunk, then a full
sort of carry + chunk by (score descending, id ascending)).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Iterable, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ralm_oracle.c")
_LIB = os.path.join(_HERE, "libralm_oracle.so")

F32, BF16, F16 = 0, 1, 2
# inner product; minus the squared Euclidean distance; inner product accumulated the other plausible
# way (products and running sum rounded to fp32, left to right), for counting reading-dependent answers
METRICS = {"ip": 0, "l2": 1, "ip_f32_sequential": 2}
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP for row-level threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.ralm_oracle_threads.restype = ctypes.c_int
        L.ralm_oracle_scores.argtypes = [vp, vp, ctypes.c_int, i64, i32, i64, vp]
        L.ralm_oracle_scores.restype = None
        L.ralm_oracle_retrieve_topk.argtypes = [vp, i64, vp, ctypes.c_int, i64, i32, i64, i32, vp, vp]
        L.ralm_oracle_retrieve_topk.restype = ctypes.c_int
        L.ralm_oracle_cache_lookup.argtypes = [vp, vp, i32, i64, vp, vp, vp, ctypes.c_int, i64, i32,
                                               i64, vp, vp]
        L.ralm_oracle_cache_lookup.restype = ctypes.c_int
        L.ralm_oracle_scores_metric.argtypes = [vp, vp, ctypes.c_int, i64, i32, i64, ctypes.c_int, vp]
        L.ralm_oracle_scores_metric.restype = None
        L.ralm_oracle_retrieve_topk_metric.argtypes = [vp, i64, vp, ctypes.c_int, i64, i32, i64, i32, ctypes.c_int,
                                                       vp, vp]
        L.ralm_oracle_retrieve_topk_metric.restype = ctypes.c_int
        L.ralm_oracle_cache_lookup_metric.argtypes = [vp, vp, i32, i64, vp, vp, vp, ctypes.c_int, i64, i32, i64,
                                                      ctypes.c_int, vp, vp]
        L.ralm_oracle_cache_lookup_metric.restype = ctypes.c_int
        L.ralm_oracle_cache_lookup_topk.argtypes = [vp, vp, i32, i64, vp, vp, vp, ctypes.c_int, i64, i32, i64,
                                                    ctypes.c_int, i32, vp, vp]
        L.ralm_oracle_cache_lookup_topk.restype = ctypes.c_int
        L.ralm_oracle_verify.argtypes = [vp, vp, i64, vp, i64, vp]
        L.ralm_oracle_verify.restype = None
        L.ralm_oracle_cache_insert.argtypes = [vp, vp, vp, i32, i64, vp, i64, vp, vp, i32, i32, i64]
        L.ralm_oracle_cache_insert.restype = None
        dbl = ctypes.c_double
        L.ralm_oracle_os3_expected_verified.argtypes = [dbl, i32]
        L.ralm_oracle_os3_expected_verified.restype = dbl
        L.ralm_oracle_os3_objective.argtypes = [dbl, dbl, dbl, i32, i32]
        L.ralm_oracle_os3_objective.restype = dbl
        L.ralm_oracle_os3_stride.argtypes = [dbl, dbl, dbl, i32, i32]
        L.ralm_oracle_os3_stride.restype = i32
        L.ralm_oracle_os3_gamma.argtypes = [vp, vp, i32, dbl]
        L.ralm_oracle_os3_gamma.restype = dbl
        L.ralm_oracle_os3_latency.argtypes = [vp, i32]
        L.ralm_oracle_os3_latency.restype = dbl
        L.ralm_oracle_knnlm_probs.argtypes = [vp, vp, i64, i32, vp, dbl, vp, vp, vp, vp]
        L.ralm_oracle_knnlm_probs.restype = None
        _lib = L
    return _lib


def threads() -> int:
    return int(_load().ralm_oracle_threads())


def _store(X: np.ndarray) -> Tuple[np.ndarray, int]:
    """Accept fp32, fp16, or bf16-as-uint16 (pass dtype tag explicitly for bf16)."""
    if X.dtype == np.float32:
        return np.ascontiguousarray(X), F32
    if X.dtype == np.float16:
        return np.ascontiguousarray(X), F16
    raise TypeError(f"datastore dtype {X.dtype} not supported (use float32/float16, or bf16_store())")


class bf16_store:
    """Wrap a uint16 array holding bf16 bit patterns."""

    def __init__(self, bits: np.ndarray):
        assert bits.dtype == np.uint16
        self.bits = np.ascontiguousarray(bits)


def _store_any(X):
    if isinstance(X, bf16_store):
        return X.bits, BF16
    return _store(X)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def scores(q: np.ndarray, X, metric: str = "ip") -> np.ndarray:
    """All scores of ONE query with the rows of X; fp32 [n]."""
    Xa, tag = _store_any(X)
    q = np.ascontiguousarray(q, dtype=np.float32)
    n, d = Xa.shape
    assert q.shape == (d,)
    out = np.empty(n, dtype=np.float32)
    _load().ralm_oracle_scores_metric(_ptr(q), _ptr(Xa), tag, n, d, d, METRICS[metric], _ptr(out))
    return out


def retrieve_topk(queries: np.ndarray, X, k: int, metric: str = "ip") -> Tuple[np.ndarray, np.ndarray]:
    """Exact top-k of every query over the whole datastore: (ids int32 [Q,k], scores fp32 [Q,k])."""
    Xa, tag = _store_any(X)
    queries = np.ascontiguousarray(queries, dtype=np.float32)
    Q, d = queries.shape
    N, d2 = Xa.shape
    assert d == d2
    ids = np.empty((Q, k), dtype=np.int32)
    sc = np.empty((Q, k), dtype=np.float32)
    rc = _load().ralm_oracle_retrieve_topk_metric(_ptr(queries), Q, _ptr(Xa), tag, N, d, d, k, METRICS[metric],
                                                  _ptr(ids), _ptr(sc))
    if rc != 0:
        raise ValueError("oracle retrieve_topk: bad arguments")
    return ids, sc


def retrieve_topk_stream(queries: np.ndarray, chunks: Iterable[Tuple[int, object]], k: int,
                         metric: str = "ip") -> Tuple[np.ndarray, np.ndarray]:
    """Same result as ``retrieve_topk`` for a datastore delivered as (base_row, rows) chunks.

    Per query a carry list of the best k (score, id) pairs so far is kept; for
    each chunk all of its scores are computed, carry + chunk is sorted by
    (score descending, id ascending) and cut to k.  Once the carry holds k
    pairs, a row of the chunk whose score is below the carry's k-th score
    cannot be among the first k of that sort (k pairs rank before it), so such
    rows are left out of the sort; rows that tie with the k-th score stay in,
    the id decides.  Chunks may come in any order.
    """
    queries = np.ascontiguousarray(queries, dtype=np.float32)
    Q = queries.shape[0]
    carry_s = [np.empty(0, np.float32) for _ in range(Q)]
    carry_i = [np.empty(0, np.int64) for _ in range(Q)]
    for base, rows in chunks:
        n = (rows.bits if isinstance(rows, bf16_store) else rows).shape[0]
        ids_here = np.arange(base, base + n, dtype=np.int64)
        for i in range(Q):
            here_s = scores(queries[i], rows, metric)
            here_i = ids_here
            if carry_s[i].shape[0] == k:
                may_enter = here_s >= carry_s[i][k - 1]
                here_s, here_i = here_s[may_enter], here_i[may_enter]
            s = np.concatenate([carry_s[i], here_s])
            j = np.concatenate([carry_i[i], here_i])
            order = np.lexsort((j, -s.astype(np.float64)))[:k]
            carry_s[i], carry_i[i] = s[order], j[order]
    ids = np.stack([c.astype(np.int32) for c in carry_i])
    sc = np.stack(carry_s)
    return ids, sc


def cache_lookup(cache_ids: np.ndarray, cache_len: np.ndarray, queries: np.ndarray,
                 q_offsets: np.ndarray, X, metric: str = "ip") -> Tuple[np.ndarray, np.ndarray]:
    """Speculative top-1 of each query over its request's cached row ids."""
    Xa, tag = _store_any(X)
    cache_ids = np.ascontiguousarray(cache_ids, dtype=np.int32)
    cache_len = np.ascontiguousarray(cache_len, dtype=np.int32)
    queries = np.ascontiguousarray(queries, dtype=np.float32)
    q_offsets = np.ascontiguousarray(q_offsets, dtype=np.int64)
    R, C = cache_ids.shape
    N, d = Xa.shape
    Qt = int(q_offsets[-1]) if R > 0 else 0
    assert queries.shape == (Qt, d) and q_offsets.shape == (R + 1,)
    ids = np.empty(Qt, dtype=np.int32)
    sc = np.empty(Qt, dtype=np.float32)
    rc = _load().ralm_oracle_cache_lookup_metric(_ptr(cache_ids), _ptr(cache_len), C, R, _ptr(queries),
                                                 _ptr(q_offsets), _ptr(Xa), tag, N, d, d, METRICS[metric],
                                                 _ptr(ids), _ptr(sc))
    if rc != 0:
        raise ValueError("oracle cache_lookup: bad arguments")
    return ids, sc


def verify(spec_ids: np.ndarray, true_ids: np.ndarray, q_offsets: np.ndarray,
           true_stride: int = 1) -> np.ndarray:
    """First mismatch per request (0-based; the stride itself when all match)."""
    spec_ids = np.ascontiguousarray(spec_ids, dtype=np.int32)
    true_ids = np.ascontiguousarray(true_ids, dtype=np.int32)
    q_offsets = np.ascontiguousarray(q_offsets, dtype=np.int64)
    R = q_offsets.shape[0] - 1
    out = np.empty(R, dtype=np.int32)
    _load().ralm_oracle_verify(_ptr(spec_ids), _ptr(true_ids), true_stride, _ptr(q_offsets), R, _ptr(out))
    return out


def cache_insert(cache_ids: np.ndarray, cache_len: np.ndarray, cache_head: np.ndarray,
                 true_ids: np.ndarray, q_offsets: np.ndarray, N: int, p: int = 1, n_next: int = 0,
                 first_mismatch=None, true_stride: int = None):
    """Cache update after a verification step; returns new (cache_ids, cache_len, cache_head).

    ``true_ids`` is [Qt, k] (or flat with ``true_stride``); ranks 0..p-1 of every taken step are
    inserted (their n_next successors instead when n_next > 0)."""
    cache_ids = np.array(cache_ids, dtype=np.int32, order="C", copy=True)
    cache_len = np.array(cache_len, dtype=np.int32, copy=True)
    cache_head = np.array(cache_head, dtype=np.int32, copy=True)
    R, C = cache_ids.shape
    true_ids = np.ascontiguousarray(true_ids, dtype=np.int32)
    if true_stride is None:
        true_stride = true_ids.shape[1] if true_ids.ndim == 2 else 1
    assert 1 <= p <= true_stride
    q_offsets = np.ascontiguousarray(q_offsets, dtype=np.int64)
    assert q_offsets.shape[0] == R + 1
    fm = None if first_mismatch is None else np.ascontiguousarray(first_mismatch, dtype=np.int32)
    _load().ralm_oracle_cache_insert(_ptr(cache_ids), _ptr(cache_len), _ptr(cache_head), C, R, _ptr(true_ids),
                                     true_stride, _ptr(q_offsets), None if fm is None else _ptr(fm), p, n_next, N)
    return cache_ids, cache_len, cache_head


def os3_expected_verified(gamma: float, s: int) -> float:
    return float(_load().ralm_oracle_os3_expected_verified(gamma, s))


def os3_objective(gamma: float, a: float, b: float, s: int, asynchronous: bool = False) -> float:
    return float(_load().ralm_oracle_os3_objective(gamma, a, b, s, 1 if asynchronous else 0))


def os3_stride(gamma: float, a: float, b: float, s_max: int, asynchronous: bool = False) -> int:
    return int(_load().ralm_oracle_os3_stride(gamma, a, b, s_max, 1 if asynchronous else 0))


def os3_gamma(strides, matched, gamma_max: float = 0.6) -> float:
    st = np.ascontiguousarray(strides, dtype=np.int32)
    m = np.ascontiguousarray(matched, dtype=np.int32)
    assert st.shape == m.shape
    return float(_load().ralm_oracle_os3_gamma(_ptr(st), _ptr(m), st.shape[0], gamma_max))


def knnlm_probs(ids: np.ndarray, scores: np.ndarray, values: np.ndarray, temperature: float = 1.0):
    """Neighbour distribution of KNN-LM: (tokens [Q,k], weights [Q,k], top_token [Q], top_prob [Q])."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    values = np.ascontiguousarray(values, dtype=np.int32)
    Q, k = ids.shape
    assert scores.shape == (Q, k) and temperature > 0
    tokens = np.empty((Q, k), dtype=np.int32)
    weights = np.empty((Q, k), dtype=np.float32)
    top_token = np.empty(Q, dtype=np.int32)
    top_prob = np.empty(Q, dtype=np.float32)
    _load().ralm_oracle_knnlm_probs(_ptr(ids), _ptr(scores), Q, k, _ptr(values), float(temperature),
                                    _ptr(tokens), _ptr(weights), _ptr(top_token), _ptr(top_prob))
    return tokens, weights, top_token, top_prob


def os3_latency(samples) -> float:
    a = np.ascontiguousarray(samples, dtype=np.float64)
    return float(_load().ralm_oracle_os3_latency(_ptr(a), a.shape[0]))


def cache_lookup_topk(cache_ids: np.ndarray, cache_len: np.ndarray, queries: np.ndarray, q_offsets: np.ndarray,
                      X, k: int, metric: str = "ip") -> Tuple[np.ndarray, np.ndarray]:
    """The k best cached entries of each query's request: (ids [Qt,k], scores [Qt,k]); -1 / -inf padding."""
    Xa, tag = _store_any(X)
    cache_ids = np.ascontiguousarray(cache_ids, dtype=np.int32)
    cache_len = np.ascontiguousarray(cache_len, dtype=np.int32)
    queries = np.ascontiguousarray(queries, dtype=np.float32)
    q_offsets = np.ascontiguousarray(q_offsets, dtype=np.int64)
    R, C = cache_ids.shape
    N, d = Xa.shape
    Qt = int(q_offsets[-1]) if R > 0 else 0
    assert queries.shape == (Qt, d) and q_offsets.shape == (R + 1,)
    ids = np.empty((Qt, k), dtype=np.int32)
    sc = np.empty((Qt, k), dtype=np.float32)
    rc = _load().ralm_oracle_cache_lookup_topk(_ptr(cache_ids), _ptr(cache_len), C, R, _ptr(queries), _ptr(q_offsets),
                                               _ptr(Xa), tag, N, d, d, METRICS[metric], k, _ptr(ids), _ptr(sc))
    if rc != 0:
        raise ValueError("oracle cache_lookup_topk: bad arguments")
    return ids, sc
