"""Thin ctypes binding over ``libralm.so`` (C ABI in ``include/ralm.h``).

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the path runs inside the library's kernels.  The
functions have the names of the C entry points.  There is no CPU fallback: if
the shared object is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RALM_LIB_PATH") or os.path.join(_HERE, "libralm.so")

RALM_F32, RALM_BF16, RALM_F16 = 0, 1, 2
RALM_METRIC_IP, RALM_METRIC_L2 = 0, 1
_DT = {torch.float32: RALM_F32, torch.bfloat16: RALM_BF16, torch.float16: RALM_F16}

STATUS = {0: "RALM_OK", 1: "RALM_ERR_NULL", 2: "RALM_ERR_SHAPE", 3: "RALM_ERR_K", 4: "RALM_ERR_DTYPE",
          5: "RALM_ERR_ALIGN", 6: "RALM_ERR_WORKSPACE", 7: "RALM_ERR_RANGE", 8: "RALM_ERR_DEVICE",
          9: "RALM_ERR_OVERFLOW"}


class ralm_datastore_t(ctypes.Structure):
    _fields_ = [("exact", ctypes.c_void_p), ("exact_dtype", ctypes.c_int32),
                ("scan", ctypes.c_void_p), ("scan_dtype", ctypes.c_int32),
                ("N", ctypes.c_int64), ("d", ctypes.c_int32),
                ("exact_stride", ctypes.c_int64), ("scan_stride", ctypes.c_int64),
                ("metric", ctypes.c_int32)]


class ralm_counters_t(ctypes.Structure):
    _fields_ = [("unanswered", ctypes.c_int32), ("ladder_overflows", ctypes.c_int32),
                ("hard_certified", ctypes.c_int32), ("soft_certified", ctypes.c_int32),
                ("exact_pass", ctypes.c_int32)]


class RalmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS.get(status, status)}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libralm.so (built in-tree by ``python -m paper_2401_14021_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2401_14021_amd.build`; "
                "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        dsp = ctypes.POINTER(ralm_datastore_t)
        L.ralm_last_error.restype = ctypes.c_char_p
        L.ralm_retrieve_topk.argtypes = [vp, i64, vp, i64, i32, i32, vp, vp]
        L.ralm_workspace_bytes.argtypes = [i64, dsp, i32, i32]
        L.ralm_workspace_bytes.restype = ctypes.c_size_t
        L.ralm_retrieve_topk_ex.argtypes = [vp, i64, dsp, i32, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ralm_retrieve_topk_seq.argtypes = L.ralm_retrieve_topk_ex.argtypes
        L.ralm_workspace_overflows.argtypes = [vp, vp, ctypes.POINTER(i32)]
        L.ralm_workspace_counters.argtypes = [vp, vp, ctypes.POINTER(ralm_counters_t)]
        L.ralm_workspace_stage_entries.argtypes = [vp, vp, ctypes.POINTER(i32), ctypes.POINTER(i64)]
        L.ralm_build_scan_copy.argtypes = [vp, i64, vp, i32, i64, i64, i32, vp]
        L.ralm_build_scan_copy_l2.argtypes = [vp, i32, i64, vp, i32, i64, i64, i32, vp]
        L.ralm_cache_lookup.argtypes = [vp, vp, i32, i64, vp, i64, vp, dsp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ralm_cache_lookup_static.argtypes = [vp, vp, i32, i64, vp, i64, vp, dsp, vp, vp, vp]
        L.ralm_cache_lookup_workspace_bytes.argtypes = [i64]
        L.ralm_cache_lookup_workspace_bytes.restype = ctypes.c_size_t
        L.ralm_cache_lookup_topk.argtypes = [vp, vp, i32, i64, vp, i64, vp, dsp, i32, vp, vp, vp, ctypes.c_size_t, vp]
        L.ralm_cache_lookup_topk_workspace_bytes.argtypes = [i64, i32]
        L.ralm_cache_lookup_topk_workspace_bytes.restype = ctypes.c_size_t
        L.ralm_verify.argtypes = [vp, vp, i64, i64, vp, i64, vp, vp]
        L.ralm_cache_insert.argtypes = [vp, vp, vp, i32, i64, vp, i64, i64, vp, vp, i32, i32, i64, vp]
        L.ralm_knnlm_probs.argtypes = [vp, vp, i64, i32, vp, i64, ctypes.c_float, vp, vp, vp, vp, vp]
        L.ralm_os3_gamma.argtypes = [vp, vp, i32, ctypes.c_double]
        L.ralm_os3_gamma.restype = ctypes.c_double
        L.ralm_os3_objective.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double, i32, i32]
        L.ralm_os3_objective.restype = ctypes.c_double
        L.ralm_os3_stride.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double, i32, i32]
        L.ralm_os3_stride.restype = i32
        L.ralm_os3_latency.argtypes = [vp, i32]
        L.ralm_os3_latency.restype = ctypes.c_double
        L.ralm_os3_next_stride.argtypes = [vp, vp, i32, vp, i32, vp, i32, ctypes.c_double, i32, i32]
        L.ralm_os3_next_stride.restype = i32
        L.ralm_release_buffers.argtypes = []
        L.ralm_release_buffers.restype = None
        L.ralm_scan_reserve_cus.argtypes = [i32]
        L.ralm_scan_reserve_cus.restype = None
        L.ralm_profile_enable.argtypes = [i32]
        L.ralm_profile_enable.restype = None
        L.ralm_profile_scan_ms.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        for name in ("ralm_retrieve_topk", "ralm_retrieve_topk_ex", "ralm_retrieve_topk_seq", "ralm_workspace_overflows",
                     "ralm_workspace_counters", "ralm_workspace_stage_entries",
                     "ralm_build_scan_copy", "ralm_build_scan_copy_l2", "ralm_cache_lookup", "ralm_cache_lookup_static",
                     "ralm_cache_lookup_topk", "ralm_verify", "ralm_cache_insert", "ralm_knnlm_probs",
                     "ralm_profile_scan_ms"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise RalmError(status, lib().ralm_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Datastore:
    """Holds the exact copy and (optionally) the low-precision scan copy of the keys."""

    def __init__(self, exact: torch.Tensor, scan: Optional[torch.Tensor] = None, metric: int = RALM_METRIC_IP):
        assert exact.dim() == 2 and exact.stride(1) == 1
        self.exact, self.scan = exact, scan
        self.N, self.d = exact.shape
        self.desc = ralm_datastore_t()
        self.desc.metric = metric
        self.desc.exact = exact.data_ptr()
        self.desc.exact_dtype = _DT[exact.dtype]
        self.desc.exact_stride = exact.stride(0)
        self.desc.N, self.desc.d = self.N, self.d
        if scan is not None:
            extra = 8 if metric == RALM_METRIC_L2 else 0
            assert scan.shape == (self.N, self.d + extra) and scan.stride(1) == 1
            self.desc.scan = scan.data_ptr()
            self.desc.scan_dtype = _DT[scan.dtype]
            self.desc.scan_stride = scan.stride(0)
        else:
            self.desc.scan = None
            self.desc.scan_dtype = self.desc.exact_dtype
            self.desc.scan_stride = 0

    @classmethod
    def from_fp32(cls, exact: torch.Tensor, scan_dtype: torch.dtype = torch.bfloat16,
                  row_chunk: int = 1 << 20) -> "Datastore":
        """Build the scan copy with the library's own rounding kernel."""
        scan = torch.empty(exact.shape, dtype=scan_dtype, device=exact.device)
        ralm_build_scan_copy(exact, scan)
        return cls(exact, scan)


    @classmethod
    def for_l2(cls, exact: torch.Tensor, scan_dtype: Optional[torch.dtype] = None) -> "Datastore":
        """Squared-distance metric: builds the [N, d + 8] scan copy (rounded row + its squared norm)."""
        if scan_dtype is None:
            scan_dtype = torch.float16 if exact.dtype == torch.float16 else torch.bfloat16
        N, d = exact.shape
        pitch = (d + 8 + 63) // 64 * 64          # rows start on 128-byte lines
        scan = torch.empty(N, pitch, dtype=scan_dtype, device=exact.device)[:, :d + 8]
        _check(lib().ralm_build_scan_copy_l2(exact.data_ptr(), _DT[exact.dtype], exact.stride(0), scan.data_ptr(),
                                             _DT[scan_dtype], scan.stride(0), N, d, _stream()))
        return cls(exact, scan, RALM_METRIC_L2)


def ralm_build_scan_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    assert src.dtype == torch.float32 and src.shape == dst.shape
    N, d = src.shape
    _check(lib().ralm_build_scan_copy(src.data_ptr(), src.stride(0), dst.data_ptr(), _DT[dst.dtype],
                                      dst.stride(0), N, d, _stream()))


def ralm_workspace_bytes(Q: int, ds: Datastore, k: int, k_prime: int = 0) -> int:
    n = lib().ralm_workspace_bytes(Q, ctypes.byref(ds.desc), k, k_prime)
    if n == 0:
        raise RalmError(-1, "ralm_workspace_bytes: bad arguments")
    return int(n)


def alloc_workspace(Q: int, ds: Datastore, k: int, k_prime: int = 0) -> torch.Tensor:
    n = ralm_workspace_bytes(Q, ds, k, k_prime)
    return torch.empty(n + 256, dtype=torch.uint8, device=ds.exact.device)


def _ws_view(ws: torch.Tensor) -> Tuple[int, int]:
    base = ws.data_ptr()
    aligned = (base + 255) & ~255
    return aligned, ws.numel() - (aligned - base)


def ralm_retrieve_topk_ex(queries: torch.Tensor, ds: Datastore, k: int, k_prime: int = 0,
                          workspace: Optional[torch.Tensor] = None,
                          out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None,
                          out_margin: Optional[torch.Tensor] = None, sequential: bool = False
                          ) -> Tuple[torch.Tensor, torch.Tensor]:
    """sequential=True calls ralm_retrieve_topk_seq (same arguments, block-by-block ladder)."""
    assert queries.dtype == torch.float32 and queries.is_contiguous()
    Q = queries.shape[0]
    dev = queries.device
    if workspace is None:
        workspace = alloc_workspace(Q, ds, k, k_prime)
    if out_ids is None:
        out_ids = torch.empty(Q, k, dtype=torch.int32, device=dev)
    if out_scores is None:
        out_scores = torch.empty(Q, k, dtype=torch.float32, device=dev)
    ws_ptr, ws_bytes = _ws_view(workspace)
    fn = lib().ralm_retrieve_topk_seq if sequential else lib().ralm_retrieve_topk_ex
    _check(fn(queries.data_ptr(), Q, ctypes.byref(ds.desc), k, k_prime, out_ids.data_ptr(), out_scores.data_ptr(),
              _ptr(out_margin), ws_ptr, ws_bytes, _stream()))
    return out_ids, out_scores


def ralm_workspace_overflows(workspace: torch.Tensor) -> int:
    ws_ptr, _ = _ws_view(workspace)
    c = ctypes.c_int32(0)
    _check(lib().ralm_workspace_overflows(ws_ptr, _stream(), ctypes.byref(c)))
    return int(c.value)


def ralm_workspace_counters(workspace: torch.Tensor) -> dict:
    """Counters of the last retrieval call on this workspace (numbers of queries)."""
    ws_ptr, _ = _ws_view(workspace)
    c = ralm_counters_t()
    _check(lib().ralm_workspace_counters(ws_ptr, _stream(), ctypes.byref(c)))
    return {name: int(getattr(c, name)) for name, _ in ralm_counters_t._fields_}


RALM_MAX_LADDER_STAGES = 40


def ralm_workspace_stage_entries(workspace: torch.Tensor) -> list:
    """Entries that the candidate lists held at the end of each ladder stage of the last retrieval
    call on this workspace, summed over the queries."""
    ws_ptr, _ = _ws_view(workspace)
    n = ctypes.c_int32(0)
    arr = (ctypes.c_int64 * RALM_MAX_LADDER_STAGES)()
    _check(lib().ralm_workspace_stage_entries(ws_ptr, _stream(), ctypes.byref(n), arr))
    return [int(arr[i]) for i in range(n.value)]


def ralm_retrieve_topk(queries: torch.Tensor, datastore: torch.Tensor, k: int
                       ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Simplest form: fp32 datastore, default stream, synchronous."""
    assert queries.dtype == torch.float32 and datastore.dtype == torch.float32
    assert queries.is_contiguous() and datastore.is_contiguous()
    Q, d = queries.shape
    N = datastore.shape[0]
    out_ids = torch.empty(Q, k, dtype=torch.int32, device=queries.device)
    out_scores = torch.empty(Q, k, dtype=torch.float32, device=queries.device)
    torch.cuda.synchronize()
    _check(lib().ralm_retrieve_topk(queries.data_ptr(), Q, datastore.data_ptr(), N, d, k,
                                    out_ids.data_ptr(), out_scores.data_ptr()))
    return out_ids, out_scores


def ralm_release_buffers() -> None:
    lib().ralm_release_buffers()


def ralm_cache_lookup(cache_ids: torch.Tensor, cache_len: torch.Tensor, queries: torch.Tensor,
                      q_offsets: torch.Tensor, ds: Datastore,
                      spec_ids: Optional[torch.Tensor] = None, spec_scores: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None, use_workspace: bool = True
                      ) -> Tuple[torch.Tensor, torch.Tensor]:
    """``workspace``: int64 tensor of at least Qt elements; allocated here when None (pass
    use_workspace=False to call without one: one workgroup per request)."""
    assert cache_ids.dtype == torch.int32 and cache_len.dtype == torch.int32
    assert q_offsets.dtype == torch.int64 and queries.dtype == torch.float32
    assert cache_ids.is_contiguous() and queries.is_contiguous()
    R, C = cache_ids.shape
    Qt = queries.shape[0]
    if spec_ids is None:
        spec_ids = torch.full((Qt,), -1, dtype=torch.int32, device=queries.device)
    if spec_scores is None:
        spec_scores = torch.full((Qt,), float("-inf"), dtype=torch.float32, device=queries.device)
    if workspace is None and use_workspace:
        workspace = torch.empty(max(Qt, 1), dtype=torch.int64, device=queries.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().ralm_cache_lookup(cache_ids.data_ptr(), cache_len.data_ptr(), C, R, queries.data_ptr(), Qt,
                                   q_offsets.data_ptr(), ctypes.byref(ds.desc), spec_ids.data_ptr(),
                                   spec_scores.data_ptr(), _ptr(workspace), ws_bytes, _stream()))
    return spec_ids, spec_scores


def ralm_cache_lookup_static(cache_ids: torch.Tensor, cache_len: torch.Tensor, queries: torch.Tensor,
                             q_offsets: torch.Tensor, ds: Datastore, spec_ids: torch.Tensor,
                             spec_scores: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """ralm_cache_lookup with the library's built-in scratch: the caller passes inputs and outputs only."""
    assert cache_ids.dtype == torch.int32 and cache_len.dtype == torch.int32
    assert q_offsets.dtype == torch.int64 and queries.dtype == torch.float32
    assert cache_ids.is_contiguous() and queries.is_contiguous()
    assert spec_ids.dtype == torch.int32 and spec_scores.dtype == torch.float32
    R, C = cache_ids.shape
    Qt = queries.shape[0]
    _check(lib().ralm_cache_lookup_static(cache_ids.data_ptr(), cache_len.data_ptr(), C, R, queries.data_ptr(), Qt,
                                          q_offsets.data_ptr(), ctypes.byref(ds.desc), spec_ids.data_ptr(),
                                          spec_scores.data_ptr(), _stream()))
    return spec_ids, spec_scores


def ralm_cache_lookup_topk(cache_ids: torch.Tensor, cache_len: torch.Tensor, queries: torch.Tensor,
                           q_offsets: torch.Tensor, ds: Datastore, k: int,
                           workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """The k best cached entries per query: (ids [Qt, k] int32, scores [Qt, k] fp32)."""
    assert cache_ids.dtype == torch.int32 and cache_len.dtype == torch.int32
    assert q_offsets.dtype == torch.int64 and queries.dtype == torch.float32
    assert cache_ids.is_contiguous() and queries.is_contiguous()
    R, C = cache_ids.shape
    Qt = queries.shape[0]
    dev = queries.device
    need = int(lib().ralm_cache_lookup_topk_workspace_bytes(Qt, C))
    if workspace is None:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=dev)
    ws_ptr, ws_bytes = _ws_view(workspace)
    out_ids = torch.empty(Qt, k, dtype=torch.int32, device=dev)
    out_scores = torch.empty(Qt, k, dtype=torch.float32, device=dev)
    _check(lib().ralm_cache_lookup_topk(cache_ids.data_ptr(), cache_len.data_ptr(), C, R, queries.data_ptr(), Qt,
                                        q_offsets.data_ptr(), ctypes.byref(ds.desc), k, out_ids.data_ptr(),
                                        out_scores.data_ptr(), ws_ptr, ws_bytes, _stream()))
    return out_ids, out_scores


def ralm_verify(spec_ids: torch.Tensor, true_ids: torch.Tensor, q_offsets: torch.Tensor,
                true_stride: int = 1, first_mismatch: Optional[torch.Tensor] = None) -> torch.Tensor:
    assert spec_ids.dtype == torch.int32 and true_ids.dtype == torch.int32 and q_offsets.dtype == torch.int64
    R = q_offsets.shape[0] - 1
    Qt = spec_ids.shape[0]
    if first_mismatch is None:
        first_mismatch = torch.empty(R, dtype=torch.int32, device=spec_ids.device)
    _check(lib().ralm_verify(spec_ids.data_ptr(), true_ids.data_ptr(), true_stride, Qt, q_offsets.data_ptr(), R,
                             first_mismatch.data_ptr(), _stream()))
    return first_mismatch


def ralm_cache_insert(cache_ids: torch.Tensor, cache_len: torch.Tensor, cache_head: torch.Tensor,
                      true_ids: torch.Tensor, q_offsets: torch.Tensor, N: int, p: int = 1, n_next: int = 0,
                      first_mismatch: Optional[torch.Tensor] = None, true_stride: Optional[int] = None) -> None:
    """In-place cache update; ``true_ids`` is the [Qt, k] out_ids of a retrieval (or flat with true_stride)."""
    assert cache_ids.dtype == torch.int32 and cache_ids.is_contiguous() and cache_ids.dim() == 2
    assert cache_len.dtype == torch.int32 and cache_head.dtype == torch.int32
    assert true_ids.dtype == torch.int32 and true_ids.is_contiguous() and q_offsets.dtype == torch.int64
    R, C = cache_ids.shape
    if true_stride is None:
        true_stride = true_ids.shape[1] if true_ids.dim() == 2 else 1
    Qt = true_ids.numel() // true_stride
    assert first_mismatch is None or first_mismatch.dtype == torch.int32
    _check(lib().ralm_cache_insert(cache_ids.data_ptr(), cache_len.data_ptr(), cache_head.data_ptr(), C, R,
                                   true_ids.data_ptr(), true_stride, Qt, q_offsets.data_ptr(),
                                   _ptr(first_mismatch), p, n_next, N, _stream()))


def ralm_knnlm_probs(ids: torch.Tensor, scores: torch.Tensor, values: torch.Tensor, temperature: float = 1.0,
                     want_top: bool = True):
    """Neighbour distribution of a retrieval result: (tokens, weights, top_token, top_prob)."""
    assert ids.dtype == torch.int32 and scores.dtype == torch.float32 and values.dtype == torch.int32
    assert ids.is_contiguous() and scores.is_contiguous() and values.is_contiguous() and ids.shape == scores.shape
    Q, k = ids.shape
    dev = ids.device
    tokens = torch.empty(Q, k, dtype=torch.int32, device=dev)
    weights = torch.empty(Q, k, dtype=torch.float32, device=dev)
    top_token = torch.empty(Q, dtype=torch.int32, device=dev) if want_top else None
    top_prob = torch.empty(Q, dtype=torch.float32, device=dev) if want_top else None
    _check(lib().ralm_knnlm_probs(ids.data_ptr(), scores.data_ptr(), Q, k, values.data_ptr(), values.shape[0],
                                  float(temperature), tokens.data_ptr(), weights.data_ptr(), _ptr(top_token),
                                  _ptr(top_prob), _stream()))
    return tokens, weights, top_token, top_prob


def ralm_os3_gamma(strides, matched, gamma_max: float = 0.6) -> float:
    """Host-side: speculation accuracy estimate from the recent (stride, matched) history."""
    w = len(strides)
    assert len(matched) == w
    s = (ctypes.c_int32 * max(w, 1))(*[int(v) for v in strides])
    m = (ctypes.c_int32 * max(w, 1))(*[int(v) for v in matched])
    return float(lib().ralm_os3_gamma(s, m, w, gamma_max))


def ralm_os3_objective(gamma: float, a: float, b: float, s: int, asynchronous: bool = False) -> float:
    return float(lib().ralm_os3_objective(gamma, a, b, s, 1 if asynchronous else 0))


def ralm_os3_stride(gamma: float, a: float, b: float, s_max: int, asynchronous: bool = False) -> int:
    return int(lib().ralm_os3_stride(gamma, a, b, s_max, 1 if asynchronous else 0))


def ralm_os3_next_stride(strides, matched, a_samples, b_samples, s_max: int, gamma_max: float = 0.6,
                         asynchronous: bool = False) -> int:
    """Host-side: stride of the next round from a request's recent history."""
    w = len(strides)
    assert len(matched) == w
    s = (ctypes.c_int32 * max(w, 1))(*[int(v) for v in strides])
    m = (ctypes.c_int32 * max(w, 1))(*[int(v) for v in matched])
    a = (ctypes.c_double * max(len(a_samples), 1))(*[float(v) for v in a_samples])
    b = (ctypes.c_double * max(len(b_samples), 1))(*[float(v) for v in b_samples])
    return int(lib().ralm_os3_next_stride(s, m, w, a, len(a_samples), b, len(b_samples), gamma_max, s_max,
                                          1 if asynchronous else 0))


def ralm_scan_reserve_cus(n: int) -> None:
    """Compute units that later retrieval calls leave free for kernels on other streams."""
    lib().ralm_scan_reserve_cus(int(n))


def ralm_profile_enable(on: bool) -> None:
    lib().ralm_profile_enable(1 if on else 0)


def ralm_profile_scan_ms() -> Tuple[float, int]:
    ms, n = ctypes.c_float(0), ctypes.c_int32(0)
    _check(lib().ralm_profile_scan_ms(ctypes.byref(ms), ctypes.byref(n)))
    return float(ms.value), int(n.value)
