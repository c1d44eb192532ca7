"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments with a status before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2401_14021_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2401_14021_amd import build
        build.build()
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    text = open(os.path.join(ROOT, "include", "ralm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(ralm_[a-z0-9_]+)\s*\(", text))
    assert {"ralm_retrieve_topk", "ralm_retrieve_topk_ex", "ralm_retrieve_topk_seq", "ralm_cache_lookup",
            "ralm_verify", "ralm_cache_insert", "ralm_knnlm_probs", "ralm_os3_stride", "ralm_cache_lookup_topk",
            "ralm_cache_lookup_static",
            "ralm_release_buffers",
            "ralm_workspace_bytes", "ralm_build_scan_copy", "ralm_last_error"} <= names
    for n in names:
        assert hasattr(L, n), n


def _ds(binding, N=1000, d=768, exact=0x1000, exact_dtype=0, scan=0x2000, scan_dtype=1):
    ds = binding.ralm_datastore_t()
    ds.exact, ds.exact_dtype, ds.scan, ds.scan_dtype = exact, exact_dtype, scan, scan_dtype
    ds.N, ds.d, ds.exact_stride, ds.scan_stride = N, d, 0, 0
    return ds


def test_argument_errors_return_status_without_a_device(L):
    from paper_2401_14021_amd import binding as b
    P = 0x10000   # fake, aligned, never dereferenced: every call below fails validation first
    ds = _ds(b)
    ref = ctypes.byref
    ws = L.ralm_workspace_bytes(8, ref(ds), 5, 0)
    assert ws > 0
    call = L.ralm_retrieve_topk_ex
    assert call(None, 8, ref(ds), 5, 0, P, P, None, P, ws, None) == 1            # NULL queries
    assert b"NULL" in L.ralm_last_error()
    assert call(P, 0, ref(ds), 5, 0, P, P, None, P, ws, None) == 2               # Q < 1
    assert call(P, 8, ref(ds), 0, 0, P, P, None, P, ws, None) == 3               # k < 1
    assert call(P, 8, ref(ds), 2000, 0, P, P, None, P, ws, None) == 3            # k > N and > max
    assert call(P, 8, ref(ds), 5, 4, P, P, None, P, ws, None) == 3               # k' < k
    assert call(P, 8, ref(ds), 5, 8192, P, P, None, P, ws, None) == 3            # k' > max
    assert call(P, 8, ref(_ds(b, exact_dtype=1)), 5, 0, P, P, None, P, ws, None) == 4   # bf16 exact copy
    assert call(P, 8, ref(_ds(b, scan_dtype=7)), 5, 0, P, P, None, P, ws, None) == 4
    assert call(P, 8, ref(_ds(b, d=770)), 5, 0, P, P, None, P, ws, None) == 2    # d not a multiple of 8
    assert call(P, 8, ref(_ds(b, exact=0x1004)), 5, 0, P, P, None, P, ws, None) == 5
    assert call(P + 4, 8, ref(ds), 5, 0, P, P, None, P, ws, None) == 5
    assert call(P, 8, ref(ds), 5, 0, P, P, None, None, ws, None) == 6            # no workspace
    assert call(P, 8, ref(ds), 5, 0, P, P, None, P + 16, ws, None) == 6          # misaligned workspace
    assert call(P, 8, ref(ds), 5, 0, P, P, None, P, ws - 1, None) == 6           # too small
    wide = _ds(b)
    wide.scan_stride = 1 << 23                                                   # 16 MiB row pitch
    assert call(P, 8, ref(wide), 5, 0, P, P, None, P, 1 << 30, None) == 2
    assert b"pitch" in L.ralm_last_error()
    huge = _ds(b, N=2_000_000_000)
    assert call(P, 1 << 20, ref(huge), 5, 0, P, P, None, P, 1 << 62, None) == 2  # too many tile pairs
    assert b"split the batch" in L.ralm_last_error()
    l2 = _ds(b)
    l2.metric = 1
    l2.scan_stride = 770
    assert call(P, 8, ref(l2), 5, 0, P, P, None, P, 1 << 30, None) == 2          # scan pitch below d + 8
    l2.scan_stride = 776
    assert L.ralm_workspace_bytes(8, ref(l2), 5, 0) > 0                          # accepted with d + 8 columns
    l2.scan = None
    assert call(P, 8, ref(l2), 5, 0, P, P, None, P, 1 << 30, None) == 1          # squared distance needs a scan copy
    l2 = _ds(b, scan_dtype=0)
    l2.metric = 1
    assert call(P, 8, ref(l2), 5, 0, P, P, None, P, 1 << 30, None) == 4          # ... in bf16 or fp16
    bad = _ds(b)
    bad.metric = 5
    assert call(P, 8, ref(bad), 5, 0, P, P, None, P, 1 << 30, None) == 4
    bl2 = L.ralm_build_scan_copy_l2
    assert bl2(P, 0, 0, None, 1, 0, 10, 768, None) == 1
    assert bl2(P, 1, 0, P, 1, 0, 10, 768, None) == 4                             # bf16 is not an exact copy
    assert bl2(P, 0, 0, P, 0, 0, 10, 768, None) == 4                             # fp32 is not a scan copy
    assert bl2(P, 0, 0, P, 1, 770, 10, 768, None) == 2                           # dst pitch below d + 8
    assert bl2(P, 2, 776, P, 1, 776, 10, 768, None) == 2                         # in place needs equal dtypes
    assert L.ralm_workspace_bytes(8, ref(ds), 0, 0) == 0
    assert L.ralm_workspace_bytes(0, ref(ds), 5, 0) == 0
    # workspace grows with Q and with k'
    assert L.ralm_workspace_bytes(1024, ref(ds), 5, 0) > ws
    assert L.ralm_workspace_bytes(8, ref(ds), 1000, 0) > ws
    # simple form
    assert L.ralm_retrieve_topk(None, 8, P, 1000, 768, 5, P, P) == 1
    assert L.ralm_retrieve_topk(P, 8, P, 1000, 768, 1001, P, P) == 3
    # cache lookup / verify / scan copy
    assert L.ralm_cache_lookup(None, P, 4, 2, P, 6, P, ref(ds), P, P, None, 0, None) == 1
    assert L.ralm_cache_lookup(P, P, 0, 2, P, 6, P, ref(ds), P, P, None, 0, None) == 2
    assert L.ralm_cache_lookup(P, P, 4, 2, P, -1, P, ref(ds), P, P, None, 0, None) == 7
    assert L.ralm_cache_lookup(P, P, 4, 2, P, 6, P, ref(ds), P, P, P, 40, None) == 6     # 8 bytes per query needed
    assert L.ralm_cache_lookup(P, P, 4, 2, P, 6, P, ref(ds), P, P, P + 4, 64, None) == 6 # misaligned scratch
    st = L.ralm_cache_lookup_static
    assert st(P, None, 4, 2, P, 6, P, ref(ds), P, P, None) == 1                   # argument errors come first,
    assert st(P, P, 0, 2, P, 6, P, ref(ds), P, P, None) == 2                      # before any device call
    assert st(P, P, 4, 2, P, 65537, P, ref(ds), P, P, None) == 7                  # beyond the built-in scratch
    assert L.ralm_cache_lookup_workspace_bytes(6) >= 48 and L.ralm_cache_lookup_workspace_bytes(-1) == 0
    ins = L.ralm_cache_insert
    assert ins(P, P, None, 4, 2, P, 5, 6, P, None, 1, 0, 1000, None) == 1         # no head array
    assert ins(P, P, P, 0, 2, P, 5, 6, P, None, 1, 0, 1000, None) == 2            # C < 1
    assert ins(P, P, P, 20000, 2, P, 5, 6, P, None, 1, 0, 1000, None) == 2        # C above the LDS limit
    assert ins(P, P, P, 4, 2, P, 5, 6, P, None, 6, 0, 1000, None) == 3            # p > true_stride
    assert ins(P, P, P, 4, 2, P, 5, 6, P, None, 0, 0, 1000, None) == 3            # p < 1
    assert ins(P, P, P, 4, 2, P, 5, -1, P, None, 1, 0, 1000, None) == 7           # Qt < 0
    assert ins(P, P, P, 4, 2, P, 5, 6, P, None, 1, -1, 1000, None) == 7           # n_next < 0
    assert ins(P, P, P, 4, 2, P, 5, 6, P, None, 1, 0, 0, None) == 2               # N < 1
    kp = L.ralm_knnlm_probs
    assert kp(P, P, 4, 8, None, 100, 1.0, P, P, P, P, None) == 1                  # no values array
    assert kp(P, P, 4, 0, P, 100, 1.0, P, P, P, P, None) == 3                     # k < 1
    assert kp(P, P, 4, 2000, P, 100, 1.0, P, P, P, P, None) == 3                  # k > max
    assert kp(P, P, 4, 8, P, 100, 0.0, P, P, P, P, None) == 7                     # temperature not positive
    assert kp(P, P, 4, 8, P, 0, 1.0, P, P, P, P, None) == 2                       # N < 1
    tk = L.ralm_cache_lookup_topk
    wsk = L.ralm_cache_lookup_topk_workspace_bytes(6, 64)
    assert wsk >= 6 * 64 * 8 + 6 * 4 and L.ralm_cache_lookup_topk_workspace_bytes(6, 0) == 0
    assert tk(P, P, 64, 2, P, 6, P, ref(ds), 8, None, P, P, wsk, None) == 1        # no output
    assert tk(P, P, 5000, 2, P, 6, P, ref(ds), 8, P, P, P, 1 << 30, None) == 2     # C above the limit
    assert tk(P, P, 64, 2, P, 6, P, ref(ds), 65, P, P, P, wsk, None) == 3          # k > C
    assert tk(P, P, 64, 2, P, 6, P, ref(ds), 8, P, P, None, wsk, None) == 6        # no workspace
    assert tk(P, P, 64, 2, P, 6, P, ref(ds), 8, P, P, P, wsk - 1, None) == 6       # too small
    assert L.ralm_verify(P, None, 1, 6, P, 2, P, None) == 1
    assert L.ralm_verify(P, P, 0, 6, P, 2, P, None) == 7
    assert L.ralm_verify(P, P, 1, 6, P, -1, P, None) == 2
    assert L.ralm_build_scan_copy(P, 0, P, 0, 0, 10, 768, None) == 4             # fp32 is not a scan copy
    assert L.ralm_build_scan_copy(P, 0, P, 1, 0, 10, 12, None) == 2
    assert L.ralm_build_scan_copy(P, 0, None, 1, 0, 10, 768, None) == 1
    n, arr = ctypes.c_int32(0), (ctypes.c_int64 * b.RALM_MAX_LADDER_STAGES)()
    assert L.ralm_workspace_stage_entries(None, None, ref(n), arr) == 1             # accessors check their pointers
    assert L.ralm_workspace_stage_entries(P, None, None, arr) == 1
    assert L.ralm_workspace_counters(None, None, ref(b.ralm_counters_t())) == 1


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    from paper_2401_14021_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libralm.so")
    with pytest.raises(FileNotFoundError):
        binding.lib()


# ---- stride scheduler: host-only functions of the library against the oracle (no GPU involved) ----
def test_os3_matches_oracle(L, oracle):
    from paper_2401_14021_amd import binding as b
    import numpy as np
    from test_oracle_pins import _read_os3_cases
    objective, gamma = _read_os3_cases()
    for g, a, bb, s, asy, val in objective:
        assert b.ralm_os3_objective(g, a, bb, s, asy) == pytest.approx(val, rel=1e-14)
    for st, m, gmax, est in gamma:
        assert b.ralm_os3_gamma(st, m, gmax) == est
    rng = np.random.default_rng(12)
    for _ in range(400):
        g = float(rng.choice([0.0, 1.0, rng.random()]))
        a, bb = float(rng.random() * 5 + 1e-3), float(rng.random() * 50)
        asy = bool(rng.integers(0, 2))
        for s in (1, 2, 3, 7, 32):
            assert b.ralm_os3_objective(g, a, bb, s, asy) == pytest.approx(oracle.os3_objective(g, a, bb, s, asy), rel=1e-12)
        s_lib = b.ralm_os3_stride(g, a, bb, 32, asy)
        s_or = oracle.os3_stride(g, a, bb, 32, asy)
        # equal, or tied within rounding (the two sum the expectation in different orders)
        assert s_lib == s_or or oracle.os3_objective(g, a, bb, s_lib, asy) == pytest.approx(
            oracle.os3_objective(g, a, bb, s_or, asy), rel=1e-12)
        w = int(rng.integers(0, 8))
        st = rng.integers(1, 9, size=w)
        m = np.minimum(rng.integers(0, 10, size=w), st)
        assert b.ralm_os3_gamma(st, m, 0.6) == oracle.os3_gamma(st, m, 0.6) if w else b.ralm_os3_gamma(st, m) == 0.0
    assert b.ralm_os3_stride(0.5, 1, 4, 16) == 2 and b.ralm_os3_stride(0.0, 1, 4, 16) == 1
    # the combined call = the oracle's pieces put together; 1 while there is no history
    assert b.ralm_os3_next_stride([], [], [1.0], [4.0], 16) == 1
    assert b.ralm_os3_next_stride([3], [3], [], [4.0], 16) == 1
    for _ in range(200):
        w = int(rng.integers(1, 6))
        st = rng.integers(1, 9, size=w)
        m = np.minimum(rng.integers(0, 10, size=w), st)
        a_s, b_s = rng.random(int(rng.integers(1, 6))) + 0.05, rng.random(int(rng.integers(1, 6))) * 20
        asy = bool(rng.integers(0, 2))
        want = oracle.os3_stride(oracle.os3_gamma(st, m, 0.6), oracle.os3_latency(a_s), oracle.os3_latency(b_s), 16, asy)
        got = b.ralm_os3_next_stride(st, m, a_s, b_s, 16, 0.6, asy)
        g, a, bb = oracle.os3_gamma(st, m, 0.6), oracle.os3_latency(a_s), oracle.os3_latency(b_s)
        assert got == want or oracle.os3_objective(g, a, bb, got, asy) == pytest.approx(
            oracle.os3_objective(g, a, bb, want, asy), rel=1e-12)
    assert b.ralm_os3_objective(0.5, 1, 4, 0) != b.ralm_os3_objective(0.5, 1, 4, 0)      # NaN for s < 1
    assert b.ralm_os3_objective(1.5, 1, 4, 2) != b.ralm_os3_objective(1.5, 1, 4, 2)      # NaN for gamma > 1
