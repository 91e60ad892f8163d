"""ctypes front end of the fp64 CPU oracle (``rocketkv_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Only the test-suite, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product package
never does.  The oracle follows RocketKV (arXiv 2502.14051): Section 3.3
(SnapKV stage), Section 3.4 / Algorithm 1 (hybrid sparse attention) and
Section 3.6 (compression decomposition).  It takes bf16 bit patterns as
``uint16`` numpy arrays in plain contiguous token-major layouts and returns
float64 / int32 numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rocketkv_oracle.c")
_LIB = os.path.join(_HERE, "librocketkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # ROCKETKV_ORACLE_LIB: a library built elsewhere from a copy of the source (the tests that plant
        # mistakes in the oracle and check that the pins notice use it); otherwise the one beside this file
        # (honoured only when ROCKETKV_ORACLE_MUTANT_RUN=1 is set as well, which only that test does)
        other = os.environ.get("ROCKETKV_ORACLE_LIB") if os.environ.get("ROCKETKV_ORACLE_MUTANT_RUN") == "1" else None
        if not other:
            build()
        _lib = C.CDLL(other or _LIB)
        _lib.okv_num_threads.restype = C.c_int
        _lib.okv_pages_to_pick.restype = C.c_int
        _lib.okv_snapkv_unit.restype = C.c_int
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "oracle inputs are bf16 bit patterns (uint16)"
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_load().okv_num_threads())


def topk(v, k):
    """Indices (ascending) of the k largest entries; ties go to the lower index."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    k = min(int(k), v.size)
    out = np.empty(k, dtype=np.int32)
    _load().okv_topk(_p(v, C.c_double), C.c_int(v.size), C.c_int(k), _p(out, C.c_int))
    return out


def pages_to_pick(n, ps, T) -> int:
    return int(_load().okv_pages_to_pick(C.c_int(n), C.c_int(ps), C.c_int(T)))


def page_summaries(K, ps):
    """Step 1 for one unit. K: [n][D] uint16 -> (kmax, kmin) each [D][P] float64."""
    K = _u16(K)
    n, D = K.shape
    P = (n + ps - 1) // ps
    kmax = np.empty((D, P), dtype=np.float64)
    kmin = np.empty((D, P), dtype=np.float64)
    _load().okv_page_summaries(_p(K, C.c_uint16), C.c_int(n), C.c_int(D), C.c_int(ps),
                               _p(kmax, C.c_double), _p(kmin, C.c_double))
    return kmax, kmin


def channel_select(q, k1):
    """q: [G][D] uint16 -> (a, s, i1): sum|q|, sum q, top-k1 channel ids ascending."""
    q = _u16(q)
    G, D = q.shape
    a = np.empty(D, dtype=np.float64)
    s = np.empty(D, dtype=np.float64)
    i1 = np.empty(k1, dtype=np.int32)
    _load().okv_channel_select(_p(q, C.c_uint16), C.c_int(G), C.c_int(D), C.c_int(k1),
                               _p(a, C.c_double), _p(s, C.c_double), _p(i1, C.c_int))
    return a, s, i1


def page_scores(s, i1, kmax, kmin):
    s = np.ascontiguousarray(s, dtype=np.float64)
    i1 = _i32(i1)
    kmax = np.ascontiguousarray(kmax, dtype=np.float64)
    kmin = np.ascontiguousarray(kmin, dtype=np.float64)
    P = kmax.shape[1]
    score = np.empty(P, dtype=np.float64)
    _load().okv_page_scores(_p(s, C.c_double), _p(i1, C.c_int), C.c_int(i1.size),
                            _p(kmax, C.c_double), _p(kmin, C.c_double), C.c_int(P),
                            _p(score, C.c_double))
    return score


def page_select(score, kp, n_recent=0):
    score = np.ascontiguousarray(score, dtype=np.float64)
    kp = min(int(kp), score.size)
    out = np.empty(kp, dtype=np.int32)
    if kp:
        _load().okv_page_select(_p(score, C.c_double), C.c_int(score.size), C.c_int(kp),
                                C.c_int(n_recent), _p(out, C.c_int))
    return out


def attend_pages(q, K, V, ps, pages):
    """Step 3 for one unit. q: [G][D], K/V: [n][D] uint16, pages ascending ids."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    G, D = q.shape
    n = K.shape[0]
    pages = _i32(pages)
    y = np.empty((G, D), dtype=np.float64)
    lse = np.empty(G, dtype=np.float64)
    _load().okv_attend_pages(_p(q, C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16),
                             C.c_int(G), C.c_int(D), C.c_int(n), C.c_int(ps),
                             _p(pages, C.c_int), C.c_int(pages.size),
                             _p(y, C.c_double), _p(lse, C.c_double))
    return y, lse


def hsa_decode(q, K, V, seq_lens, ps, k1, T, n_recent=0, want_scores=False):
    """Batch Algorithm 1.  q: [B][Hq][D]; K, V: [B][Hkv][n_cap][D] uint16.

    Returns dict(y [B][Hq][D] f64, lse [B][Hq], pages [B][Hkv][pages_cap] (-1 pad),
    chans [B][Hkv][k1], scores [B][Hkv][pages_cap] or None).
    """
    q, K, V = _u16(q), _u16(K), _u16(V)
    seq_lens = _i32(seq_lens)
    B, Hq, D = q.shape
    _, Hkv, n_cap, _ = K.shape
    pages_cap = max(1, (n_cap + ps - 1) // ps)
    y = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    pages = np.full((B, Hkv, pages_cap), -1, dtype=np.int32)
    chans = np.zeros((B, Hkv, k1), dtype=np.int32)
    scores = np.full((B, Hkv, pages_cap), np.nan, dtype=np.float64) if want_scores else None
    _load().okv_hsa_decode(_p(q, C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16),
                           _p(seq_lens, C.c_int), C.c_int(B), C.c_int(Hq), C.c_int(Hkv),
                           C.c_int(D), C.c_int(n_cap), C.c_int(ps), C.c_int(k1), C.c_int(T),
                           C.c_int(n_recent), _p(y, C.c_double), _p(lse, C.c_double),
                           _p(pages, C.c_int), C.c_int(pages_cap), _p(chans, C.c_int),
                           _p(scores, C.c_double))
    return dict(y=y, lse=lse, pages=pages, chans=chans, scores=scores)


def dense_decode(q, K, V, seq_lens):
    """Full-KV attention (Table 1, first row).  Returns (y, lse)."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    seq_lens = _i32(seq_lens)
    B, Hq, D = q.shape
    _, Hkv, n_cap, _ = K.shape
    y = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    _load().okv_dense_decode(_p(q, C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16),
                             _p(seq_lens, C.c_int), C.c_int(B), C.c_int(Hq), C.c_int(Hkv),
                             C.c_int(D), C.c_int(n_cap), _p(y, C.c_double), _p(lse, C.c_double))
    return y, lse


def attend_given(q, K, V, seq_lens, ps, pages):
    """Step 3 on a supplied page list [B][Hkv][cap] (-1 terminates a row)."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    seq_lens = _i32(seq_lens)
    pages = _i32(pages)
    B, Hq, D = q.shape
    _, Hkv, n_cap, _ = K.shape
    y = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    _load().okv_attend_given(_p(q, C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16),
                             _p(seq_lens, C.c_int), C.c_int(B), C.c_int(Hq), C.c_int(Hkv),
                             C.c_int(D), C.c_int(n_cap), C.c_int(ps), _p(pages, C.c_int),
                             C.c_int(pages.shape[2]), _p(y, C.c_double), _p(lse, C.c_double))
    return y, lse


def build_summaries(K, seq_lens, ps, pages_cap=None):
    """Batch Step 1.  K: [B][Hkv][n_cap][D] -> kmax, kmin [B][Hkv][D][pages_cap] f64 (NaN pad)."""
    K = _u16(K)
    seq_lens = _i32(seq_lens)
    B, Hkv, n_cap, D = K.shape
    if pages_cap is None:
        pages_cap = max(1, (n_cap + ps - 1) // ps)
    kmax = np.full((B, Hkv, D, pages_cap), np.nan, dtype=np.float64)
    kmin = np.full((B, Hkv, D, pages_cap), np.nan, dtype=np.float64)
    _load().okv_build_summaries(_p(K, C.c_uint16), _p(seq_lens, C.c_int), C.c_int(B),
                                C.c_int(Hkv), C.c_int(D), C.c_int(n_cap), C.c_int(ps),
                                C.c_int(pages_cap), _p(kmax, C.c_double), _p(kmin, C.c_double))
    return kmax, kmin


def snapkv(qobs, K, seq_lens, ks, N, want_votes=False):
    """Batch SnapKV stage.  qobs: [B][Hq][W][D]; K: [B][Hkv][S_cap][D] uint16.

    Returns dict(kept [B][Hkv][N] (-1 pad), n_kept [B], gv, pooled [B][Hkv][S_cap] or None).
    """
    qobs, K = _u16(qobs), _u16(K)
    seq_lens = _i32(seq_lens)
    B, Hq, W, D = qobs.shape
    _, Hkv, S_cap, _ = K.shape
    kept = np.full((B, Hkv, N), -1, dtype=np.int32)
    n_kept = np.zeros(B, dtype=np.int32)
    gv = np.full((B, Hkv, S_cap), np.nan, dtype=np.float64) if want_votes else None
    pooled = np.full((B, Hkv, S_cap), np.nan, dtype=np.float64) if want_votes else None
    _load().okv_snapkv(_p(qobs, C.c_uint16), _p(K, C.c_uint16), _p(seq_lens, C.c_int),
                       C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(S_cap),
                       C.c_int(W), C.c_int(ks), C.c_int(N), _p(kept, C.c_int),
                       _p(n_kept, C.c_int), _p(gv, C.c_double), _p(pooled, C.c_double))
    return dict(kept=kept, n_kept=n_kept, gv=gv, pooled=pooled)


def decompose(c):
    """Section 3.6 split: returns dict(r, stage1, stage2, page, head_ratio)."""
    out = np.zeros(5, dtype=np.float64)
    _load().okv_decompose(C.c_double(float(c)), _p(out, C.c_double))
    return dict(r=out[0], stage1=out[1], stage2=out[2], page=int(out[3]), head_ratio=out[4])

def cost_model(c):
    """Table 1 (RocketKV / RocketKV-MT rows): dict(storage, storage_mt, traffic) relative to full KV."""
    out = np.zeros(3, dtype=np.float64)
    _load().okv_cost_model(C.c_double(float(c)), _p(out, C.c_double))
    return dict(storage=out[0], storage_mt=out[1], traffic=out[2])


def decompose_budget(S, t, D):
    """Section 3.6 + Appendix A.3: integer operating point dict(page, keep, channels, attend_tokens)."""
    out = np.zeros(4, dtype=np.int32)
    _load().okv_decompose_budget(C.c_longlong(int(S)), C.c_int(int(t)), C.c_int(int(D)), _p(out, C.c_int))
    return dict(page=int(out[0]), keep=int(out[1]), channels=int(out[2]), attend_tokens=int(out[3]))
