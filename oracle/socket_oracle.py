"""numpy/ctypes front end of the C oracle in socket_oracle.c (test infrastructure only).

Each function converts its arguments to the C layout, calls the C routine and
returns numpy arrays.  There is no arithmetic of the method in this file.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        # SOCKET_ORACLE_LIB: a build of the same source to load instead (the sanitizer run of the pins)
        path = os.environ.get("SOCKET_ORACLE_LIB") or _build.build(force=False)
        lib = ctypes.CDLL(path)
        _LIB = lib
    return _LIB


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    """Threads the oracle's parallel loops use (OMP_NUM_THREADS or the core count)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def hash_keys(K, W, L, P, zero_margin=1e-4):
    """Alg. 1.  K [n,d], W [d,L*P] -> (codes uint16 [n,L], near_zero bool [n,L])."""
    K = _f32(K)
    W = _f32(W)
    n, d = K.shape
    assert W.shape == (d, L * P)
    codes = np.zeros((n, L), dtype=np.uint16)
    nz = np.zeros((n, L), dtype=np.uint8)
    rc = _lib().socket_oracle_hash_keys(
        _p(K, ctypes.c_float), ctypes.c_long(n), ctypes.c_int(d), _p(W, ctypes.c_float),
        ctypes.c_int(L), ctypes.c_int(P), _p(codes, ctypes.c_uint16), _p(nz, ctypes.c_uint8),
        ctypes.c_double(zero_margin))
    _check(rc, "hash_keys")
    return codes, nz.astype(bool)


def soft_probs(q, W, L, P, tau):
    """Alg. 2.  q [d], W [d,L*P] -> p float64 [L, 2^P]."""
    q = _f32(q)
    W = _f32(W)
    d = q.shape[0]
    assert W.shape == (d, L * P)
    p = np.zeros((L, 1 << P), dtype=np.float64)
    rc = _lib().socket_oracle_soft_probs(
        _p(q, ctypes.c_float), ctypes.c_int(d), _p(W, ctypes.c_float), ctypes.c_int(L),
        ctypes.c_int(P), ctypes.c_double(tau), _p(p, ctypes.c_double))
    _check(rc, "soft_probs")
    return p


def score(codes, p, P, vnorm=None, mask=None, seq_len=None):
    """Alg. 5.  codes [n,L], p [G,L,R] or [L,R] -> scores float64 [n]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    p = np.ascontiguousarray(p, dtype=np.float64)
    if p.ndim == 2:
        p = p[None]
    n, L = codes.shape
    G = p.shape[0]
    assert p.shape == (G, L, 1 << P)
    if seq_len is None:
        seq_len = n
    vn = _f32(vnorm) if vnorm is not None else None
    mk = np.ascontiguousarray(mask, dtype=np.uint8) if mask is not None else None
    out = np.zeros(n, dtype=np.float64)
    rc = _lib().socket_oracle_score(
        _p(codes, ctypes.c_uint16), ctypes.c_long(n), ctypes.c_int(L), ctypes.c_int(P),
        _p(p, ctypes.c_double), ctypes.c_int(G), _p(vn, ctypes.c_float),
        _p(mk, ctypes.c_uint8), ctypes.c_long(seq_len), _p(out, ctypes.c_double))
    _check(rc, "score")
    return out


def hard_score(codes, qcodes):
    """Eq. 3 (hard).  codes [n,L], qcodes [L] -> collision counts float64 [n]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    qcodes = np.ascontiguousarray(qcodes, dtype=np.uint16)
    n, L = codes.shape
    out = np.zeros(n, dtype=np.float64)
    rc = _lib().socket_oracle_hard_score(
        _p(codes, ctypes.c_uint16), ctypes.c_long(n), ctypes.c_int(L),
        _p(qcodes, ctypes.c_uint16), _p(out, ctypes.c_double))
    _check(rc, "hard_score")
    return out


def topk(scores, k):
    """TopK of Alg. 3.  scores [n] -> (idx int32 [k] padded with -1, n_selected)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    n = scores.shape[0]
    idx = np.full(max(k, 0), -1, dtype=np.int32)
    nsel = ctypes.c_long(0)
    rc = _lib().socket_oracle_topk(
        _p(scores, ctypes.c_double), ctypes.c_long(n), ctypes.c_long(k),
        _p(idx, ctypes.c_int32), ctypes.byref(nsel))
    _check(rc, "topk")
    return idx, int(nsel.value)


def sparse_decode(q, K, V, idx, scale=1.0):
    """Eq. 2.  q [d], K,V [n,d], idx [k] -> y float64 [d]."""
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    n, d = K.shape
    y = np.zeros(d, dtype=np.float64)
    rc = _lib().socket_oracle_sparse_decode(
        _p(q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), ctypes.c_long(n),
        ctypes.c_int(d), _p(idx, ctypes.c_int32), ctypes.c_long(idx.shape[0]),
        ctypes.c_double(scale), _p(y, ctypes.c_double))
    _check(rc, "sparse_decode")
    return y


def dense_decode(q, K, V, scale=1.0):
    """Eq. 1.  q [d], K,V [n,d] -> y float64 [d]."""
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    n, d = K.shape
    y = np.zeros(d, dtype=np.float64)
    rc = _lib().socket_oracle_dense_decode(
        _p(q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), ctypes.c_long(n),
        ctypes.c_int(d), ctypes.c_double(scale), _p(y, ctypes.c_double))
    _check(rc, "dense_decode")
    return y


def force_tokens(scores, seq_len, n_sink, n_window):
    """Sink / local-window override: +inf for the first n_sink and last n_window valid tokens.
    scores float64 [n] -> new float64 [n]."""
    out = np.ascontiguousarray(scores, dtype=np.float64).copy()
    rc = _lib().socket_oracle_force_tokens(
        _p(out, ctypes.c_double), ctypes.c_long(out.shape[0]), ctypes.c_long(int(seq_len)),
        ctypes.c_long(int(n_sink)), ctypes.c_long(int(n_window)))
    _check(rc, "force_tokens")
    return out


def value_norms(V):
    """||v_j||_2 as returned by Alg. 1.  V [n,d] -> float32 [n]."""
    V = _f32(V)
    n, d = V.shape
    out = np.zeros(n, dtype=np.float32)
    rc = _lib().socket_oracle_value_norms(
        _p(V, ctypes.c_float), ctypes.c_long(n), ctypes.c_int(d), _p(out, ctypes.c_float))
    _check(rc, "value_norms")
    return out


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def precision(retrieved, relevant):
    """Precision = |S_k & R| / k (appendix, metric definitions).  Index arrays -> float."""
    s, r = _i32(retrieved), _i32(relevant)
    out = ctypes.c_double(0.0)
    rc = _lib().socket_oracle_precision(_p(s, ctypes.c_int32), ctypes.c_long(s.shape[0]),
                                        _p(r, ctypes.c_int32), ctypes.c_long(r.shape[0]), ctypes.byref(out))
    _check(rc, "precision")
    return out.value


def jaccard(a, b):
    """Jaccard(A, B) = |A & B| / |A | B| (appendix, metric definitions).  Index arrays -> float."""
    a, b = _i32(a), _i32(b)
    out = ctypes.c_double(0.0)
    rc = _lib().socket_oracle_jaccard(_p(a, ctypes.c_int32), ctypes.c_long(a.shape[0]),
                                      _p(b, ctypes.c_int32), ctypes.c_long(b.shape[0]), ctypes.byref(out))
    _check(rc, "jaccard")
    return out.value


def ndcg(rel_ranked, rel_all):
    """NDCG of a ranked list (appendix, metric definitions): rel_ranked [k] relevance of the
    retrieved items best-ranked first, rel_all [n] relevance of every candidate -> float."""
    rr = np.ascontiguousarray(rel_ranked, dtype=np.float64)
    ra = np.ascontiguousarray(rel_all, dtype=np.float64)
    out = ctypes.c_double(0.0)
    rc = _lib().socket_oracle_ndcg(_p(rr, ctypes.c_double), ctypes.c_long(rr.shape[0]),
                                   _p(ra, ctypes.c_double), ctypes.c_long(ra.shape[0]), ctypes.byref(out))
    _check(rc, "ndcg")
    return out.value
