"""ctypes front end of the C oracle, numpy arrays in and out.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module.
Each function forwards to the C routine of the same name in dessert_oracle.c,
which carries the citations; `search` chains them in the order of Alg. 2.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(os.fspath(path))
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def rademacher(seed: int, P: int, d: int) -> np.ndarray:
    R = np.empty((P, d), dtype=np.int8)
    lib().oracle_rademacher(C.c_uint64(seed), C.c_uint32(P), C.c_uint32(d), _p(R))
    return R


def hash_i8(X: np.ndarray, R: np.ndarray, L: int, Cbits: int, want_proj: bool = False):
    X = np.ascontiguousarray(X, dtype=np.int8)
    R = np.ascontiguousarray(R, dtype=np.int8)
    n, d = X.shape
    assert R.shape == (L * Cbits, d)
    if Cbits > 8:      # wide codes: 16 bits per table
        assert Cbits <= 16 and not want_proj
        codes = np.empty((n, L), dtype=np.uint16)
        lib().oracle_hash_i8_wide(_p(X), C.c_uint64(n), C.c_uint32(d), _p(R), C.c_uint32(L), C.c_uint32(Cbits), _p(codes))
        return codes
    codes = np.empty((n, L), dtype=np.uint8)
    proj = np.empty((n, L * Cbits), dtype=np.int32) if want_proj else None
    lib().oracle_hash_i8(_p(X), C.c_uint64(n), C.c_uint32(d), _p(R), C.c_uint32(L), C.c_uint32(Cbits),
                         _p(codes), _p(proj))
    return (codes, proj) if want_proj else codes


def hash_fp(X: np.ndarray, R: np.ndarray, L: int, Cbits: int, want_proj: bool = False):
    """X: fp16 (or fp32) values, R: fp32 matrix; both widened exactly to double inside."""
    X = np.ascontiguousarray(X).astype(np.float32)   # fp16 -> fp32 is exact
    R = np.ascontiguousarray(R, dtype=np.float32)
    n, d = X.shape
    assert R.shape == (L * Cbits, d)
    if Cbits > 8:
        assert Cbits <= 16
        codes = np.empty((n, L), dtype=np.uint16)
        proj = np.empty((n, L * Cbits), dtype=np.float64) if want_proj else None
        lib().oracle_hash_fp_wide(_p(X), C.c_uint64(n), C.c_uint32(d), _p(R), C.c_uint32(L), C.c_uint32(Cbits),
                                  _p(codes), _p(proj))
        return (codes, proj) if want_proj else codes
    codes = np.empty((n, L), dtype=np.uint8)
    proj = np.empty((n, L * Cbits), dtype=np.float64) if want_proj else None
    lib().oracle_hash_fp(_p(X), C.c_uint64(n), C.c_uint32(d), _p(R), C.c_uint32(L), C.c_uint32(Cbits),
                         _p(codes), _p(proj))
    return (codes, proj) if want_proj else codes


def _scores_wide(doc_codes, offsets, q_codes, eq1_C, doc_ids):
    doc_codes = np.ascontiguousarray(doc_codes, dtype=np.uint16)
    q_codes = np.ascontiguousarray(q_codes, dtype=np.uint16)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    L = q_codes.shape[1]
    assert doc_codes.ndim == 2 and doc_codes.shape[1] == L and offsets[-1] <= doc_codes.shape[0]
    n_docs = offsets.shape[0] - 1
    if doc_ids is None:
        n, ids = n_docs, None
    else:
        ids = np.ascontiguousarray(doc_ids, dtype=np.int64)
        n = ids.shape[0]
        assert n == 0 or (ids.min() >= 0 and ids.max() < n_docs)
    out = np.empty(n, dtype=np.int32)
    lib().oracle_scores_wide(_p(doc_codes), _p(offsets), C.c_uint32(L), C.c_uint32(eq1_C), _p(q_codes),
                             C.c_uint32(q_codes.shape[0]), _p(ids), C.c_uint64(n), _p(out))
    return out


def scores(doc_codes: np.ndarray, offsets: np.ndarray, q_codes: np.ndarray, doc_ids=None) -> np.ndarray:
    if np.asarray(doc_codes).dtype == np.uint16:
        return _scores_wide(doc_codes, offsets, q_codes, 0, doc_ids)
    doc_codes = np.ascontiguousarray(doc_codes, dtype=np.uint8)
    q_codes = np.ascontiguousarray(q_codes, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    L = q_codes.shape[1]
    assert doc_codes.ndim == 2 and doc_codes.shape[1] == L
    assert offsets[-1] <= doc_codes.shape[0]
    n_docs = offsets.shape[0] - 1
    if doc_ids is None:
        n = n_docs
        ids = None
    else:
        ids = np.ascontiguousarray(doc_ids, dtype=np.int64)
        n = ids.shape[0]
        assert n == 0 or (ids.min() >= 0 and ids.max() < n_docs)
    out = np.empty(n, dtype=np.int32)
    lib().oracle_scores(_p(doc_codes), _p(offsets), C.c_uint32(L), _p(q_codes), C.c_uint32(q_codes.shape[0]),
                        _p(ids), C.c_uint64(n), _p(out))
    return out


def scores_eq1(doc_codes: np.ndarray, offsets: np.ndarray, q_codes: np.ndarray, Cbits: int, doc_ids=None,
               want_table: bool = False):
    """Scores with the Eq. 1 similarity remap, Q16 fixed point (see oracle_scores_eq1)."""
    if np.asarray(doc_codes).dtype == np.uint16:
        assert not want_table
        return _scores_wide(doc_codes, offsets, q_codes, Cbits, doc_ids)
    doc_codes = np.ascontiguousarray(doc_codes, dtype=np.uint8)
    q_codes = np.ascontiguousarray(q_codes, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    L = q_codes.shape[1]
    assert doc_codes.ndim == 2 and doc_codes.shape[1] == L and offsets[-1] <= doc_codes.shape[0]
    n_docs = offsets.shape[0] - 1
    if doc_ids is None:
        n, ids = n_docs, None
    else:
        ids = np.ascontiguousarray(doc_ids, dtype=np.int64)
        n = ids.shape[0]
        assert n == 0 or (ids.min() >= 0 and ids.max() < n_docs)
    out = np.empty(n, dtype=np.int32)
    table = np.empty(L + 1, dtype=np.float64) if want_table else None
    lib().oracle_scores_eq1(_p(doc_codes), _p(offsets), C.c_uint32(L), C.c_uint32(Cbits), _p(q_codes),
                            C.c_uint32(q_codes.shape[0]), _p(ids), C.c_uint64(n), _p(out), _p(table))
    return (out, table) if want_table else out


PHI_IDENTITY, PHI_EXPM1, PHI_SIGMOID, PHI_EQ1 = 0, 1, 2, 3
SIGMA_MAX, SIGMA_MEAN = 0, 1


def scores_general(doc_codes: np.ndarray, offsets: np.ndarray, q_codes: np.ndarray, phi: int, sigma: int,
                   weights=None, doc_ids=None, want_table: bool = False, eq1_C: int = 1):
    """Alg. 2 with sigma = max or mean of phi(count / L) and a weighted sum over the query vectors, in Q16
    (see oracle_scores_general).  weights: integers in [0, 65536], one per query vector, or None."""
    wide = np.asarray(doc_codes).dtype == np.uint16
    dt = np.uint16 if wide else np.uint8
    doc_codes = np.ascontiguousarray(doc_codes, dtype=dt)
    q_codes = np.ascontiguousarray(q_codes, dtype=dt)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    L = q_codes.shape[1]
    assert doc_codes.ndim == 2 and doc_codes.shape[1] == L and offsets[-1] <= doc_codes.shape[0]
    n_docs = offsets.shape[0] - 1
    if doc_ids is None:
        n, ids = n_docs, None
    else:
        ids = np.ascontiguousarray(doc_ids, dtype=np.int64)
        n = ids.shape[0]
        assert n == 0 or (ids.min() >= 0 and ids.max() < n_docs)
    w = None
    if weights is not None:
        w = np.ascontiguousarray(weights, dtype=np.uint32)
        assert w.shape == (q_codes.shape[0],) and (w.size == 0 or w.max() <= 65536)
    out = np.empty(n, dtype=np.int32)
    table = np.empty(L + 1, dtype=np.float64) if want_table else None
    lib().oracle_scores_general(_p(doc_codes), _p(offsets), C.c_uint32(L), C.c_uint32(2 if wide else 1),
                                C.c_uint32(phi), C.c_uint32(eq1_C), C.c_uint32(sigma), _p(q_codes),
                                C.c_uint32(q_codes.shape[0]),
                                _p(w), _p(ids), C.c_uint64(n), _p(out), _p(table))
    return (out, table) if want_table else out


def assign_centroids(X: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    X = np.ascontiguousarray(X, dtype=np.int8)
    centroids = np.ascontiguousarray(centroids, dtype=np.int8)
    assert X.shape[1] == centroids.shape[1]
    out = np.empty(X.shape[0], dtype=np.int32)
    lib().oracle_assign_centroids(_p(X), C.c_uint64(X.shape[0]), C.c_uint32(X.shape[1]), _p(centroids),
                                  C.c_uint32(centroids.shape[0]), _p(out))
    return out


def kmeans(X: np.ndarray, init_centroids: np.ndarray, iters: int, want_inertia: bool = False):
    """Lloyd's k-means in integers (see oracle_kmeans): returns the centroids after `iters` iterations."""
    X = np.ascontiguousarray(X, dtype=np.int8)
    Cn = np.array(init_centroids, dtype=np.int8, order="C", copy=True)
    assert X.ndim == 2 and Cn.ndim == 2 and X.shape[1] == Cn.shape[1] and Cn.shape[0] >= 1
    inertia = np.zeros(iters, dtype=np.int64) if want_inertia else None
    lib().oracle_kmeans(_p(X), C.c_uint64(X.shape[0]), C.c_uint32(X.shape[1]), _p(Cn), C.c_uint32(Cn.shape[0]),
                        C.c_uint32(iters), _p(inertia))
    return (Cn, inertia) if want_inertia else Cn


def inverted_index(assign: np.ndarray, offsets: np.ndarray, K: int):
    """(bucket_offsets [K+1] int64, bucket_docs uint32): sorted set of documents per centroid."""
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    assert assign.shape[0] >= offsets[-1] and (assign.size == 0 or (assign.min() >= 0 and assign.max() < K))
    n_docs = offsets.shape[0] - 1
    bo = np.empty(K + 1, dtype=np.int64)
    lib().oracle_inverted_index(_p(assign), _p(offsets), C.c_uint64(n_docs), C.c_uint32(K), _p(bo), None)
    docs = np.empty(int(bo[-1]), dtype=np.uint32)
    lib().oracle_inverted_index(_p(assign), _p(offsets), C.c_uint64(n_docs), C.c_uint32(K), _p(bo), _p(docs))
    return bo, docs


def filter_query(Q: np.ndarray, centroids: np.ndarray, bucket_offsets: np.ndarray, bucket_docs: np.ndarray,
                 n_docs: int, probe: int, filter_k: int):
    """One query set: (ids [filter_k] uint32, counts [filter_k] int32), padded with 0xFFFFFFFF / -1."""
    Q = np.ascontiguousarray(Q, dtype=np.int8)
    centroids = np.ascontiguousarray(centroids, dtype=np.int8)
    bo = np.ascontiguousarray(bucket_offsets, dtype=np.int64)
    bd = np.ascontiguousarray(bucket_docs, dtype=np.uint32)
    assert bo.shape[0] == centroids.shape[0] + 1 and probe <= centroids.shape[0]
    ids = np.empty(filter_k, dtype=np.uint32)
    cnt = np.empty(filter_k, dtype=np.int32)
    lib().oracle_filter_query(_p(Q), C.c_uint32(Q.shape[0]), C.c_uint32(Q.shape[1]), _p(centroids),
                              C.c_uint32(centroids.shape[0]), _p(bo), _p(bd), C.c_uint64(n_docs), C.c_uint32(probe),
                              C.c_uint32(filter_k), _p(ids), _p(cnt))
    return ids, cnt


def topk(score: np.ndarray, k: int, ids=None):
    score = np.ascontiguousarray(score, dtype=np.int32)
    ids_a = None if ids is None else np.ascontiguousarray(ids, dtype=np.int64)
    out_ids = np.empty(k, dtype=np.uint32)
    out_scores = np.empty(k, dtype=np.int32)
    lib().oracle_topk(_p(score), _p(ids_a), C.c_uint64(score.shape[0]), C.c_uint32(k), _p(out_ids), _p(out_scores))
    return out_ids, out_scores


def search(doc_codes, offsets, q_codes_list, k, cand_ids=None):
    """Alg. 2 for a batch: per query set, score (all docs or its candidates) then top-k.

    Returns (ids [B,k] uint32, scores [B,k] int32, raw score arrays list)."""
    B = len(q_codes_list)
    ids_out = np.empty((B, k), dtype=np.uint32)
    sc_out = np.empty((B, k), dtype=np.int32)
    raw = []
    for b in range(B):
        cand = None if cand_ids is None else np.asarray(cand_ids[b], dtype=np.int64)
        s = scores(doc_codes, offsets, q_codes_list[b], cand)
        raw.append(s)
        ids_out[b], sc_out[b] = topk(s, k, cand)
    return ids_out, sc_out, raw
