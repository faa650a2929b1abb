"""ctypes front-end of the plain-C PQTopK oracle (`pq_oracle.c`) -- TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.  It never touches the
HIP library or its Python binding.  Arrays are numpy, host memory; shapes follow the paper's notation
(codes [N][m] = G of Eq. 1, centroids [m][b][d/m] = Psi, queries [B][d] = phi, S [B][m][b] of Eq. 4).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pq_oracle.c")
_LIB = os.path.join(_HERE, "libpq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pq_oracle.c with gcc.  No fast-math, no contraction: the source states the evaluation order."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P, I, LL = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
        lib.pq_oracle_num_threads.restype = I
        lib.pq_oracle_set_num_threads.argtypes = [I]
        lib.pq_oracle_subitem_scores.argtypes = [P, P, P, I, I, I, I]
        lib.pq_oracle_item_scores.argtypes = [P, P, P, LL, I, I]
        lib.pq_oracle_item_scores_split_major.argtypes = [P, P, P, LL, I, I]
        lib.pq_oracle_topk_fullsort.argtypes = [P, LL, I, P, P]
        lib.pq_oracle_topk.argtypes = [P, LL, I, P, P]
        lib.pq_oracle_score_topk.argtypes = [P, P, LL, I, I, I, I, P, P]
        lib.pq_oracle_score_topk_subset.argtypes = [P, P, P, LL, LL, I, I, I, I, P, P]
        lib.pq_oracle_pqtopk.argtypes = [P, P, P, LL, I, I, I, I, I, P, P]
        lib.pq_oracle_bruteforce_topk.argtypes = [P, P, P, LL, I, I, I, I, I, P, P]
        lib.pq_oracle_reconstruct.argtypes = [P, P, LL, I, I, I, P]
        lib.pq_oracle_default_scores.argtypes = [P, P, LL, I, I, P]
        lib.pq_oracle_item_scores_u16.argtypes = [P, P, P, LL, I, I]
        lib.pq_oracle_score_topk_u16.argtypes = [P, P, LL, I, I, I, I, P, P]
        lib.pq_oracle_bruteforce_topk_u16.argtypes = [P, P, P, LL, I, I, I, I, I, P, P]
        _lib = lib
    return _lib


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: argument error (rc={rc})")


def num_threads() -> int:
    return _load().pq_oracle_num_threads()


def set_num_threads(n: int) -> None:
    _load().pq_oracle_set_num_threads(int(n))


def subitem_scores(queries: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """Eq. 4 -> S fp32 [B][m][b]."""
    queries = _c(queries, np.float32)
    centroids = _c(centroids, np.float32)
    B, d = queries.shape
    m, b, s = centroids.shape
    if m * s != d:
        raise ValueError("centroids do not match d")
    S = np.empty((B, m, b), dtype=np.float32)
    _check(_load().pq_oracle_subitem_scores(_p(queries), _p(centroids), _p(S), B, d, m, b), "subitem_scores")
    return S


def item_scores(codes: np.ndarray, S1: np.ndarray, split_major: bool = False) -> np.ndarray:
    """Eq. 5 for one query (S1 is [m][b]) -> fp32 [N].  split_major=True runs Algorithm 2's loop order."""
    codes = _c(codes, np.uint8)
    S1 = _c(S1, np.float32)
    N, m = codes.shape
    if S1.shape[0] != m:
        raise ValueError("S does not match m")
    b = S1.shape[1]
    out = np.empty(N, dtype=np.float32)
    fn = _load().pq_oracle_item_scores_split_major if split_major else _load().pq_oracle_item_scores
    _check(fn(_p(codes), _p(S1), _p(out), N, m, b), "item_scores")
    return out


def topk(score: np.ndarray, K: int, fullsort: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """TopK of Algorithm 1's last line -> (ids int32 [K], scores fp32 [K]), score desc then id asc."""
    score = _c(score, np.float32)
    ids = np.empty(K, dtype=np.int32)
    sc = np.empty(K, dtype=np.float32)
    fn = _load().pq_oracle_topk_fullsort if fullsort else _load().pq_oracle_topk
    _check(fn(_p(score), score.shape[0], K, _p(ids), _p(sc)), "topk")
    return ids, sc


def score_topk(codes: np.ndarray, S: np.ndarray, K: int) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 1 (V = I) for a batch -> (ids int32 [B][K], scores fp32 [B][K])."""
    codes = _c(codes, np.uint8)
    S = _c(S, np.float32)
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m:
        raise ValueError("S does not match m")
    ids = np.empty((B, K), dtype=np.int32)
    sc = np.empty((B, K), dtype=np.float32)
    _check(_load().pq_oracle_score_topk(_p(codes), _p(S), N, B, m, b, K, _p(ids), _p(sc)), "score_topk")
    return ids, sc


def score_topk_subset(codes: np.ndarray, S: np.ndarray, subset: np.ndarray, K: int) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 1 with a candidate list V (distinct item ids, shared by the batch) -> (ids [B][K], scores [B][K])."""
    codes = _c(codes, np.uint8)
    S = _c(S, np.float32)
    subset = _c(subset, np.int32)
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m:
        raise ValueError("S does not match m")
    ids = np.empty((B, K), dtype=np.int32)
    sc = np.empty((B, K), dtype=np.float32)
    _check(_load().pq_oracle_score_topk_subset(_p(codes), _p(S), _p(subset), subset.shape[0], N, B, m, b, K, _p(ids),
                                                _p(sc)), "score_topk_subset")
    return ids, sc


def pqtopk(codes: np.ndarray, centroids: np.ndarray, queries: np.ndarray, K: int):
    """Eq. 4 then Algorithm 1 -> (ids int32 [B][K], scores fp32 [B][K])."""
    codes = _c(codes, np.uint8)
    centroids = _c(centroids, np.float32)
    queries = _c(queries, np.float32)
    N, m = codes.shape
    B, d = queries.shape
    m2, b, s = centroids.shape
    if m2 != m or m * s != d:
        raise ValueError("shape mismatch")
    ids = np.empty((B, K), dtype=np.int32)
    sc = np.empty((B, K), dtype=np.float32)
    _check(_load().pq_oracle_pqtopk(_p(codes), _p(centroids), _p(queries), N, B, d, m, b, K, _p(ids), _p(sc)),
           "pqtopk")
    return ids, sc


def bruteforce_topk(codes: np.ndarray, centroids: np.ndarray, queries: np.ndarray, K: int):
    """Reconstruct every item embedding (Eq. 2), score by full dot product in float64 (Eq. 3), sort.
    -> (ids int32 [B][K], scores float64 [B][K])."""
    codes = _c(codes, np.uint8)
    centroids = _c(centroids, np.float32)
    queries = _c(queries, np.float32)
    N, m = codes.shape
    B, d = queries.shape
    m2, b, s = centroids.shape
    if m2 != m or m * s != d:
        raise ValueError("shape mismatch")
    ids = np.empty((B, K), dtype=np.int32)
    sc = np.empty((B, K), dtype=np.float64)
    _check(_load().pq_oracle_bruteforce_topk(_p(codes), _p(centroids), _p(queries), N, B, d, m, b, K,
                                             _p(ids), _p(sc)), "bruteforce_topk")
    return ids, sc


def reconstruct(codes: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """Eq. 2: item embedding matrix W fp32 [N][d], row i = concatenation of item i's sub-item embeddings."""
    codes = _c(codes, np.uint8)
    centroids = _c(centroids, np.float32)
    N, m = codes.shape
    m2, b, s = centroids.shape
    if m2 != m:
        raise ValueError("shape mismatch")
    W = np.empty((N, m * s), dtype=np.float32)
    _check(_load().pq_oracle_reconstruct(_p(codes), _p(centroids), N, m * s, m, b, _p(W)), "reconstruct")
    return W


def default_scores(W: np.ndarray, queries: np.ndarray) -> np.ndarray:
    """Eq. 3 in float64: r = W phi -> scores float64 [B][N]."""
    W = _c(W, np.float32)
    queries = _c(queries, np.float32)
    N, d = W.shape
    B, d2 = queries.shape
    if d2 != d:
        raise ValueError("shape mismatch")
    out = np.empty((B, N), dtype=np.float64)
    _check(_load().pq_oracle_default_scores(_p(W), _p(queries), N, B, d, _p(out)), "default_scores")
    return out



def item_scores_u16(codes: np.ndarray, S1: np.ndarray) -> np.ndarray:
    """Eq. 5 for one query over uint16 codes (S1 is [m][b], b up to 65536) -> fp32 [N]."""
    codes = _c(codes, np.uint16)
    S1 = _c(S1, np.float32)
    N, m = codes.shape
    if S1.shape[0] != m:
        raise ValueError("S does not match m")
    out = np.empty(N, dtype=np.float32)
    _check(_load().pq_oracle_item_scores_u16(_p(codes), _p(S1), _p(out), N, m, S1.shape[1]), "item_scores_u16")
    return out


def score_topk_u16(codes: np.ndarray, S: np.ndarray, K: int) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 1 (V = I) over uint16 codes for a batch -> (ids int32 [B][K], scores fp32 [B][K])."""
    codes = _c(codes, np.uint16)
    S = _c(S, np.float32)
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m:
        raise ValueError("S does not match m")
    ids = np.empty((B, K), dtype=np.int32)
    sc = np.empty((B, K), dtype=np.float32)
    _check(_load().pq_oracle_score_topk_u16(_p(codes), _p(S), N, B, m, b, K, _p(ids), _p(sc)), "score_topk_u16")
    return ids, sc


def bruteforce_topk_u16(codes: np.ndarray, centroids: np.ndarray, queries: np.ndarray, K: int):
    """Reconstruction (Eq. 2) and full dot products in float64 (Eq. 3) over uint16 codes, sorted.
    -> (ids int32 [B][K], scores float64 [B][K])."""
    codes = _c(codes, np.uint16)
    centroids = _c(centroids, np.float32)
    queries = _c(queries, np.float32)
    N, m = codes.shape
    B, d = queries.shape
    m2, b, s = centroids.shape
    if m2 != m or m * s != d:
        raise ValueError("shape mismatch")
    ids = np.empty((B, K), dtype=np.int32)
    sc = np.empty((B, K), dtype=np.float64)
    _check(_load().pq_oracle_bruteforce_topk_u16(_p(codes), _p(centroids), _p(queries), N, B, d, m, b, K,
                                                 _p(ids), _p(sc)), "bruteforce_topk_u16")
    return ids, sc
