"""Python names for the C ABI in include/pqtopk.h: argument marshalling only.

Every computation happens in the HIP kernels of libpqtopk.so.  Tensors are torch CUDA (ROCm) tensors, used here
only as device memory; work is enqueued on torch's current stream.  If the library has not been built the import
of the first entry point raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpqtopk.so")

PQ_OK, PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED, PQ_ERR_WORKSPACE, PQ_ERR_ALIGN, PQ_ERR_HIP = 0, -1, -2, -3, -4, -5, -6
PQ_ERR_TOO_LARGE = -7
PQ_STATIC_SCRATCH_BYTES = 8 << 20

_lib = None


class PQError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {pq_strerror(code)} (code {code})")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it was never built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_09992_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        P, I, LL, SZ = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_size_t
        L.pq_subitem_scores.argtypes = [P, P, P, I, I, I, I, P]
        L.pq_subitem_scores.restype = I
        L.pq_score_topk_workspace_bytes.argtypes = [LL, I, I, I, I]
        L.pq_score_topk_workspace_bytes.restype = SZ
        L.pq_score_topk.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P]
        L.pq_score_topk.restype = I
        L.pq_score_topk_static.argtypes = [P, P, LL, I, I, I, I, P, P, P]
        L.pq_score_topk_static.restype = I
        L.pq_score_topk_profile.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P, I, ctypes.POINTER(ctypes.c_float)]
        L.pq_score_topk_profile.restype = I
        L.pq_score_topk_u16_workspace_bytes.argtypes = [LL, I, I, I, I]
        L.pq_score_topk_u16_workspace_bytes.restype = SZ
        L.pq_score_topk_u16.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P]
        L.pq_score_topk_u16.restype = I
        L.pq_score_topk_u16_profile.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P, I, ctypes.POINTER(ctypes.c_float)]
        L.pq_score_topk_u16_profile.restype = I
        L.pq_score_topk_subset_workspace_bytes.argtypes = [LL, I, I, I, I]
        L.pq_score_topk_subset_workspace_bytes.restype = SZ
        L.pq_score_topk_subset.argtypes = [P, P, P, LL, LL, I, I, I, I, P, P, P, SZ, P]
        L.pq_score_topk_subset.restype = I
        L.pq_topk_scores_workspace_bytes.argtypes = [LL, I, I]
        L.pq_topk_scores_workspace_bytes.restype = SZ
        L.pq_topk_scores.argtypes = [P, LL, LL, I, I, P, P, P, SZ, P]
        L.pq_topk_scores.restype = I
        L.pq_recjpq_scores.argtypes = [P, P, LL, I, I, I, P, LL, P]
        L.pq_recjpq_scores.restype = I
        L.pq_reconstruct_items.argtypes = [P, P, LL, I, I, I, P, P]
        L.pq_reconstruct_items.restype = I
        L.pq_default_scores.argtypes = [P, P, LL, I, I, P, LL, P]
        L.pq_default_scores.restype = I
        L.pq_read_bandwidth_profile.argtypes = [P, SZ, P, I, ctypes.POINTER(ctypes.c_float)]
        L.pq_read_bandwidth_profile.restype = I
        L.pq_measure_empty_launch.argtypes = [I, I, P, I, ctypes.POINTER(ctypes.c_float)]
        L.pq_measure_empty_launch.restype = I
        L.pq_measure_lds_gather.argtypes = [I, I, I, I, I, I, I, P, P, I, ctypes.POINTER(ctypes.c_float)]
        L.pq_measure_lds_gather.restype = I
        L.pq_measure_sync_variant.argtypes = [I, P, SZ, P, I, ctypes.POINTER(ctypes.c_float)]
        L.pq_measure_sync_variant.restype = I
        L.pq_measure_force_general.argtypes = [I]
        L.pq_measure_force_general.restype = I
        L.pq_measure_step_stamps.argtypes = [P, P, P, LL, I, I, I, I, I, P, P, P, P, SZ, P, SZ, ctypes.POINTER(I * 2), P]
        L.pq_measure_step_stamps.restype = I
        L.pq_strerror.argtypes = [I]
        L.pq_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def pq_strerror(code: int) -> str:
    return lib().pq_strerror(int(code)).decode()


def _dev(t: torch.Tensor, dtype: torch.dtype, what: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{what} must live in device memory")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous {dtype}")
    return t


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def pq_subitem_scores(queries: torch.Tensor, centroids: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 4: queries [B][d], centroids [m][b][d/m] -> S [B][m][b] (all fp32, on the device)."""
    _dev(queries, torch.float32, "queries")
    _dev(centroids, torch.float32, "centroids")
    B, d = queries.shape
    m, b, s = centroids.shape
    if m * s != d:
        raise PQError(PQ_ERR_SHAPE, "pq_subitem_scores")
    S = out if out is not None else torch.empty((B, m, b), dtype=torch.float32, device=queries.device)
    _dev(S, torch.float32, "S")
    rc = lib().pq_subitem_scores(queries.data_ptr(), centroids.data_ptr(), S.data_ptr(), B, d, m, b, _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_subitem_scores")
    return S


def pq_score_topk_workspace_bytes(N: int, B: int, m: int, b: int, K: int) -> int:
    return int(lib().pq_score_topk_workspace_bytes(N, B, m, b, K))


def _topk_args(codes, S, K, workspace, out_ids, out_scores, wide=False):
    _dev(codes, torch.uint16 if wide else torch.uint8, "codes")
    _dev(S, torch.float32, "S")
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m:
        raise PQError(PQ_ERR_SHAPE, "pq_score_topk")
    need = (pq_score_topk_u16_workspace_bytes if wide else pq_score_topk_workspace_bytes)(N, B, m, b, K)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=codes.device)
    if out_ids is None:
        out_ids = torch.empty((B, K), dtype=torch.int32, device=codes.device)
    if out_scores is None:
        out_scores = torch.empty((B, K), dtype=torch.float32, device=codes.device)
    _dev(out_ids, torch.int32, "out_ids")
    _dev(out_scores, torch.float32, "out_scores")
    return N, B, m, b, workspace, out_ids, out_scores


def pq_score_topk(codes: torch.Tensor, S: torch.Tensor, K: int, workspace: Optional[torch.Tensor] = None,
                  out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None
                  ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Algorithm 1 (V = I): codes uint8 [N][m], S fp32 [B][m][b] -> (ids int32 [B][K], scores fp32 [B][K])."""
    N, B, m, b, workspace, out_ids, out_scores = _topk_args(codes, S, K, workspace, out_ids, out_scores)
    rc = lib().pq_score_topk(codes.data_ptr(), S.data_ptr(), N, B, m, b, K, out_ids.data_ptr(),
                             out_scores.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_score_topk")
    return out_ids, out_scores


def pq_score_topk_static(codes: torch.Tensor, S: torch.Tensor, K: int, out_ids: torch.Tensor, out_scores: torch.Tensor
                         ) -> Tuple[torch.Tensor, torch.Tensor]:
    """pq_score_topk on the library's built-in scratch: the call allocates nothing (outputs are the caller's)."""
    _dev(codes, torch.uint8, "codes")
    _dev(S, torch.float32, "S")
    _dev(out_ids, torch.int32, "out_ids")
    _dev(out_scores, torch.float32, "out_scores")
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m or tuple(out_ids.shape) != (B, K) or tuple(out_scores.shape) != (B, K):
        raise PQError(PQ_ERR_SHAPE, "pq_score_topk_static")
    rc = lib().pq_score_topk_static(codes.data_ptr(), S.data_ptr(), N, B, m, b, K, out_ids.data_ptr(),
                                    out_scores.data_ptr(), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_score_topk_static")
    return out_ids, out_scores


def pq_score_topk_u16_workspace_bytes(N: int, B: int, m: int, b: int, K: int) -> int:
    return int(lib().pq_score_topk_u16_workspace_bytes(N, B, m, b, K))


def pq_score_topk_u16(codes: torch.Tensor, S: torch.Tensor, K: int, workspace: Optional[torch.Tensor] = None,
                      out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None
                      ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Algorithm 1 (V = I) over 16-bit sub-ids: codes uint16 [N][m], S fp32 [B][m][b], b <= 65536
    -> (ids int32 [B][K], scores fp32 [B][K])."""
    N, B, m, b, workspace, out_ids, out_scores = _topk_args(codes, S, K, workspace, out_ids, out_scores, wide=True)
    rc = lib().pq_score_topk_u16(codes.data_ptr(), S.data_ptr(), N, B, m, b, K, out_ids.data_ptr(),
                                 out_scores.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_score_topk_u16")
    return out_ids, out_scores


def pq_score_topk_u16_profile(codes: torch.Tensor, S: torch.Tensor, K: int, iters: int,
                              workspace: Optional[torch.Tensor] = None) -> float:
    """Mean duration (ms) of pq_score_topk_u16's scan kernel over `iters` launches, from HIP events on the stream."""
    N, B, m, b, workspace, out_ids, out_scores = _topk_args(codes, S, K, workspace, None, None, wide=True)
    ms = ctypes.c_float(0.0)
    rc = lib().pq_score_topk_u16_profile(codes.data_ptr(), S.data_ptr(), N, B, m, b, K, out_ids.data_ptr(),
                                         out_scores.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(),
                                         iters, ctypes.byref(ms))
    if rc != PQ_OK:
        raise PQError(rc, "pq_score_topk_u16_profile")
    return float(ms.value)


def pq_score_topk_subset_workspace_bytes(n_subset: int, B: int, m: int, b: int, K: int) -> int:
    return int(lib().pq_score_topk_subset_workspace_bytes(n_subset, B, m, b, K))


def _subset_args(codes, S, subset, K, workspace, out_ids, out_scores):
    _dev(codes, torch.uint8, "codes")
    _dev(S, torch.float32, "S")
    _dev(subset, torch.int32, "subset")
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m or subset.dim() != 1:
        raise PQError(PQ_ERR_SHAPE, "pq_score_topk_subset")
    n = subset.numel()
    if workspace is None:
        need = pq_score_topk_subset_workspace_bytes(n, B, m, b, K)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=codes.device)
    if out_ids is None:
        out_ids = torch.empty((B, K), dtype=torch.int32, device=codes.device)
    if out_scores is None:
        out_scores = torch.empty((B, K), dtype=torch.float32, device=codes.device)
    _dev(out_ids, torch.int32, "out_ids")
    _dev(out_scores, torch.float32, "out_scores")
    return n, N, B, m, b, workspace, out_ids, out_scores


def pq_score_topk_subset(codes: torch.Tensor, S: torch.Tensor, subset: torch.Tensor, K: int,
                         workspace: Optional[torch.Tensor] = None, out_ids: Optional[torch.Tensor] = None,
                         out_scores: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Algorithm 1 with a candidate list V: subset int32 [n] of distinct item ids -> the K best items of the list."""
    n, N, B, m, b, workspace, out_ids, out_scores = _subset_args(codes, S, subset, K, workspace, out_ids, out_scores)
    rc = lib().pq_score_topk_subset(codes.data_ptr(), S.data_ptr(), subset.data_ptr(), n, N, B, m, b, K,
                                    out_ids.data_ptr(), out_scores.data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_score_topk_subset")
    return out_ids, out_scores


def pq_topk_scores_workspace_bytes(N: int, B: int, K: int) -> int:
    return int(lib().pq_topk_scores_workspace_bytes(N, B, K))


def pq_topk_scores(scores: torch.Tensor, K: int, N: Optional[int] = None, workspace: Optional[torch.Tensor] = None,
                   out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None
                   ) -> Tuple[torch.Tensor, torch.Tensor]:
    """TopK over score rows: scores fp32 [B][ld] (the first N of each row count; default N = ld)."""
    _dev(scores, torch.float32, "scores")
    B, ld = scores.shape
    N = ld if N is None else N
    if workspace is None:
        workspace = torch.empty(max(pq_topk_scores_workspace_bytes(N, B, K), 16), dtype=torch.uint8, device=scores.device)
    if out_ids is None:
        out_ids = torch.empty((B, K), dtype=torch.int32, device=scores.device)
    if out_scores is None:
        out_scores = torch.empty((B, K), dtype=torch.float32, device=scores.device)
    _dev(out_ids, torch.int32, "out_ids")
    _dev(out_scores, torch.float32, "out_scores")
    rc = lib().pq_topk_scores(scores.data_ptr(), ld, N, B, K, out_ids.data_ptr(), out_scores.data_ptr(),
                              workspace.data_ptr(), workspace.numel(), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_topk_scores")
    return out_ids, out_scores


def pq_recjpq_scores(codes: torch.Tensor, S: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Algorithm 2 without its TopK: codes uint8 [N][m], S fp32 [B][m][b] -> scores fp32 [B][ld] (ld = N rounded up
    to a multiple of 4 when allocated here)."""
    _dev(codes, torch.uint8, "codes")
    _dev(S, torch.float32, "S")
    N, m = codes.shape
    B, m2, b = S.shape
    if m2 != m:
        raise PQError(PQ_ERR_SHAPE, "pq_recjpq_scores")
    if out is None:
        out = torch.empty((B, (N + 3) // 4 * 4), dtype=torch.float32, device=codes.device)
    _dev(out, torch.float32, "scores")
    rc = lib().pq_recjpq_scores(codes.data_ptr(), S.data_ptr(), N, B, m, b, out.data_ptr(), out.shape[1], _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_recjpq_scores")
    return out


def pq_reconstruct_items(codes: torch.Tensor, centroids: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 2: codes uint8 [N][m], centroids fp32 [m][b][d/m] -> W fp32 [N][d]."""
    _dev(codes, torch.uint8, "codes")
    _dev(centroids, torch.float32, "centroids")
    N, m = codes.shape
    m2, b, s = centroids.shape
    if m2 != m:
        raise PQError(PQ_ERR_SHAPE, "pq_reconstruct_items")
    if out is None:
        out = torch.empty((N, m * s), dtype=torch.float32, device=codes.device)
    _dev(out, torch.float32, "W")
    rc = lib().pq_reconstruct_items(codes.data_ptr(), centroids.data_ptr(), N, m * s, m, b, out.data_ptr(), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_reconstruct_items")
    return out


def pq_default_scores(W: torch.Tensor, queries: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 3: W fp32 [N][d], queries fp32 [B][d] -> scores fp32 [B][ld]."""
    _dev(W, torch.float32, "W")
    _dev(queries, torch.float32, "queries")
    N, d = W.shape
    B, d2 = queries.shape
    if d2 != d:
        raise PQError(PQ_ERR_SHAPE, "pq_default_scores")
    if out is None:
        out = torch.empty((B, (N + 3) // 4 * 4), dtype=torch.float32, device=W.device)
    _dev(out, torch.float32, "scores")
    rc = lib().pq_default_scores(W.data_ptr(), queries.data_ptr(), N, B, d, out.data_ptr(), out.shape[1], _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_default_scores")
    return out


def pq_score_topk_profile(codes: torch.Tensor, S: torch.Tensor, K: int, iters: int,
                          workspace: Optional[torch.Tensor] = None) -> float:
    """Mean duration (ms) of the catalogue scan kernel over `iters` calls, from HIP events on the stream."""
    N, B, m, b, workspace, out_ids, out_scores = _topk_args(codes, S, K, workspace, None, None)
    ms = ctypes.c_float(0.0)
    rc = lib().pq_score_topk_profile(codes.data_ptr(), S.data_ptr(), N, B, m, b, K, out_ids.data_ptr(),
                                     out_scores.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(),
                                     iters, ctypes.byref(ms))
    if rc != PQ_OK:
        raise PQError(rc, "pq_score_topk_profile")
    return float(ms.value)


def pq_read_bandwidth_profile(buf: torch.Tensor, iters: int) -> float:
    """Mean duration (ms) of a plain streaming-read kernel over the whole of `buf`."""
    if not buf.is_cuda or not buf.is_contiguous():
        raise ValueError("buf must be a contiguous device tensor")
    ms = ctypes.c_float(0.0)
    rc = lib().pq_read_bandwidth_profile(buf.data_ptr(), buf.numel() * buf.element_size(), _stream(), iters,
                                         ctypes.byref(ms))
    if rc != PQ_OK:
        raise PQError(rc, "pq_read_bandwidth_profile")
    return float(ms.value)


def pq_measure_empty_launch(blocks: int, threads: int, iters: int) -> float:
    """Mean cost (ms) of launching an empty kernel on that grid, back to back on the current stream."""
    ms = ctypes.c_float(0.0)
    rc = lib().pq_measure_empty_launch(blocks, threads, _stream(), iters, ctypes.byref(ms))
    if rc != PQ_OK:
        raise PQError(rc, "pq_measure_empty_launch")
    return float(ms.value)


def pq_measure_lds_gather(width: int, table_bytes: int, rounds: int, conflict_free: bool, blocks: int, threads: int,
                          iters: int, sink: torch.Tensor, copies: int = 1) -> float:
    """Mean duration (ms) of a launch in which every lane reads `rounds` words of `width` bytes from a table in LDS."""
    ms = ctypes.c_float(0.0)
    rc = lib().pq_measure_lds_gather(width, table_bytes, rounds, int(conflict_free), copies, blocks, threads, sink.data_ptr(),
                                     _stream(), iters, ctypes.byref(ms))
    if rc != PQ_OK:
        raise PQError(rc, "pq_measure_lds_gather")
    return float(ms.value)


PQ_SYNC_VARIANT_NAMES = ("empty", "fold_launch", "last_folds_fenced", "last_folds_relaxed", "last_folds_relaxed_2level",
                         "eq4_launch", "eq4_barrier_fenced", "eq4_barrier_relaxed")
PQ_SYNC_SCRATCH_BYTES = 2 << 20


def pq_measure_sync_variant(variant: int, scratch: torch.Tensor, iters: int) -> float:
    """Mean time (ms) per iteration of one of the in-launch synchronisation stand-ins (see pqtopk_measure.h)."""
    ms = ctypes.c_float(0.0)
    rc = lib().pq_measure_sync_variant(variant, scratch.data_ptr(), scratch.numel() * scratch.element_size(), _stream(),
                                       iters, ctypes.byref(ms))
    if rc != PQ_OK:
        raise PQError(rc, "pq_measure_sync_variant")
    return float(ms.value)


def pq_measure_force_general(mask: int) -> int:
    """Bit 0: scans avoid the short kernel; bit 1: folds avoid the small-K fold; bit 2: Eq. 4 avoids the matrix cores;
    0: the library's choice.  Returns the previous mask."""
    return int(lib().pq_measure_force_general(int(mask)))


PQ_STAMP_SLOTS, PQ_STAMP_RECORDS = 16, 8192


def pq_measure_step_stamps(queries: torch.Tensor, centroids: torch.Tensor, codes: torch.Tensor, K: int, S: torch.Tensor,
                           out_ids: torch.Tensor, out_scores: torch.Tensor, workspace: torch.Tensor,
                           stamps: torch.Tensor) -> Tuple[int, int]:
    """One step (Eq. 4, scan, fold) with the stamping instances of the kernels; `stamps` is an int64 device tensor of
    shape [3][PQ_STAMP_RECORDS][PQ_STAMP_SLOTS], zeroed by the caller.  Returns (scan workgroups, waves per workgroup)."""
    N, m = codes.shape
    B, d = queries.shape
    b = centroids.shape[1]
    grid = (ctypes.c_int * 2)()
    rc = lib().pq_measure_step_stamps(queries.data_ptr(), centroids.data_ptr(), codes.data_ptr(), N, B, d, m, b, K,
                                      S.data_ptr(), out_ids.data_ptr(), out_scores.data_ptr(), workspace.data_ptr(),
                                      workspace.numel(), stamps.data_ptr(), stamps.numel() * stamps.element_size(),
                                      ctypes.byref(grid), _stream())
    if rc != PQ_OK:
        raise PQError(rc, "pq_measure_step_stamps")
    return int(grid[0]), int(grid[1])


class _Prepared:
    """An entry point with its arguments marshalled once; calling the object only enqueues (for tight serving loops).
    The tensors are kept alive by the object; `stream` is a raw hipStream_t handle (default: torch's current stream at
    construction)."""

    def _prepare(self, entry: str, keep, result, stream: Optional[int], make_args):
        self._entry, self._keep, self._result = entry, keep, result
        self._fn = getattr(lib(), entry)
        self._args = make_args(ctypes.c_void_p(_stream() if stream is None else stream))

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != PQ_OK:
            raise PQError(rc, self._entry)
        return self._result


class PreparedSubitemScores(_Prepared):
    """pq_subitem_scores, marshalled once; returns S."""

    def __init__(self, queries: torch.Tensor, centroids: torch.Tensor, out: Optional[torch.Tensor] = None,
                 stream: Optional[int] = None):
        _dev(queries, torch.float32, "queries")
        _dev(centroids, torch.float32, "centroids")
        B, d = queries.shape
        m, b, s = centroids.shape
        if m * s != d:
            raise PQError(PQ_ERR_SHAPE, "pq_subitem_scores")
        self.S = out if out is not None else torch.empty((B, m, b), dtype=torch.float32, device=queries.device)
        _dev(self.S, torch.float32, "S")
        c = ctypes
        self._prepare("pq_subitem_scores", (queries, centroids), self.S, stream, lambda st: (
            c.c_void_p(queries.data_ptr()), c.c_void_p(centroids.data_ptr()), c.c_void_p(self.S.data_ptr()),
            c.c_int(B), c.c_int(d), c.c_int(m), c.c_int(b), st))


class PreparedScoreTopK(_Prepared):
    """pq_score_topk, marshalled once (workspace and outputs allocated here if not given); returns (ids, scores)."""
    _ENTRY, _WIDE = "pq_score_topk", False

    def __init__(self, codes: torch.Tensor, S: torch.Tensor, K: int, workspace: Optional[torch.Tensor] = None,
                 out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None,
                 stream: Optional[int] = None):
        N, B, m, b, workspace, out_ids, out_scores = _topk_args(codes, S, K, workspace, out_ids, out_scores, wide=self._WIDE)
        self.ids, self.scores, self.workspace = out_ids, out_scores, workspace
        c = ctypes
        self._prepare(self._ENTRY, (codes, S), (out_ids, out_scores), stream, lambda st: (
            c.c_void_p(codes.data_ptr()), c.c_void_p(S.data_ptr()), c.c_longlong(N), c.c_int(B), c.c_int(m),
            c.c_int(b), c.c_int(K), c.c_void_p(out_ids.data_ptr()), c.c_void_p(out_scores.data_ptr()),
            c.c_void_p(workspace.data_ptr()), c.c_size_t(workspace.numel()), st))


class PreparedScoreTopKU16(PreparedScoreTopK):
    """pq_score_topk_u16, marshalled once (same signature, uint16 codes)."""
    _ENTRY, _WIDE = "pq_score_topk_u16", True


class PreparedScoreTopKSubset(_Prepared):
    """pq_score_topk_subset, marshalled once (workspace and outputs allocated here if not given); returns (ids, scores)."""

    def __init__(self, codes: torch.Tensor, S: torch.Tensor, subset: torch.Tensor, K: int,
                 workspace: Optional[torch.Tensor] = None, stream: Optional[int] = None):
        n, N, B, m, b, workspace, self.ids, self.scores = _subset_args(codes, S, subset, K, workspace, None, None)
        self.workspace = workspace
        c = ctypes
        self._prepare("pq_score_topk_subset", (codes, S, subset), (self.ids, self.scores), stream, lambda st: (
            c.c_void_p(codes.data_ptr()), c.c_void_p(S.data_ptr()), c.c_void_p(subset.data_ptr()),
            c.c_longlong(n), c.c_longlong(N), c.c_int(B), c.c_int(m), c.c_int(b), c.c_int(K),
            c.c_void_p(self.ids.data_ptr()), c.c_void_p(self.scores.data_ptr()),
            c.c_void_p(workspace.data_ptr()), c.c_size_t(workspace.numel()), st))
