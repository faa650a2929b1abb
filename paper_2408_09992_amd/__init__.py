"""PQTopK scoring for sub-item-id (RecJPQ) recommendation models on MI355X (gfx950).

`workloads` draws the seeded synthetic inputs; the HIP path is reached through the names below, which load the
C-ABI library on first use and raise if it has not been built (there is no CPU fallback).
"""
from __future__ import annotations

__all__ = ["workloads", "pq_subitem_scores", "pq_score_topk", "pq_score_topk_workspace_bytes", "pq_score_topk_u16",
           "pq_score_topk_u16_workspace_bytes", "pq_score_topk_subset",
           "pq_score_topk_subset_workspace_bytes", "pq_topk_scores", "pq_topk_scores_workspace_bytes", "pq_recjpq_scores",
           "pq_reconstruct_items", "pq_default_scores", "pq_strerror"]


def __getattr__(name):
    if name in __all__[1:]:
        from . import binding
        return getattr(binding, name)
    if name in ("workloads", "binding", "build"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
