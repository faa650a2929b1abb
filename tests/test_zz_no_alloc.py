"""pq_score_topk_static(): the entry point that allocates nothing (its scratch is an array built into the library)
against pq_score_topk() on the same inputs, through the C ABI."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _call_pair(pq, torch, W, cfg_name, N, B, K):
    cfg = W.CONFIGS[cfg_name]
    G, cent, Q = W.make(cfg, B=B, N=N)
    Gd = torch.from_numpy(G).cuda()
    S = pq.pq_subitem_scores(torch.from_numpy(Q).cuda(), torch.from_numpy(cent).cuda())
    ref_ids, ref_sc = pq.pq_score_topk(Gd, S, K)
    ids = torch.full((B, K), -7, dtype=torch.int32, device="cuda")
    sc = torch.full((B, K), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    L = pq.lib()
    rc = L.pq_score_topk_static(Gd.data_ptr(), S.data_ptr(), N, B, cfg.m, cfg.b, K, ids.data_ptr(), sc.data_ptr(),
                                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, pq.pq_strerror(rc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert np.array_equal(ids.cpu().numpy(), ref_ids.cpu().numpy())
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), ref_sc.cpu().numpy().view(np.uint32))
    return G, cent, Q, ids.cpu().numpy(), sc.cpu().numpy()


def test_static_scratch_matches_workspace_call_twice_in_a_row(pq, oracle):
    import torch
    from paper_2408_09992_amd import workloads as W
    # a batch on the Gowalla-shaped workload first (many lists in the scratch), then a smaller single query: the second
    # call finds the first one's keys in the array and must not be disturbed by them
    G, cent, Q, ids, sc = _call_pair(pq, torch, W, "large", 400_000, 5, 100)
    rid, rsc = oracle.pqtopk(G, cent, Q, 100)
    assert np.array_equal(ids, rid) and np.array_equal(sc.view(np.uint32), rsc.view(np.uint32))
    G, cent, Q, ids, sc = _call_pair(pq, torch, W, "large", 50_001, 1, 10)
    rid, rsc = oracle.pqtopk(G, cent, Q, 10)
    assert np.array_equal(ids, rid) and np.array_equal(sc.view(np.uint32), rsc.view(np.uint32))
    # ... and the tiny configuration after that (another kernel instance, m = 4)
    G, cent, Q, ids, sc = _call_pair(pq, torch, W, "tiny", 10_000, 1, 10)
    rid, rsc = oracle.pqtopk(G, cent, Q, 10)
    assert np.array_equal(ids, rid) and np.array_equal(sc.view(np.uint32), rsc.view(np.uint32))


def test_static_scratch_rejects_what_does_not_fit(pq):
    import torch
    L = pq.lib()
    # 65535 queries x K = 512: far more partial lists than 8 MiB hold; rejected on the host, nothing enqueued
    N, B, m, b, K = 100_000, 60_000, 8, 256, 512
    assert pq.pq_score_topk_workspace_bytes(N, B, m, b, K) > pq.PQ_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    rc = L.pq_score_topk_static(dummy.data_ptr(), dummy.data_ptr(), N, B, m, b, K, dummy.data_ptr(), dummy.data_ptr(), None)
    assert rc == pq.PQ_ERR_TOO_LARGE
    assert "scratch" in pq.pq_strerror(rc)
