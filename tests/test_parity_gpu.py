"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.
Bar: item ids bit-exact (ties to the lower id), scores within 1e-5 relative (they are in fact bit-equal, and the
tests say so where they check it)."""
import numpy as np
import pytest
import torch

from paper_2408_09992_amd import workloads as W

pytestmark = pytest.mark.gpu

REL = 1e-5


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_scores(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.all(np.abs(got - ref) <= REL * np.maximum(np.abs(ref), 1.0))


def run_topk(pq, G, S, K):
    ids, sc = pq.pq_score_topk(dev(G), dev(S), K)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), sc.cpu().numpy()


def assert_same_topk(pq, oracle, G, S, K, tag=""):
    print(f"case {tag} N={G.shape[0]} m={G.shape[1]} B={S.shape[0]} b={S.shape[2]} K={K}", flush=True)
    ids, sc = run_topk(pq, G, S, K)
    rid, rsc = oracle.score_topk(G, S, K)
    assert np.array_equal(ids, rid), tag
    check_scores(sc, rsc)
    assert np.array_equal(sc.view(np.uint32), rsc.view(np.uint32)), tag      # stronger than the bar: same bits
    return ids, sc


# ---------------------------------------------------------------- Eq. 4

@pytest.mark.parametrize("B,d,m,b", [(1, 64, 4, 256), (1, 512, 8, 256), (5, 512, 16, 256), (3, 96, 3, 7),
                                     (2, 8, 8, 256), (64, 512, 8, 256), (2, 640, 5, 100), (1, 33, 1, 1),
                                     (9, 512, 8, 256), (70, 512, 16, 256), (17, 64, 4, 256), (33, 512, 8, 100),
                                     (1024, 512, 8, 256), (12, 96, 3, 7), (1, 768, 8, 256), (64, 768, 8, 256),
                                     (300, 1024, 8, 256), (3, 1536, 12, 256), (5, 72, 6, 100), (9, 40, 8, 256),
                                     (2, 768, 64, 256), (70, 768, 16, 256)])
def test_subitem_scores_bit_exact(pq, oracle, B, d, m, b):
    print(f"case subitem B={B} d={d} m={m} b={b}", flush=True)
    cent = W.centroids(m, b, d, seed=B + d)
    Q = W.queries(B, d, seed=B + d)
    S = pq.pq_subitem_scores(dev(Q), dev(cent))
    torch.cuda.synchronize()
    ref = oracle.subitem_scores(Q, cent)
    got = S.cpu().numpy()
    check_scores(got, ref)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


# ---------------------------------------------------------------- Algorithm 1, small shapes, several tiles + ragged tails

@pytest.mark.parametrize("B,d,m,b", [(1024, 512, 8, 256), (449, 512, 16, 256), (470, 768, 16, 256), (500, 1024, 8, 256),
                                     (600, 768, 8, 256), (529, 128, 8, 100), (460, 512, 8, 1000), (512, 64, 4, 256),
                                     (457, 2048, 8, 7), (3000, 96, 6, 70)])
def test_subitem_scores_on_the_matrix_cores(pq, oracle, B, d, m, b):
    # batches large enough for the matrix-core kernel (chains of K = 1 fp32 matrix instructions): the same bits as the
    # oracle's fused chain, the same bits as the scalar kernels (measurement hook), also with denormal products and
    # with magnitudes that differ by many orders inside one chain; ragged batches, alphabets that are no multiple of
    # 64, chunks of 16, 32 and 64 elements, several chunks per chain
    print(f"case subitem mfma B={B} d={d} m={m} b={b}", flush=True)
    for scale_c, scale_q in ((1.0, 1.0), (1e-21, 1e-19), (1e8, 1e-3)):
        cent = (W.centroids(m, b, d, seed=B + d) * scale_c).astype(np.float32)
        Q = (W.queries(B, d, seed=B + d) * scale_q).astype(np.float32)
        if scale_c == 1e8:
            cent[:, :, ::3] *= 1e-12                               # alternating magnitudes along the chain
        got = pq.pq_subitem_scores(dev(Q), dev(cent))
        prev = pq.pq_measure_force_general(4)
        try:
            scalar = pq.pq_subitem_scores(dev(Q), dev(cent))
        finally:
            pq.pq_measure_force_general(prev)
        torch.cuda.synchronize()
        ref = oracle.subitem_scores(Q, cent)
        assert np.array_equal(got.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (scale_c, scale_q)
        assert torch.equal(got.view(torch.int32), scalar.view(torch.int32)), (scale_c, scale_q)


@pytest.mark.parametrize("m", [1, 2, 3, 4, 8, 16, 32, 64])
def test_score_topk_small_shapes(pq, oracle, m):
    for N in (1, 2, 5, 63, 64, 65, 127, 1000, 4099, 70_001):
        for b in (256, 16):
            for B in (1, 3):
                G = W.codes_uniform(N, m, b, seed=N + m)
                S = W.normal_f32(W.stream_key(N + m, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
                for K in sorted({1, min(N, 10), min(N, 100)}):
                    assert_same_topk(pq, oracle, G, S, K, "small")


def test_score_topk_large_k(pq, oracle):
    for N, m, K in ((5000, 8, 512), (3000, 4, 500), (512, 16, 512), (200_000, 8, 257), (100_000, 64, 512), (50_000, 128, 64)):
        G = W.codes_uniform(N, m, 256, seed=K)
        S = W.normal_f32(W.stream_key(K, W.STREAM_QUERIES), 2 * m * 256).reshape(2, m, 256)
        assert_same_topk(pq, oracle, G, S, K, "largeK")


def test_score_topk_single_query_mid_k(pq, oracle):
    """K around the sizes at which paths change (lists cut back early up to K = 12 in the batched kernel, the fold of
    256 lists in one 512-thread workgroup up to K = 24, in one 1024-thread workgroup up to K = 52, in two levels
    above), one query, several rounds per workgroup and a ragged tail."""
    for N, m in ((1_500_001, 8), (700_003, 4), (300_001, 16)):
        G = W.codes_uniform(N, m, 256, seed=N)
        S = W.normal_f32(W.stream_key(N, W.STREAM_QUERIES), m * 256).reshape(1, m, 256)
        for K in (12, 13, 24, 25, 28, 29, 50, 52, 53, 64, 65):
            assert_same_topk(pq, oracle, G, S, K, "midK")


@pytest.mark.parametrize("N,m,B,K", [(1_280_000, 8, 1, 400), (1_280_000, 8, 1, 512), (1_280_000, 8, 3, 52), (1_280_000, 8, 4, 100),
                                     (600_001, 4, 2, 300), (1_280_000, 8, 1, 350)])
def test_score_topk_fold_levels(pq, oracle, N, m, B, K):
    """Folds of more keys than one 512-thread workgroup holds: one 1024-thread workgroup (up to 13,312 keys), groups of
    lists side by side and a second level, and a second level that is itself a 1024-thread fold (K = 400, 512)."""
    G = W.codes_uniform(N, m, 256, seed=K)
    S = W.normal_f32(W.stream_key(N + K, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    assert_same_topk(pq, oracle, G, S, K, "fold-levels")
    # heavy ties: the wide fold's staged fallback
    Sc = (np.round(S * 2) / 2).astype(np.float32)
    assert_same_topk(pq, oracle, G, Sc, K, "fold-levels-coarse")


@pytest.mark.parametrize("N,m,B,K", [(40_000_003, 4, 1, 10), (30_000_001, 8, 2, 10), (18_000_001, 16, 1, 100),
                                     (4_500_001, 64, 1, 10), (20_000_001, 3, 1, 10), (70_000_001, 2, 1, 64)])
def test_score_topk_many_rounds(pq, oracle, N, m, B, K):
    """Scans of sixteen or more rounds per workgroup, for the replicated-table, plain, wide-item and generic kernels:
    the streaming loop with work units taken from the counter in LDS runs long, and the last item sits in the last,
    ragged round."""
    assert pq.pq_score_topk_workspace_bytes(N, B, m, 256, K) % 256 == 0
    G = W.codes_uniform(N, m, 256, seed=m + B)
    S = W.normal_f32(W.stream_key(N, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    assert_same_topk(pq, oracle, G, S, K, "many-rounds")
    G[N - 1] = S[B - 1].argmax(axis=1)                 # the very last item wins for the last query
    ids, _ = assert_same_topk(pq, oracle, G, S, K, "many-rounds+last")
    if m >= 4:
        assert ids[B - 1][0] == N - 1


@pytest.mark.parametrize("N,m,B,K", [(30_000_001, 8, 1, 512), (20_000_003, 4, 2, 200), (12_000_001, 16, 1, 300),
                                     (9_000_001, 8, 3, 100), (3_000_001, 64, 1, 100), (8_000_001, 5, 1, 64)])
def test_score_topk_long_scans_at_larger_k(pq, oracle, N, m, B, K):
    """Single-query scans of six or more rounds with K > 28: the waves share a floor from the running histogram."""
    G = W.codes_uniform(N, m, 256, seed=m + K)
    S = W.normal_f32(W.stream_key(N + K, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    assert_same_topk(pq, oracle, G, S, K, "long-scan-K")


@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_long_monotone_scan_at_larger_k(pq, oracle, sign):
    """score == +-id over 16.7M items at K = 100: ascending, every item beats everything before it (all of them pass
    any floor and the lists overflow over and over); descending, nothing after the first K does.  Then a coarse table:
    a handful of distinct scores, so whole buckets of the running histogram tie."""
    N, m = 16_700_000, 4
    i = np.arange(N, dtype=np.int64)
    G = np.stack([(i >> (8 * k)) & 255 for k in range(m)], axis=1).astype(np.uint8)
    S = np.zeros((1, m, 256), dtype=np.float32)
    for k in range(3):
        S[0, k] = sign * np.arange(256, dtype=np.float32) * (256.0 ** k)
    ids, _ = assert_same_topk(pq, oracle, G, S, 100, "long monotone")
    assert ids[0].tolist() == (list(range(N - 1, N - 101, -1)) if sign > 0 else list(range(100)))
    Sc = (np.round(W.normal_f32(W.stream_key(5, W.STREAM_QUERIES), m * 256) * 2) / 2).astype(np.float32).reshape(1, m, 256)
    assert_same_topk(pq, oracle, G, Sc, 100, "long coarse")


def test_long_scan_with_late_outliers_and_tiny_ranges(pq, oracle):
    """Shared floors under score distributions the first round does not announce: a few hundred items far above the
    first round's range, all of them late in the catalogue (they land in the histogram's top bucket); and tables of
    denormal entries (the range is too small for a histogram: every score is a candidate)."""
    N, m, K = 12_000_001, 8, 100
    G = W.codes_uniform(N, m, 255, seed=21)                       # sub-id 255 of split 0 is never drawn ...
    S = W.normal_f32(W.stream_key(21, W.STREAM_QUERIES), m * 256).reshape(1, m, 256)
    S[0, 0, 255] = 1.0e6                                          # ... and is worth a million
    late = N - 1 - W.plant_ids(N // 10, 300, seed=3)              # 300 distinct ids in the last tenth
    G[late, 0] = 255
    ids, sc = assert_same_topk(pq, oracle, G, S, K, "late outliers")
    assert set(ids[0].tolist()) <= set(late.tolist()) and sc[0].min() > 9.0e5
    ids, _ = assert_same_topk(pq, oracle, G, S, 10, "late outliers K=10")
    assert set(ids[0].tolist()) <= set(late.tolist())
    Sd = (np.abs(S) * np.float32(1e-41)).astype(np.float32)       # denormals: 0 .. ~4e-41
    Sd[0, 0, 255] = 0.0
    assert Sd.max() < 1.2e-38 and Sd.max() > 0
    assert_same_topk(pq, oracle, G[:3_000_001], Sd, 50, "denormal tables")


def test_subset_long_list(pq, oracle):
    N, m = 20_000_000, 8
    G = W.codes_uniform(N, m, 256, seed=9)
    S = W.normal_f32(W.stream_key(9, W.STREAM_QUERIES), m * 256).reshape(1, m, 256)
    V = W.candidate_list(N, 17_000_001, seed=2)
    assert_same_subset_topk(pq, oracle, G, S, V, 10, "subset-long")


@pytest.mark.parametrize("N,m,B", [(17_000_003, 4, 1), (17_000_001, 2, 1), (34_000_001, 1, 1), (6_000_001, 4, 3)])
def test_score_topk_long_scans_replicated_tables(pq, oracle, N, m, B):
    """Catalogues long enough for the single-query kernel that keeps several copies of the score tables in LDS
    (1024-thread workgroups, work handed to waves from a counter), for every m it is built for; N leaves a tail
    of items after the last whole 16-byte code vector.  m = 8 is covered by the 50M-item configuration."""
    G = W.codes_uniform(N, m, 256, seed=m)
    S = W.normal_f32(W.stream_key(m, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    ids, sc = assert_same_topk(pq, oracle, G, S, 10, "long")
    # the last item wins when it is given the best row: the tail after the last whole vector is really scanned
    G[N - 1] = S[0].argmax(axis=1)
    ids, sc = assert_same_topk(pq, oracle, G, S, 10, "long+tail")
    if m >= 4:                                     # (with fewer splits thousands of items share the best row: lower ids win)
        assert ids[0, 0] == N - 1


# ---------------------------------------------------------------- ties and adversarial orders

@pytest.mark.parametrize("N,m,B,K", [(1_000_003, 64, 1, 10), (600_001, 64, 2, 100), (2_000_001, 32, 1, 10),
                                     (300_000, 64, 3, 10), (150_001, 64, 1, 300), (5_000_000, 32, 1, 64)])
def test_score_topk_wide_items(pq, oracle, N, m, B, K):
    # m = 32, 64: one item spans two or four code vectors; long m = 64 scans run 1024-thread workgroups
    G = W.codes_uniform(N, m, 256, seed=m)
    S = W.normal_f32(W.stream_key(N, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    assert_same_topk(pq, oracle, G, S, K, "wide")


@pytest.mark.parametrize("N,m,B,K,b", [(700_001, 8, 64, 10, 256), (700_002, 8, 65, 1, 256), (700_003, 8, 66, 100, 256),
                                       (350_001, 16, 67, 10, 256), (350_000, 16, 64, 512, 256),
                                       (1_400_000, 8, 33, 300, 256), (700_005, 8, 64, 10, 16), (2_000_003, 16, 13, 28, 256),
                                       (300_007, 8, 48, 10, 256), (300_009, 8, 96, 10, 256), (200_003, 8, 384, 10, 256),
                                       (200_005, 8, 383, 100, 256), (150_001, 16, 1100, 10, 256)])
def test_score_topk_batched_kernel_shapes(pq, oracle, N, m, B, K, b):
    # B * N * m is large enough for the four-queries-per-workgroup kernel: ragged ends of the catalogue, partly filled
    # tiles, the K range, a short code alphabet, and batches whose tiles share the CUs unevenly (21, 10 or 5 item
    # blocks per tile; more tiles than CUs)
    G = W.codes_uniform(N, m, b, seed=B)
    S = W.normal_f32(W.stream_key(N + B, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
    assert_same_topk(pq, oracle, G, S, K, "batched")


@pytest.mark.parametrize("N,m,B,K", [(300_001, 64, 17, 10), (200_003, 64, 40, 100), (150_001, 64, 100, 10), (300_005, 4, 100, 10),
                                     (100_003, 4, 1024, 100), (200_001, 32, 100, 10), (150_007, 5, 100, 10), (120_001, 48, 40, 10),
                                     (100_001, 64, 300, 10)])
def test_score_topk_many_queries_side_by_side(pq, oracle, N, m, B, K):
    # batches that run as B single-query scans with few item blocks each: 15, 6, 5 or 2 blocks per query, one block
    # per query, 1024-thread workgroups for the large tables
    G = W.codes_uniform(N, m, 256, seed=B + m)
    S = W.normal_f32(W.stream_key(N + B, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    assert_same_topk(pq, oracle, G, S, K, "side-by-side")


@pytest.mark.parametrize("N,m,b,B,K", [(300, 8, 256, 2000, 10), (40, 16, 256, 5000, 40), (5000, 8, 1, 7, 50),
                                       (1_200_000, 128, 256, 1, 10), (900, 4, 256, 65535, 1)])
def test_score_topk_odd_corners(pq, oracle, N, m, b, B, K):
    # thousands of queries over a tiny catalogue (one workgroup per query), K = N, a single sub-id per split, the largest
    # m on a scan long enough for 1024-thread workgroups, the largest batch
    G = W.codes_uniform(N, m, b, seed=N)
    S = W.normal_f32(W.stream_key(N + B, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
    assert_same_topk(pq, oracle, G, S, K, "corner")


def test_score_topk_seeded_random_shapes(pq, oracle):
    # a seeded walk through shape space: every m from 1 to 20 plus the wide ones, short alphabets, odd batch sizes,
    # K anywhere up to min(N, 512), with and without a candidate list
    rng = np.random.default_rng(20240819)
    for case in range(160):
        m = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16, 20, 32, 64]))
        b = int(rng.choice([1, 2, 7, 16, 100, 255, 256]))
        N = int(rng.choice([1, 2, 17, 64, 255, 1000, 4097, 20_000]))
        B = int(rng.integers(1, 10))
        K = int(rng.integers(1, min(N, 512) + 1))
        G = W.codes_uniform(N, m, b, seed=case)
        S = W.normal_f32(W.stream_key(case, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
        if rng.random() < 0.3:                              # coarse tables: many exact ties
            S = np.round(S * 2).astype(np.float32) / 2
        assert_same_topk(pq, oracle, G, S, K, f"random#{case}")
        if case % 4 == 0:
            n = int(rng.integers(K, N + 1))
            V = W.candidate_list(N, n, seed=case)
            assert_same_subset_topk(pq, oracle, G, S, V, K, f"random-subset#{case}")


def test_seeded_random_shapes_larger_catalogues_and_wide_codes(pq, oracle):
    # a second seeded walk: catalogues of 10^5 to 3*10^6 items (several rounds per workgroup, every kernel instance and
    # both folds), one- and two-byte sub-ids, K at the values where paths change, duplicated rows and coarse tables
    rng = np.random.default_rng(20240820)
    for case in range(60):
        wide = rng.random() < 0.35
        m = int(rng.choice([1, 2, 3, 4, 5, 8, 8, 8, 12, 16, 16, 32, 64]))
        b = int(rng.choice([257, 1000, 4096, 9000, 65536])) if wide else int(rng.choice([16, 255, 256, 256]))
        N = int(10 ** rng.uniform(5.0, 6.5))
        B = int(rng.choice([1, 1, 2, 3, 5, 8, 24, 33, 64]))
        if N * m * B > 2.5e8:
            B = max(1, int(2.5e8 // (N * m)))
        K = int(rng.choice([1, 10, 10, 12, 13, 28, 29, 52, 53, 64, 100, 192, 193, 300, 512]))
        G = (W.codes_uniform_u16 if wide else W.codes_uniform)(N, m, b, seed=case)
        if rng.random() < 0.3:                              # a tenth of the rows copied from elsewhere: exact ties
            idx, src = rng.integers(0, N, size=N // 10), rng.integers(0, N, size=N // 10)
            G[idx] = G[src]
        S = W.normal_f32(W.stream_key(1000 + case, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
        if rng.random() < 0.3:
            S = np.round(S * 2).astype(np.float32) / 2
        (assert_same_topk_u16 if wide else assert_same_topk)(pq, oracle, G, S, K, f"random2#{case}")


def test_score_topk_largest_catalogue(pq, oracle):
    # N = 2^31 - 1, the largest the interface takes (m = 1: 2 GB of codes): every index computation at its limit,
    # with the winner planted as the very last item
    N, m, K = 2 ** 31 - 1, 1, 10
    G = np.empty((N, m), dtype=np.uint8)
    step = 1 << 26
    for a0 in range(0, N, step):                              # a cheap seeded pattern, drawn in chunks
        idx = np.arange(a0, min(a0 + step, N), dtype=np.uint64)
        G[a0:a0 + len(idx), 0] = ((idx * np.uint64(0x9E3779B97F4A7C15)) >> np.uint64(56)).astype(np.uint8)
    S = W.normal_f32(W.stream_key(31, W.STREAM_QUERIES), m * 256).reshape(1, m, 256)
    best = int(S[0, 0].argmax())
    G[G[:, 0] == best, 0] = (best + 1) % 256                  # nobody holds the best sub-id ...
    G[N - 1, 0] = best                                        # ... except the last item
    ids, sc = assert_same_topk(pq, oracle, G, S, K, "largest")
    assert ids[0][0] == N - 1


def test_billion_items_of_64_splits(pq, oracle):
    # the far end of the catalogue-size sweep (Section 5: up to 10^9 items, m = 64): 64 GB of codes drawn on the device,
    # byte offsets far beyond 2^32.  No oracle run over that; instead four planted rows (the best sub-id of every
    # split, and with the first one, two, three splits on their second-best) at the last item, just past a 2^32-byte
    # boundary, in the middle and near the start must come back first, in that order, with the oracle's scores
    N, m, K = 1_000_000_000, 64, 10
    Gd = W.codes_uniform_device(N, m, 256, seed=9)
    S = tables(64, 1, m, 256)
    best = S[0].argmax(axis=1).astype(np.uint8)
    second = np.argsort(S[0], axis=1)[:, -2].astype(np.uint8)
    places = [N - 1, (1 << 26) + 5, N // 2 + 1, 3]
    rows = np.stack([best] * 4)
    for j in range(1, 4):
        rows[j, :j] = second[:j]
    for i, row in zip(places, rows):
        Gd[i] = torch.from_numpy(row).cuda()
    ids, sc = pq.pq_score_topk(Gd, dev(S), K)
    torch.cuda.synchronize()
    want = oracle.item_scores(rows, S[0])
    assert want[0] > want[1] > want[2] > want[3]
    assert ids.cpu().numpy()[0, :4].tolist() == places
    assert np.array_equal(sc.cpu().numpy()[0, :4].view(np.uint32), want.view(np.uint32))
    assert float(sc[0, 4]) < 0.5 * float(want[3])           # (random rows score far below)
    del Gd
    torch.cuda.empty_cache()


def test_all_items_equal(pq, oracle):
    for N in (500, 100_000):
        G = np.full((N, 8), 17, dtype=np.uint8)
        S = W.normal_f32(W.stream_key(1, W.STREAM_QUERIES), 8 * 256).reshape(1, 8, 256)
        ids, _ = assert_same_topk(pq, oracle, G, S, 25, "all-equal")
        assert ids[0].tolist() == list(range(25))


def test_short_scans_with_larger_k_select_from_registers(pq, oracle):
    # at most two rounds per workgroup and K >= 32: one selection over all the workgroup's scores; every item equal
    # (the cut bucket holds them all: back to the lists), a last odd item that wins, and one- and two-byte sub-ids
    for N in (100_001, 1_280_001):
        G = np.full((N, 8), 9, dtype=np.uint8)
        S = W.normal_f32(W.stream_key(N, W.STREAM_QUERIES), 8 * 256).reshape(1, 8, 256)
        ids, _ = assert_same_topk(pq, oracle, G, S, 64, "short all-equal")
        assert ids[0].tolist() == list(range(64))
        G = W.codes_uniform(N, 8, 256, seed=N)
        G[N - 1] = S[0].argmax(axis=1)                         # the item after the last whole code vector is the best
        ids, _ = assert_same_topk(pq, oracle, G, S, 100, "short last-wins")
        assert ids[0][0] == N - 1
        G16 = W.codes_uniform_u16(N, 4, 1000, seed=N)          # rows of 8 bytes: N odd leaves one item after the vectors
        S16 = tables(N, 2, 4, 1000)
        G16[N - 1] = S16[1].argmax(axis=1)
        ids, _ = assert_same_topk_u16(pq, oracle, G16, S16, 50, "short last-wins u16")
        assert ids[1][0] == N - 1


@pytest.mark.parametrize("m", [1, 2, 4, 8, 16, 32, 64])
def test_short_scan_every_number_of_units_per_thread(pq, oracle, m):
    # single-query scans whose workgroups hold their whole share in registers (the short kernel) take a kernel instance
    # per number of units a thread holds; catalogue sizes that land on each of them, odd so that the last slot is ragged
    # and items follow the last whole code vector; K = 1, 10 and 31 (the largest the short kernel and small fold take)
    unit_items = 16 // m if m <= 16 else 1
    max_units = {1: 2, 2: 2, 4: 6, 8: 12, 16: 12, 32: 8, 64: 4}[m]
    S = tables(m, 1, m, 256)
    for units in range(1, max_units + 1):
        N = (units - 1) * 256 * 512 * unit_items + 77_001 * unit_items + 3
        G = W.codes_uniform(N, m, 256, seed=units + m)
        G[N - 1] = S[0].argmax(axis=1)                         # the last item (after the last whole vector) is the best
        for K in (1, 10, 31):
            ids, _ = assert_same_topk(pq, oracle, G, S, K, f"short units={units}")
            if m >= 4:                                             # (fewer splits: other items share its row, lower ids first)
                assert ids[0][0] == N - 1


def test_short_scan_and_small_fold_against_the_general_kernels(pq, oracle):
    # the same calls through the general scan and fold kernels (measurement hook) give the same bits; heavy ties take
    # the short kernel's slow path (more candidates than its array holds): all items equal, coarse tables, -0 tables
    cases = []
    N = 1_280_000
    cases.append((W.codes_uniform(N, 8, 256, seed=5), tables(5, 1, 8, 256), 10, "headline shape"))
    cases.append((np.full((300_001, 8), 3, dtype=np.uint8), tables(6, 1, 8, 256), 31, "all equal"))
    coarse = (np.round(tables(7, 1, 4, 16) * 2) / 2).astype(np.float32)
    cases.append((W.codes_uniform(900_001, 4, 16, seed=7), coarse, 20, "coarse tables"))
    zeros = np.zeros((2, 8, 256), dtype=np.float32)
    zeros[:, ::2] = -0.0
    cases.append((W.codes_uniform(200_003, 8, 256, seed=8), zeros, 7, "zero tables"))
    cases.append((W.codes_uniform(31, 8, 256, seed=9), tables(9, 3, 8, 256), 31, "K = N"))
    cases.append((W.codes_uniform(5, 16, 256, seed=10), tables(10, 1, 16, 256), 2, "one code vector"))
    for G, S, K, tag in cases:
        ids, sc = assert_same_topk(pq, oracle, G, S, K, tag)
        for mask in (1, 2, 3):
            prev = pq.pq_measure_force_general(mask)
            try:
                ids2, sc2 = run_topk(pq, G, S, K)
            finally:
                pq.pq_measure_force_general(prev)
            assert np.array_equal(ids, ids2) and np.array_equal(sc.view(np.uint32), sc2.view(np.uint32)), (tag, mask)


@pytest.mark.parametrize("B", [2, 5, 64, 257, 1024])
def test_short_scans_side_by_side(pq, oracle, B):
    # batches of short scans in one launch (grid.y = B): the grid is spread over the CUs by B, so the number of
    # workgroups per query (256 / B, at least one) and of code vectors per thread change with it; m = 8, 4 and 64
    for N, m, K in ((3_001, 8, 10), (40_001, 8, 31), (9_001, 4, 1), (2_003, 64, 5)):
        G = W.codes_uniform(N, m, 256, seed=B + m)
        assert_same_topk(pq, oracle, G, tables(N + B, B, m, 256), K, "short side by side")


def test_small_fold_many_lists(pq, oracle):
    # the small-K fold with both of its instances: up to 3072 and up to 6144 keys per query (256 lists of K = 10, 24; with
    # K = 28, 31 the 256 lists go to the general fold: a third instance of 16 keys per thread was slower than it),
    # a batch of queries folded side by side, and lists with empty slots (fewer than K items in a workgroup's share)
    for N, B, K in ((1_280_000, 1, 24), (2_000_003, 2, 12), (1_280_001, 2, 31), (300, 1, 10), (70_000, 5, 31),
                    (1_280_000, 1, 31), (1_280_003, 1, 28)):
        G = W.codes_uniform(N, 8, 256, seed=N % 97)
        assert_same_topk(pq, oracle, G, tables(N % 89, B, 8, 256), K, "small fold")


def test_coarse_tables_many_ties(pq, oracle):
    G = W.codes_uniform(300_000, 4, 16, seed=3)
    S = (np.round(W.normal_f32(W.stream_key(3, W.STREAM_QUERIES), 2 * 4 * 16) * 2) / 2).astype(np.float32)
    assert_same_topk(pq, oracle, G, S.reshape(2, 4, 16), 100, "coarse")


def test_batched_kernel_heavy_ties_at_larger_k(pq, oracle):
    # the four-queries-per-workgroup kernel with K = 100 (lists cut by the final floors before the merge): coarse
    # tables (few distinct scores, ties everywhere), every item equal, and a monotone table
    N, m, B = 700_001, 8, 64
    G = W.codes_uniform(N, m, 16, seed=9)
    S = (np.round(W.normal_f32(W.stream_key(9, W.STREAM_QUERIES), B * m * 16) * 2) / 2).astype(np.float32).reshape(B, m, 16)
    assert_same_topk(pq, oracle, G, S, 100, "batched coarse")
    G = np.full((N, m), 7, dtype=np.uint8)
    ids, _ = assert_same_topk(pq, oracle, G, W.normal_f32(W.stream_key(10, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256), 100,
                              "batched all-equal")
    assert all(row.tolist() == list(range(100)) for row in ids)
    G = digits_codes(N, m)
    S = np.zeros((B, m, 256), dtype=np.float32)
    for q in range(B):
        for k in range(3):
            S[q, k] = (1.0 if q % 2 else -1.0) * np.arange(256, dtype=np.float32) * (256.0 ** k)
    ids, _ = assert_same_topk(pq, oracle, G, S, 100, "batched monotone")
    assert ids[0].tolist() == list(range(100)) and ids[1].tolist() == list(range(N - 1, N - 101, -1))


def digits_codes(N, m):
    i = np.arange(N, dtype=np.int64)
    return np.stack([(i >> (8 * k)) & 255 for k in range(m)], axis=1).astype(np.uint8)


@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_monotone_scores(pq, oracle, sign):
    """score == +-id exactly: ascending order makes every item beat the running threshold (worst case for the
    candidate lists), descending makes none after the first K."""
    N, m = 300_000, 4
    G = digits_codes(N, m)
    S = np.zeros((1, m, 256), dtype=np.float32)
    for k in range(3):
        S[0, k] = sign * np.arange(256, dtype=np.float32) * (256.0 ** k)
    ids, sc = assert_same_topk(pq, oracle, G, S, 100, "monotone")
    expect = np.arange(N - 1, N - 101, -1) if sign > 0 else np.arange(100)
    assert ids[0].tolist() == expect.tolist()


def test_negative_zero_tables(pq, oracle):
    S = np.full((1, 2, 256), -0.0, dtype=np.float32)
    S[0, 0, 1] = 0.0
    G = W.codes_uniform(1000, 2, 2, seed=4)
    ids, sc = assert_same_topk(pq, oracle, G, S, 50, "negzero")
    assert ids[0].tolist() == list(range(50)) and not np.signbit(sc).any()


def test_duplicates_and_straddle(pq, oracle):
    cfg = W.CONFIGS["finer"]
    N, K = 400_000, cfg.K
    G, cent, Q = W.make(cfg, B=4, N=N)
    S = pq.pq_subitem_scores(dev(Q), dev(cent)).cpu().numpy()
    planted = W.plant_ids(N, K + 3, seed=1)
    W.plant_rows(G, planted, S[0].argmax(axis=1))
    ids, sc = assert_same_topk(pq, oracle, G, S, K, "dup+straddle")
    assert ids[0].tolist() == planted[:K].tolist()


def test_deterministic_and_workspace_reuse(pq, oracle):
    cfg = W.CONFIGS["large"]
    G, cent, Q = W.make(cfg, B=2, N=300_000)
    Gd, Sd = dev(G), pq.pq_subitem_scores(dev(Q), dev(cent))
    need = pq.pq_score_topk_workspace_bytes(G.shape[0], 2, cfg.m, cfg.b, cfg.K)
    ws = torch.full((need,), 0xAB, dtype=torch.uint8, device="cuda")          # dirty workspace on purpose
    a = pq.pq_score_topk(Gd, Sd, cfg.K, workspace=ws)
    a = (a[0].clone(), a[1].clone())
    ws.fill_(0x5C)
    b2 = pq.pq_score_topk(Gd, Sd, cfg.K, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b2[0]) and torch.equal(a[1], b2[1])
    rid, _ = oracle.score_topk(G, Sd.cpu().numpy(), cfg.K)
    assert np.array_equal(a[0].cpu().numpy(), rid)


def test_side_streams_and_concurrent_calls(pq, oracle):
    # two calls in flight on two streams, each with its own workspace and outputs: the library keeps no state between
    # calls, so both must equal what the oracle says
    cfg = W.CONFIGS["large"]
    G, cent, Q = W.make(cfg, B=2, N=400_000)
    Gd = dev(G)
    S = pq.pq_subitem_scores(dev(Q), dev(cent))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for rep in range(3):
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                outs.append((i, pq.pq_score_topk(Gd, S[i:i + 1].contiguous(), cfg.K)))
    torch.cuda.synchronize()
    rid, rsc = oracle.score_topk(G, S.cpu().numpy(), cfg.K)
    for i, (ids, sc) in outs:
        assert np.array_equal(ids.cpu().numpy()[0], rid[i])
        assert np.array_equal(sc.cpu().numpy()[0].view(np.uint32), rsc[i].view(np.uint32))


@pytest.mark.parametrize("N,m,B", [(100_000, 8, 1), (100_000, 3, 2), (50_000, 64, 1), (700_001, 8, 64)])
def test_tables_that_are_only_four_byte_aligned(pq, oracle, N, m, B):
    # S may sit at any 4-byte boundary (the table fill then copies element by element, or loads unaligned)
    G = W.codes_uniform(N, m, 256, seed=m)
    S = W.normal_f32(W.stream_key(N + m, W.STREAM_QUERIES), B * m * 256).reshape(B, m, 256)
    flat = torch.empty(S.size + 1, dtype=torch.float32, device="cuda")
    Sd = flat[1:].view(B, m, 256)
    Sd.copy_(torch.from_numpy(S))
    assert Sd.data_ptr() % 16 == 4 and Sd.is_contiguous()
    ids, sc = pq.pq_score_topk(dev(G), Sd, 10)
    torch.cuda.synchronize()
    rid, rsc = oracle.score_topk(G, S, 10)
    assert np.array_equal(ids.cpu().numpy(), rid)
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), rsc.view(np.uint32))


def test_errors_reach_python(pq):
    G = dev(W.codes_uniform(100, 8))
    S = dev(np.zeros((1, 8, 256), dtype=np.float32))
    with pytest.raises(pq.PQError) as e:
        pq.pq_score_topk(G, S, 101)
    assert e.value.code == pq.PQ_ERR_SHAPE
    with pytest.raises(pq.PQError) as e:
        pq.pq_score_topk(G, S, 10, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == pq.PQ_ERR_WORKSPACE


# ---------------------------------------------------------------- Algorithm 1 over 16-bit sub-ids (b up to 65536)

def tables(seed, B, m, b):
    return W.normal_f32(W.stream_key(seed, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)


def assert_same_topk_u16(pq, oracle, G, S, K, tag=""):
    print(f"case u16 {tag} N={G.shape[0]} m={G.shape[1]} B={S.shape[0]} b={S.shape[2]} K={K}", flush=True)
    assert G.dtype == np.uint16
    ids, sc = pq.pq_score_topk_u16(dev(G), dev(S), K)
    torch.cuda.synchronize()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    rid, rsc = oracle.score_topk_u16(G, S, K)
    assert np.array_equal(ids, rid), tag
    check_scores(sc, rsc)
    assert np.array_equal(sc.view(np.uint32), rsc.view(np.uint32)), tag
    return ids, sc


@pytest.mark.parametrize("m,b", [(4, 8192), (8, 1024), (8, 4096), (16, 2048), (4, 300)])
def test_u16_short_scan_every_number_of_units_per_thread(pq, oracle, m, b):
    # two-byte sub-ids, K < 32, a share per thread that fits its registers: the short kernel with the table in dynamic
    # LDS, an instance per number of units a thread holds (code vectors; items of two vectors for m = 16); catalogue
    # sizes that land on each, odd so that the last slot is ragged (and, for rows of 8 bytes, an item follows the last
    # whole vector); the last item planted as the winner; against the oracle and against the general kernel's bits
    unit_items = 2 if m == 4 else 1
    max_units = 6 if m == 16 else 12
    S = tables(m + b, 1, m, b)
    for units in (1, 2, 3, 5, 6, 7, 9, 12):
        if units > max_units:
            continue
        N = (units - 1) * 256 * 512 * unit_items + 50_001 * unit_items
        G = W.codes_uniform_u16(N, m, b, seed=units + m)
        G[N - 1] = S[0].argmax(axis=1)
        for K in (1, 10, 31):
            ids, sc = assert_same_topk_u16(pq, oracle, G, S, K, f"u16 short units={units}")
            assert ids[0][0] == N - 1
        prev = pq.pq_measure_force_general(1)
        try:
            ids2, sc2 = pq.pq_score_topk_u16(dev(G), dev(S), 31)
            torch.cuda.synchronize()
        finally:
            pq.pq_measure_force_general(prev)
        assert np.array_equal(ids, ids2.cpu().numpy()) and np.array_equal(sc.view(np.uint32), sc2.cpu().numpy().view(np.uint32))
    # a batch (fewer workgroups per query) and heavy ties
    G = W.codes_uniform_u16(200_001, m, b, seed=1)
    assert_same_topk_u16(pq, oracle, G, tables(3, 5, m, b), 10, "u16 short batch")
    Ge = np.full((150_001, m), b - 1, dtype=np.uint16)
    ids, _ = assert_same_topk_u16(pq, oracle, Ge, tables(4, 1, m, b), 31, "u16 short all equal")
    assert ids[0].tolist() == list(range(31))


@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 8, 12, 16, 24])
def test_u16_small_shapes(pq, oracle, m):
    for N in (1, 2, 3, 5, 63, 64, 65, 1000, 4099, 70_001):
        for b in (257, 1000):
            for B in (1, 3):
                G = W.codes_uniform_u16(N, m, b, seed=N + m)
                S = tables(N + m, B, m, b)
                for K in sorted({1, min(N, 10), min(N, 100)}):
                    assert_same_topk_u16(pq, oracle, G, S, K, "small")


@pytest.mark.parametrize("N,m,b,B,K", [(3_000_001, 8, 1024, 1, 10), (2_000_003, 4, 4096, 2, 10), (1_500_001, 4, 8192, 1, 100),
                                       (1_000_001, 16, 2048, 1, 10), (2_000_001, 8, 4096, 1, 10), (700_001, 5, 6000, 2, 10),
                                       (900_001, 16, 300, 3, 100), (5_000_001, 2, 16384, 1, 10), (3_000_001, 1, 32768, 1, 10),
                                       (400_001, 8, 1000, 64, 10), (300_001, 8, 600, 1, 512), (1_000_001, 3, 257, 1, 10),
                                       (200_001, 32, 1024, 2, 10), (20_000_001, 8, 1024, 1, 10)])
def test_u16_long_scans(pq, oracle, N, m, b, B, K):
    # many rounds per workgroup; tables from 5 KB to 128 KB (the larger ones run 1024-thread workgroups); vector rows
    # (m = 4, 8, 16) and row-by-row ones; sub-ids up to b - 1 are present
    G = W.codes_uniform_u16(N, m, b, seed=N % 1000 + m)
    G[N // 2] = b - 1
    assert_same_topk_u16(pq, oracle, G, tables(N % 1000 + b, B, m, b), K, "long")


def test_u16_with_byte_sized_sub_ids_equals_the_uint8_path(pq, oracle):
    for (N, m, B, K) in ((100_003, 8, 2, 10), (50_001, 4, 1, 100), (30_001, 16, 1, 10), (20_001, 3, 2, 10)):
        G8 = W.codes_uniform(N, m, 256, seed=N)
        S = tables(N, B, m, 256)
        ids, sc = assert_same_topk_u16(pq, oracle, G8.astype(np.uint16), S, K, "bytes")
        ids8, sc8 = run_topk(pq, G8, S, K)
        assert np.array_equal(ids, ids8) and np.array_equal(sc.view(np.uint32), sc8.view(np.uint32))


def test_u16_high_byte_selects_the_table_entry(pq, oracle):
    # score == item id exactly, spelled in base 1000 over three splits: any sub-id read modulo 256 breaks the order
    N, m, b = 400_000, 4, 1000
    i = np.arange(N, dtype=np.int64)
    G = np.stack([i % 1000, (i // 1000) % 1000, np.zeros(N, dtype=np.int64), (i * 7) % 1000], axis=1).astype(np.uint16)
    S = np.zeros((1, m, b), dtype=np.float32)
    S[0, 0] = np.arange(b)
    S[0, 1] = np.arange(b) * 1000.0
    ids, sc = assert_same_topk_u16(pq, oracle, G, S, 100, "digits")
    assert ids[0].tolist() == list(range(N - 1, N - 101, -1)) and sc[0].tolist() == [float(x) for x in range(N - 1, N - 101, -1)]


def test_u16_ties(pq, oracle):
    N, m, b, K = 200_000, 8, 700, 20
    G = np.full((N, m), 699, dtype=np.uint16)
    S = tables(7, 1, m, b)
    ids, _ = assert_same_topk_u16(pq, oracle, G, S, K, "all-equal")
    assert ids[0].tolist() == list(range(K))
    # K + 3 copies of the best row at seeded ids: the K lowest of them, in id order
    G = W.codes_uniform_u16(N, m, b, seed=11)
    planted = W.plant_ids(N, K + 3, seed=2)
    G[planted] = S[0].argmax(axis=1).astype(np.uint16)
    ids, _ = assert_same_topk_u16(pq, oracle, G, S, K, "straddle")
    assert ids[0].tolist() == planted[:K].tolist()
    # coarse tables: heavy ties everywhere
    Sc = (np.round(tables(9, 2, 4, 300) * 2) / 2).astype(np.float32)
    assert_same_topk_u16(pq, oracle, W.codes_uniform_u16(300_000, 4, 300, seed=5), Sc, 100, "coarse")


@pytest.mark.parametrize("N,m,b,B", [(100_000, 8, 1000, 1), (100_000, 3, 257, 2), (60_000, 4, 4096, 1)])
def test_u16_tables_that_are_only_four_byte_aligned(pq, oracle, N, m, b, B):
    G = W.codes_uniform_u16(N, m, b, seed=m)
    S = tables(N + m, B, m, b)
    flat = torch.empty(S.size + 1, dtype=torch.float32, device="cuda")
    Sd = flat[1:].view(B, m, b)
    Sd.copy_(torch.from_numpy(S))
    assert Sd.data_ptr() % 16 == 4 and Sd.is_contiguous()
    ids, sc = pq.pq_score_topk_u16(dev(G), Sd, 10)
    torch.cuda.synchronize()
    rid, rsc = oracle.score_topk_u16(G, S, 10)
    assert np.array_equal(ids.cpu().numpy(), rid)
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), rsc.view(np.uint32))


def test_u16_from_embeddings(pq, oracle):
    # the whole path with an alphabet of 1024 sub-ids per split: Eq. 4 on the GPU, then the scan
    N, d, m, b, B, K = 500_000, 512, 8, 1024, 3, 10
    cent, Q = W.centroids(m, b, d, seed=3), W.queries(B, d, seed=3)
    G = W.codes_uniform_u16(N, m, b, seed=3)
    Sd = pq.pq_subitem_scores(dev(Q), dev(cent))
    S = Sd.cpu().numpy()
    assert np.array_equal(S.view(np.uint32), oracle.subitem_scores(Q, cent).view(np.uint32))
    assert_same_topk_u16(pq, oracle, G, S, K, "embeddings")


@pytest.mark.parametrize("N,m,b,B,K", [(300_001, 8, 65536, 1, 10), (200_003, 2, 65536, 2, 100), (150_001, 16, 8192, 1, 10),
                                       (100_001, 5, 40000, 3, 10), (2_000_001, 8, 8192, 1, 10), (50_001, 32, 4096, 1, 512),
                                       (7, 3, 65536, 1, 7), (400_001, 4, 65536, 64, 10)])
def test_u16_tables_too_large_for_lds(pq, oracle, N, m, b, B, K):
    # tables from 256 KB to 2 MB per query: looked up in device memory; the largest sub-id (b - 1) is present
    G = W.codes_uniform_u16(N, m, b, seed=N % 1000 + m)
    G[N // 2] = b - 1
    assert_same_topk_u16(pq, oracle, G, tables(N % 1000 + b, B, m, b), K, "memory tables")


def test_u16_errors_reach_python(pq):
    G = dev(W.codes_uniform_u16(1000, 8, 300))
    with pytest.raises(pq.PQError) as e:
        pq.pq_score_topk_u16(G, dev(np.zeros((1, 8, 300), dtype=np.float32)), 1001)
    assert e.value.code == pq.PQ_ERR_SHAPE
    with pytest.raises(ValueError):
        pq.pq_score_topk_u16(dev(W.codes_uniform(1000, 8)), dev(np.zeros((1, 8, 300), dtype=np.float32)), 10)   # uint8 codes


# ---------------------------------------------------------------- Algorithm 1 with a candidate list V

def assert_same_subset_topk(pq, oracle, G, S, V, K, tag=""):
    print(f"case {tag} N={G.shape[0]} |V|={V.shape[0]} m={G.shape[1]} B={S.shape[0]} b={S.shape[2]} K={K}", flush=True)
    ids, sc = pq.pq_score_topk_subset(dev(G), dev(S), dev(V), K)
    torch.cuda.synchronize()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    rid, rsc = oracle.score_topk_subset(G, S, V, K)
    assert np.array_equal(ids, rid), tag
    check_scores(sc, rsc)
    assert np.array_equal(sc.view(np.uint32), rsc.view(np.uint32)), tag
    return ids, sc


@pytest.mark.parametrize("m", [1, 3, 4, 8, 16, 64])
def test_subset_small_shapes(pq, oracle, m):
    for N in (1, 5, 64, 1000, 70_001):
        for b in (256, 16):
            G = W.codes_uniform(N, m, b, seed=N + m)
            for B in (1, 3):
                S = W.normal_f32(W.stream_key(N + m, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
                for n in sorted({1, min(N, 2), min(N, 65), min(N, 2049), min(N, 20_000), N}):
                    V = W.candidate_list(N, n, seed=n)
                    for K in sorted({1, min(n, 10), min(n, 100)}):
                        assert_same_subset_topk(pq, oracle, G, S, V, K, "subset-small")


def test_subset_of_the_large_catalogue(pq, oracle, large_codes):
    cfg = W.CONFIGS["large"]
    cent, Q = W.centroids(cfg.m, cfg.b, cfg.d, cfg.seed), W.queries(3, cfg.d, cfg.seed)
    S = pq.pq_subitem_scores(dev(Q), dev(cent)).cpu().numpy()
    full_ids, _ = oracle.score_topk(large_codes, S, cfg.K)
    for n, K in ((10, 10), (1000, 10), (100_000, 10), (100_000, 512), (1_000_000, 100), (1_280_000, 10)):
        V = W.candidate_list(cfg.N, n, seed=n, ascending=(n == 1_000_000))
        ids, _ = assert_same_subset_topk(pq, oracle, large_codes, S, V, K, "subset-large")
        if n == cfg.N:                                     # V = I in a shuffled order: the full scan's answer
            assert np.array_equal(ids, full_ids)


@pytest.mark.parametrize("m", [4, 8, 16])
def test_subset_lists_held_in_registers(pq, oracle, m):
    # candidate lists with K < 32 whose share per thread fits its registers take a kernel of their own (every row of a
    # thread requested at once), with an instance per number of code vectors' worth of rows a thread holds: list
    # lengths that land on each of them (ragged last slots), batches (fewer workgroups per query), ascending lists,
    # every item equal (ties by item id; more candidates than the selection's array holds), ids clamped never
    N = 2_400_001
    G = W.codes_uniform(N, m, 256, seed=m)
    ipv = 16 // m
    for vecs in range(1, 9):
        n = (vecs - 1) * ipv * 256 * 512 + 3 * 256 * 512 // 4 + 77
        if n > N:
            break
        V = W.candidate_list(N, n, seed=vecs, ascending=(vecs % 3 == 0))
        for B, K in ((1, 10), (1, 31), (3, 1)):
            ids, sc = assert_same_subset_topk(pq, oracle, G, tables(vecs + B, B, m, 256), V, K, f"subset registers vecs={vecs}")
            prev = pq.pq_measure_force_general(1)                  # the general kernel gives the same bits
            try:
                ids2, sc2 = pq.pq_score_topk_subset(dev(G), dev(tables(vecs + B, B, m, 256)), dev(V), K)
                torch.cuda.synchronize()
            finally:
                pq.pq_measure_force_general(prev)
            assert np.array_equal(ids, ids2.cpu().numpy()) and np.array_equal(sc.view(np.uint32), sc2.cpu().numpy().view(np.uint32))
    Ge = np.full((300_000, m), 9, dtype=np.uint8)
    V = W.candidate_list(300_000, 200_001, seed=5)
    ids, _ = assert_same_subset_topk(pq, oracle, Ge, tables(5, 2, m, 256), V, 31, "subset registers all equal")
    assert ids[0].tolist() == np.sort(V)[:31].tolist()
    Gs = W.codes_uniform(5000, m, 16, seed=3)                  # a short alphabet and a list of a few candidates
    for n in (1, 2, 31, 513):
        assert_same_subset_topk(pq, oracle, Gs, tables(n, 2, m, 16), W.candidate_list(5000, n, seed=n), min(n, 10), "subset registers tiny")


def test_subset_ties_go_to_the_lower_item_id(pq, oracle):
    # every item scores the same: the K lowest ITEM ids of the list win, wherever they sit in it
    N, m, K = 50_000, 8, 20
    G = np.zeros((N, m), dtype=np.uint8)
    S = np.ones((2, m, 256), dtype=np.float32)
    V = W.candidate_list(N, 7001, seed=3)
    ids, _ = assert_same_subset_topk(pq, oracle, G, S, V, K, "subset-ties")
    assert ids[0].tolist() == np.sort(V)[:K].tolist()


def test_subset_errors_reach_python(pq):
    G = dev(W.codes_uniform(100, 8))
    S = dev(np.zeros((1, 8, 256), dtype=np.float32))
    V = dev(np.arange(50, dtype=np.int32))
    with pytest.raises(pq.PQError) as e:
        pq.pq_score_topk_subset(G, S, V, 51)
    assert e.value.code == pq.PQ_ERR_SHAPE
    with pytest.raises(ValueError):
        pq.pq_score_topk_subset(G, S, V.to(torch.int64), 10)


# ---------------------------------------------------------------- the paper's two other scorers (comparison path)

def test_topk_scores_matches_oracle(pq, oracle):
    for N in (1, 3, 4, 5, 63, 1000, 4099, 70_001, 1_280_000, 3_000_003):
        for B in ((1, 3) if N < 2_000_000 else (1,)):
            ld = (N + 3) // 4 * 4 + (8 if B > 1 else 0)
            sc = np.zeros((B, ld), dtype=np.float32)
            sc[:, :N] = W.normal_f32(W.stream_key(N + B, W.STREAM_QUERIES), B * N).reshape(B, N)
            if N > 100:
                sc[:, 7] = -0.0                                  # a negative zero, and a tie at the very top
                sc[0, N - 1] = sc[0, 11] = sc[0].max() + 1.0
            for K in sorted({1, min(N, 10), min(N, 100), min(N, 512)}):
                print(f"case topk-scores N={N} B={B} K={K}", flush=True)
                ids, out = pq.pq_topk_scores(dev(sc), K, N=N)
                torch.cuda.synchronize()
                ids, out = ids.cpu().numpy(), out.cpu().numpy()
                for q in range(B):
                    rid, rsc = oracle.topk(sc[q, :N], K)
                    assert np.array_equal(ids[q], rid)
                    assert np.array_equal(out[q], rsc)               # same values (a -0 comes back as +0)
                    assert not np.any(np.signbit(out[q]) & (out[q] == 0))


@pytest.mark.parametrize("N,m,b,B", [(1, 8, 256, 1), (1027, 3, 7, 2), (70_001, 8, 256, 3), (300_000, 64, 256, 1),
                                     (1_280_000, 8, 256, 1)])
def test_recjpq_scores_equal_algorithm_1(pq, oracle, N, m, b, B):
    # Algorithm 2 adds the same terms in the same order per item: bit-equal scores, hence the same TopK as PQTopK
    G = W.codes_uniform(N, m, b, seed=N)
    S = W.normal_f32(W.stream_key(N, W.STREAM_QUERIES), B * m * b).reshape(B, m, b)
    sc = pq.pq_recjpq_scores(dev(G), dev(S))
    torch.cuda.synchronize()
    got = sc.cpu().numpy()[:, :N]
    for q in range(B):
        ref = oracle.item_scores(G, S[q], split_major=True)
        assert np.array_equal(got[q].view(np.uint32), ref.view(np.uint32))
    K = min(N, 10)
    ids, out = pq.pq_topk_scores(sc, K, N=N)
    ids2, out2 = pq.pq_score_topk(dev(G), dev(S), K)
    torch.cuda.synchronize()
    assert torch.equal(ids, ids2) and torch.equal(out, out2)
    rid, rsc = oracle.score_topk(G, S, K)
    assert np.array_equal(ids.cpu().numpy(), rid)


@pytest.mark.parametrize("N,d,m,b,B", [(1, 8, 2, 4, 1), (1000, 64, 4, 256, 2), (4099, 96, 3, 7, 1), (200_000, 512, 8, 256, 2),
                                       (70_001, 512, 8, 256, 17), (30_000, 96, 3, 7, 64), (5_003, 512, 8, 256, 130),
                                       (999, 8, 2, 4, 5)])
def test_default_scoring_against_float64(pq, oracle, N, d, m, b, B):
    # (batches of two and more take one pass over W on the matrix cores when d is a multiple of 16; a single query, and
    # d = 8, take the mat-vec kernel once per query)
    cent = W.centroids(m, b, d, seed=N)
    Q = W.queries(B, d, seed=N)
    G = W.codes_uniform(N, m, b, seed=N)
    Wd = pq.pq_reconstruct_items(dev(G), dev(cent))
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy(), oracle.reconstruct(G, cent))           # Eq. 2 copies: exact
    sc = pq.pq_default_scores(Wd, dev(Q))
    torch.cuda.synchronize()
    got = sc.cpu().numpy()[:, :N]
    ref = oracle.default_scores(oracle.reconstruct(G, cent), Q)                    # Eq. 3 in float64
    check_scores(got, ref)
    # ranking: the GPU's TopK of its own float32 scores is exact; against the float64 ranking ids agree wherever the
    # float64 scores are further apart than the float32 tolerance (what is unique), and every returned item is valid
    K = min(N, 10)
    ids, out = pq.pq_topk_scores(sc, K, N=N)
    torch.cuda.synchronize()
    ids, out = ids.cpu().numpy(), out.cpu().numpy()
    for q in range(B):
        rid, rsc = oracle.topk(got[q], K)
        assert np.array_equal(ids[q], rid) and np.array_equal(out[q].view(np.uint32), rsc.view(np.uint32))
        order = np.lexsort((np.arange(N), -ref[q]))[:K + 1]
        for r in range(K):
            gap_ok = r + 1 >= len(order) or ref[q][order[r]] - ref[q][order[r + 1]] > 2e-5 * max(abs(ref[q][order[r]]), 1.0)
            prev_ok = r == 0 or ref[q][order[r - 1]] - ref[q][order[r]] > 2e-5 * max(abs(ref[q][order[r]]), 1.0)
            if gap_ok and prev_ok:
                assert ids[q][r] == order[r]
        check_scores(out[q], ref[q][ids[q]])


# ---------------------------------------------------------------- the named configurations at full size

def end_to_end(pq, oracle, cfg, B, G=None):
    print(f"config {cfg.name} B={B}", flush=True)
    G0, cent, Q = W.make(cfg, B=B) if G is None else (G, W.centroids(cfg.m, cfg.b, cfg.d, cfg.seed),
                                                       W.queries(B, cfg.d, cfg.seed))
    Gd = dev(G0)
    S = pq.pq_subitem_scores(dev(Q), dev(cent))
    ids, sc = pq.pq_score_topk(Gd, S, cfg.K)
    torch.cuda.synchronize()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    rid, rsc = oracle.pqtopk(G0, cent, Q, cfg.K)
    assert np.array_equal(ids, rid)
    check_scores(sc, rsc)
    assert np.array_equal(sc.view(np.uint32), rsc.view(np.uint32))
    return G0, cent, Q, ids, sc


def test_config_tiny_brute_force(pq, oracle):
    cfg = W.CONFIGS["tiny"]
    G, cent, Q, ids, sc = end_to_end(pq, oracle, cfg, 1)
    bid, bsc = oracle.bruteforce_topk(G, cent, Q, cfg.K)
    assert np.array_equal(ids, bid)
    check_scores(sc, bsc)


@pytest.fixture(scope="module")
def large_codes():
    return W.codes_uniform(1_280_000, 8)


@pytest.mark.parametrize("B", [1, 64])
def test_config_large(pq, oracle, large_codes, B):
    end_to_end(pq, oracle, W.CONFIGS["large"], B, G=large_codes)


def test_config_serving_zipf(pq, oracle):
    end_to_end(pq, oracle, W.CONFIGS["serving"], 1024)


def test_config_finer_with_duplicates(pq, oracle):
    cfg = W.CONFIGS["finer"]
    G, cent, Q, ids, sc = end_to_end(pq, oracle, cfg, 16)
    # ties really occur among the returned entries
    assert sum(len(set(row.tolist())) < cfg.K for row in sc) >= 1


def test_config_huge(pq, oracle):
    cfg = W.CONFIGS["huge"]
    G = W.codes_uniform(cfg.N, cfg.m)
    end_to_end(pq, oracle, cfg, 1, G=G)
    end_to_end(pq, oracle, cfg, 32, G=G)
