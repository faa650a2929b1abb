"""The seeded input generators: determinism, element-wise addressability, distributions, structure."""
import numpy as np
import pytest

from paper_2408_09992_amd import workloads as W


def test_u64_counter_based():
    key = W.stream_key(0, W.STREAM_CODES)
    a = W.u64_at(key, 0, 1000)
    b = np.concatenate([W.u64_at(key, 0, 333), W.u64_at(key, 333, 667)])
    assert np.array_equal(a, b)
    assert len(np.unique(a)) == 1000
    # the finaliser is the published splitmix64 one: first outputs of the generator seeded with 0
    ref = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [int(x) for x in W.u64_at(0, 0, 3)] == ref


def test_streams_differ_and_seed_matters():
    k = [W.stream_key(0, s) for s in range(1, 8)] + [W.stream_key(1, 1)]
    assert len(set(k)) == len(k)
    assert not np.array_equal(W.codes_uniform(100, 8, seed=0), W.codes_uniform(100, 8, seed=1))


def test_codes_uniform_prefix_stable_and_flat():
    a = W.codes_uniform(1000, 8)
    b = W.codes_uniform(5000, 8)
    assert a.dtype == np.uint8 and a.shape == (1000, 8)
    assert np.array_equal(a, b[:1000])
    big = W.codes_uniform(200_000, 8)
    counts = np.bincount(big.ravel(), minlength=256)
    expect = big.size / 256
    assert abs(counts - expect).max() < 6 * np.sqrt(expect)
    # odd m and ragged byte count
    c = W.codes_uniform(13, 3)
    assert c.shape == (13, 3)
    small_b = W.codes_uniform(10_000, 4, b=7)
    assert small_b.max() == 6 and small_b.min() == 0


def test_normals_moments():
    x = W.normal_f32(W.stream_key(0, W.STREAM_QUERIES), 400_000)
    assert x.dtype == np.float32
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01
    assert np.isfinite(x).all()
    c = W.centroids(8, 256, 512)
    assert c.shape == (8, 256, 64)
    assert abs(float(c.std()) - 512 ** -0.5) < 0.01 * 512 ** -0.5
    q = W.queries(3, 512)
    assert np.array_equal(q[:2], W.queries(2, 512))


def test_zipf_codes():
    G = W.codes_zipf(200_000, 8)
    perm = W.zipf_permutations(8, 256)
    for k in range(8):
        assert sorted(perm[k].tolist()) == list(range(256))
        counts = np.bincount(G[:, k], minlength=256)
        # most popular sub-id is perm[k][0], frequencies fall with rank like r^-1.1
        assert counts.argmax() == perm[k][0]
        p1 = counts[perm[k][0]] / G.shape[0]
        assert abs(p1 - (1.0 / (np.arange(1, 257) ** -1.1).sum())) < 0.01
        assert counts[perm[k][0]] > 1.8 * counts[perm[k][1]]


def test_duplicates():
    G0 = W.codes_uniform(50_000, 16)
    G, src = W.duplicate_rows(G0.copy(), 0.05)
    assert (src <= np.arange(len(src))).all()
    frac = (src != np.arange(len(src))).mean()
    assert 0.04 < frac < 0.06
    assert np.array_equal(G, G0[src])
    assert (src[src] == src).all()          # chains are fully resolved


def test_plant():
    ids = W.plant_ids(1000, 13, seed=3)
    assert len(set(ids.tolist())) == 13 and ids.min() >= 0 and ids.max() < 1000
    G = W.codes_uniform(1000, 4)
    W.plant_rows(G, ids, np.array([1, 2, 3, 4]))
    assert (G[ids] == np.array([1, 2, 3, 4], dtype=np.uint8)).all()


def test_named_configs():
    assert W.CONFIGS["large"].N == 1_280_000 and W.CONFIGS["large"].m == 8 and W.CONFIGS["large"].K == 10
    G, C, Q = W.make(W.CONFIGS["tiny"])
    assert G.shape == (10_000, 4) and C.shape == (4, 256, 16) and Q.shape == (1, 64)
    G2, _, _ = W.make(W.CONFIGS["finer"], N=20_000)
    assert G2.shape == (20_000, 16)
    # duplicated rows exist
    _, inv, cnt = np.unique(G2, axis=0, return_inverse=True, return_counts=True)
    assert (cnt > 1).sum() > 100


def test_candidate_lists_are_seeded_distinct_and_in_range():
    a = W.candidate_list(10_000, 777, seed=3)
    b = W.candidate_list(10_000, 777, seed=3)
    c = W.candidate_list(10_000, 777, seed=4)
    assert a.dtype == np.int32 and a.shape == (777,)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert len(set(a.tolist())) == 777 and a.min() >= 0 and a.max() < 10_000
    assert not np.array_equal(a, np.sort(a))                                  # a random order, not a sorted one
    s = W.candidate_list(10_000, 777, seed=3, ascending=True)
    assert np.array_equal(s, np.sort(a))
    full = W.candidate_list(500, 500, seed=1)
    assert np.array_equal(np.sort(full), np.arange(500))                      # the whole catalogue: a permutation
    with pytest.raises(ValueError):
        W.candidate_list(10, 11)

