"""Checks of the seeded input generators (no method arithmetic is involved).  CPU only."""
import numpy as np

from harness import configs, graphs, sampler


def test_scale_to_matches_big_integer_arithmetic():
    rng = np.random.default_rng(0)
    key = rng.integers(0, 2 ** 64, 1000, dtype=np.uint64)
    for n in (1, 7, 1000, 86_054_151, 2 ** 32 - 1):
        got = sampler.scale_to(key, n)
        want = np.array([(int(x) * n) >> 64 for x in key], dtype=np.int64)
        np.testing.assert_array_equal(got, want)


def test_sampler_is_a_function_of_seed_and_step():
    a = sampler.uniform_negatives(3, 17, 4, 9, 1000)
    b = sampler.uniform_negatives(3, 17, 4, 9, 1000)
    c = sampler.uniform_negatives(3, 18, 4, 9, 1000)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, c)
    assert a.shape == (4, 9) and a.min() >= 0 and a.max() < 1000


def test_uniform_negatives_are_uniform():
    n = 50
    ids = np.concatenate([sampler.uniform_negatives(1, s, 8, 125, n).ravel() for s in range(50)])
    counts = np.bincount(ids, minlength=n)
    expected = ids.size / n
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 100.0  # 49 degrees of freedom: mean 49, sd 9.9


def test_degree_negatives_come_from_the_batch():
    """Sec. 3.3: degree-proportional negatives reuse heads (tails) of triples of the same mini-batch."""
    bs = configs.BatchStream(configs.MEDIUM.scaled(n_entities=5000, n_triples=20000))
    for s in range(3):
        h, r, t, neg, side = bs.step(s)
        pool = h if side == 1 else t
        assert set(neg.ravel().tolist()) <= set(pool.tolist())
        assert neg.shape == (8, 256)


def test_alternating_side_starts_with_tail():
    assert [sampler.side_of_step("alternate", s) for s in range(4)] == [0, 1, 0, 1]


def test_zipf_and_scramble():
    z = graphs.ZipfTable(1000, 1.0)
    rng = np.random.default_rng(0)
    ranks = z.sample(rng.random(200_000))
    counts = np.bincount(ranks, minlength=1000)
    # P(rank 0) / P(rank 9) = 10 for s = 1
    assert 8.0 < counts[0] / counts[9] < 12.5
    ids = graphs.scramble(np.arange(1000), 1000)
    assert sorted(ids.tolist()) == list(range(1000))
    ids = graphs.scramble(np.arange(0, 86_054_151, 997), 86_054_151)
    assert ids.min() >= 0 and ids.max() < 86_054_151 and len(set(ids.tolist())) == ids.size


def test_workload_shapes_follow_the_configurations():
    w = configs.FREEBASE_TRANSE
    assert (w.n_entities, w.n_relations) == (86_054_151, 14_824)  # Table 3 of the paper
    assert (w.batch, w.chunk, w.neg_per_chunk, w.ent_dim) == (1000, 1000, 200, 400)
    t = configs.TINY
    bs = configs.BatchStream(t)
    h, r, t_, neg, side = bs.step(0)
    assert h.shape == (256,) and neg.shape == (8, 64) and side == 0
    assert bs.triples.shape == (10_000, 3)
    E, R = configs.init_tables(t)
    assert E.shape == (1000, 64) and R.shape == (20, 64)
    assert np.abs(E).max() <= 14.0 / 64
