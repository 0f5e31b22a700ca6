"""Pins of the oracle's evaluation functions (rank of a positive among its negatives, Hit@k / MR / MRR): worked
examples and closed forms."""
import numpy as np

import oracle


def test_rank_counts_strictly_better_negatives():
    pos = np.array([0.5, -1.0, 3.0])
    neg = np.array([[0.6, 0.4, 0.5, 0.7],     # two strictly better, one tie: rank 3
                    [-2.0, -3.0, -1.5, -4.0],  # none better: rank 1
                    [4.0, 5.0, 6.0, 7.0]])     # all better: rank 5
    assert oracle.ranks(pos, neg).tolist() == [3, 1, 5]


def test_metrics_of_a_hand_example():
    m = oracle.rank_metrics([1, 2, 4, 11])
    assert np.allclose(m, [0.25, 0.5, 0.75, 4.5, (1 + 0.5 + 0.25 + 1 / 11) / 4], rtol=0, atol=1e-15)


def test_metrics_closed_forms():
    n = 1000
    r = np.arange(1, n + 1)                       # every rank once
    m = oracle.rank_metrics(r)
    assert m[0] == 1 / n and m[1] == 3 / n and m[2] == 10 / n
    assert m[3] == (n + 1) / 2                    # mean of 1..n
    assert abs(m[4] - np.sum(1.0 / r) / n) < 1e-15
    assert np.array_equal(oracle.rank_metrics(np.ones(7)), [1, 1, 1, 1, 1])


def test_ranks_follow_the_score_order_of_the_oracle():
    """With the true tail among the candidates its rank is 1 plus the number of candidates that score strictly
    higher; a model whose positives score gamma (TransE with h + r = t) ranks them first."""
    rng = np.random.default_rng(0)
    D, n = 8, 50
    E = rng.normal(size=(n, D)).astype(np.float32)
    R = rng.normal(size=(3, D)).astype(np.float32)
    h = np.array([1, 2, 3]); r = np.array([0, 1, 2]); t = np.array([10, 11, 12])
    E[t] = E[h] + R[r]                            # exact translations
    neg = np.arange(20, 40).reshape(1, -1)
    pos_s, neg_s = oracle.scores("transe_l2", E, R, h, r, t, neg, 20, 3, 0, 12.0)
    assert np.allclose(pos_s, 12.0)
    assert oracle.ranks(pos_s, neg_s).tolist() == [1, 1, 1]
