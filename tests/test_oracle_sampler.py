"""Pins for oracle/sampler.py."""
import numpy as np

from oracle import sampler


def test_greedy_lowest_index_on_ties():
    assert sampler.greedy(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert sampler.greedy(np.array([5.0, 5.0])) == 0


def test_topk_candidates_order_and_ties():
    l = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 1.0])
    assert list(sampler.top_k_candidates(l, 4)) == [1, 2, 4, 5]
    assert list(sampler.top_k_candidates(l, 100)) == [1, 2, 4, 5, 0, 3]


def test_k1_is_greedy_and_u0_is_argmax():
    rng = np.random.default_rng(0)
    for _ in range(50):
        l = rng.standard_normal(37)
        u = rng.random()
        assert sampler.top_k_sample(l, 1, 1.0, u) == sampler.greedy(l)
        assert sampler.top_k_sample(l, 10, 0.7, 0.0) == sampler.greedy(l)


def test_bruteforce_cdf_tiny():
    # three candidates with probabilities that are exact in binary: 1/2, 1/4, 1/4
    l = np.log(np.array([0.25, 0.5, 0.01, 0.25]))
    # order: idx1 (0.5), idx0 (0.25), idx3 (0.25); idx2 is dropped by k=3
    assert sampler.top_k_sample(l, 3, 1.0, 0.49) == 1
    assert sampler.top_k_sample(l, 3, 1.0, 0.51) == 0
    assert sampler.top_k_sample(l, 3, 1.0, 0.76) == 3
    assert sampler.top_k_sample(l, 3, 1.0, 0.999999) == 3
    # temperature 0.5 squares the probabilities: 4/6, 1/6, 1/6
    assert sampler.top_k_sample(l, 3, 0.5, 0.66) == 1
    assert sampler.top_k_sample(l, 3, 0.5, 0.67) == 0
    assert sampler.top_k_sample(l, 3, 0.5, 0.84) == 3


def test_full_vocab_is_categorical_chi_square():
    rng = np.random.default_rng(1)
    l = rng.standard_normal(12)
    p = np.exp(l) / np.exp(l).sum()
    n = 20000
    counts = np.zeros(12)
    for u in rng.random(n):
        counts[sampler.top_k_sample(l, 12, 1.0, u)] += 1
    chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 40.0        # 11 degrees of freedom: P(chi2 > 40) ~ 4e-5


def test_topk_mass_restricted_to_k():
    rng = np.random.default_rng(2)
    l = rng.standard_normal(100)
    keep = set(sampler.top_k_candidates(l, 5).tolist())
    for u in rng.random(500):
        assert sampler.top_k_sample(l, 5, 1.0, u) in keep
