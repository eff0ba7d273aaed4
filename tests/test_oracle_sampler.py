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


# ---- nucleus (top-p), categorical, log-probabilities ------------------------------------
def brute_force_nucleus(p, top_p):
    """Smallest set of most probable entries with mass >= top_p, by trying every prefix
    length of the entries sorted by (probability desc, index asc)."""
    order = sorted(range(len(p)), key=lambda i: (-p[i], i))
    for n in range(1, len(p) + 1):
        if sum(p[i] for i in order[:n]) >= top_p:
            return order[:n]
    return order


def test_top_p_one_is_top_k_and_tiny_top_p_is_greedy():
    rng = np.random.default_rng(3)
    for _ in range(40):
        l = rng.standard_normal(50)
        u = rng.random()
        assert sampler.top_k_top_p_sample(l, 10, 0.8, 1.0, u) == sampler.top_k_sample(l, 10, 0.8, u)
        assert sampler.top_k_top_p_sample(l, 10, 0.8, 1e-9, u) == sampler.greedy(l)


def test_nucleus_is_the_smallest_prefix_reaching_top_p():
    rng = np.random.default_rng(4)
    for _ in range(200):
        n = int(rng.integers(2, 12))
        l = np.round(rng.standard_normal(n) * 2) / 2            # exact ties happen
        top_p = float(rng.uniform(0.05, 0.99))
        idx, q = sampler.top_k_top_p_probs(l, n, 1.0, top_p)
        p = np.exp(l - l.max()); p = p / p.sum()
        want = brute_force_nucleus(p, top_p)
        assert list(idx) == want
        assert abs(q.sum() - 1.0) < 1e-12
        assert np.allclose(q, p[want] / p[want].sum())
        # dropping the last kept entry falls short of top_p
        assert len(want) == 1 or p[want[:-1]].sum() < top_p


def test_nucleus_exact_binary_cases_and_tie_at_the_boundary():
    l = np.log(np.array([0.25, 0.5, 0.125, 0.125]))
    # sorted: idx1 0.5, idx0 0.25, idx2 0.125, idx3 0.125
    assert list(sampler.top_k_top_p_probs(l, 4, 1.0, 0.5)[0]) == [1]
    assert list(sampler.top_k_top_p_probs(l, 4, 1.0, 0.51)[0]) == [1, 0]
    assert list(sampler.top_k_top_p_probs(l, 4, 1.0, 0.75)[0]) == [1, 0]
    assert list(sampler.top_k_top_p_probs(l, 4, 1.0, 0.76)[0]) == [1, 0, 2]       # of the tied pair the lower index
    assert list(sampler.top_k_top_p_probs(l, 4, 1.0, 0.9)[0]) == [1, 0, 2, 3]
    # inside the nucleus {1, 0}: renormalised 2/3, 1/3
    assert sampler.top_k_top_p_sample(l, 4, 1.0, 0.75, 0.66) == 1
    assert sampler.top_k_top_p_sample(l, 4, 1.0, 0.75, 0.67) == 0
    # the top-k cut comes first: with k = 2 the candidates are renormalised to 2/3, 1/3, so
    # top_p = 0.7 needs both although 0.5 + 0.25 of the full distribution would not
    assert list(sampler.top_k_top_p_probs(l, 2, 1.0, 0.7)[0]) == [1, 0]
    assert list(sampler.top_k_top_p_probs(l, 2, 1.0, 0.6)[0]) == [1]


def test_nucleus_frequencies_chi_square():
    rng = np.random.default_rng(5)
    l = rng.standard_normal(30)
    idx, q = sampler.top_k_top_p_probs(l, 20, 0.8, 0.7)
    n = 20000
    counts = {int(i): 0 for i in idx}
    for u in rng.random(n):
        counts[sampler.top_k_top_p_sample(l, 20, 0.8, 0.7, u)] += 1       # KeyError = token outside the nucleus
    chi2 = sum((counts[int(i)] - n * qi) ** 2 / (n * qi) for i, qi in zip(idx, q))
    assert len(idx) >= 3 and chi2 < 50.0


def test_categorical_exact_binary_cdf_in_index_order():
    l = np.log(np.array([0.25, 0.5, 0.125, 0.125]))
    assert sampler.categorical_sample(l, 1.0, 0.24) == 0
    assert sampler.categorical_sample(l, 1.0, 0.26) == 1
    assert sampler.categorical_sample(l, 1.0, 0.74) == 1
    assert sampler.categorical_sample(l, 1.0, 0.76) == 2
    assert sampler.categorical_sample(l, 1.0, 0.88) == 3
    assert sampler.categorical_sample(l, 1.0, 0.9999999) == 3
    # temperature 0.5 squares the probabilities: 4, 16, 1, 1 of 22
    assert sampler.categorical_sample(l, 0.5, 3.9 / 22) == 0
    assert sampler.categorical_sample(l, 0.5, 4.1 / 22) == 1
    assert sampler.categorical_sample(l, 0.5, 20.1 / 22) == 2


def test_categorical_frequencies_chi_square():
    rng = np.random.default_rng(6)
    l = rng.standard_normal(12)
    T = 0.8
    p = np.exp(l / T) / np.exp(l / T).sum()
    n = 20000
    counts = np.zeros(12)
    for u in rng.random(n):
        counts[sampler.categorical_sample(l, T, u)] += 1
    assert ((counts - n * p) ** 2 / (n * p)).sum() < 40.0


def test_token_logprob_closed_forms():
    V = 37
    assert abs(sampler.token_logprob(np.zeros(V), 0.8, 5) + np.log(V)) < 1e-14          # uniform
    rng = np.random.default_rng(7)
    l = rng.standard_normal(V) * 3
    lp = np.array([sampler.token_logprob(l, 0.8, t) for t in range(V)])
    assert abs(np.exp(lp).sum() - 1.0) < 1e-12                                          # a distribution
    assert np.allclose(lp, [sampler.token_logprob(l + 11.5, 0.8, t) for t in range(V)])  # shift invariant
    assert np.allclose(lp[3] - lp[9], (l[3] - l[9]) / 0.8)                              # log-odds = logit gap / T
    # two logits: log sigmoid
    assert abs(sampler.token_logprob(np.array([0.0, 2.0]), 1.0, 1) + np.log1p(np.exp(-2.0))) < 1e-14
