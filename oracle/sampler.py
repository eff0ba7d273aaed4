"""Token samplers (oracle side).  TEST INFRASTRUCTURE ONLY.

The paper samples rollouts from the policy (Eq. 1, a ~ pi(theta_k)) with a
temperature (appendix, rollout configuration table) and states nothing else, so
the samplers are the textbook ones in the build's documented reading:

greedy : arg-max of the logits, the lowest index winning ties.
top-k  : keep the k largest logits (ties: lower index first), in descending
         order; p = softmax(logit / temperature) over those k in float64; the
         token is the first kept entry whose inclusive cumulative probability
         exceeds u (the last entry if rounding leaves none).

Pins (tests/test_oracle_sampler.py): k = 1 equals greedy; u -> 0 picks the
arg-max; k = vocab at temperature 1 is the plain categorical distribution
(chi-square of empirical frequencies against softmax); brute-force CDF on tiny
rows.
"""
import numpy as np


def greedy(logits):
    """Lowest index among the maxima (numpy's argmax returns the first maximum)."""
    return int(np.argmax(np.asarray(logits)))


def top_k_candidates(logits, k):
    """Indices of the k largest logits, descending, ties by lower index."""
    logits = np.asarray(logits, dtype=np.float64)
    k = min(int(k), logits.shape[0])
    order = np.lexsort((np.arange(logits.shape[0]), -logits))   # primary: -logit, then index
    return order[:k]


def top_k_probs(logits, k, temperature):
    idx = top_k_candidates(logits, k)
    z = np.asarray(logits, dtype=np.float64)[idx] / float(temperature)
    e = np.exp(z - z[0])
    return idx, e / np.sum(e)


def top_k_sample(logits, k, temperature, u):
    idx, p = top_k_probs(logits, k, temperature)
    c = 0.0
    for j in range(idx.shape[0]):
        c += p[j]
        if c > u:
            return int(idx[j])
    return int(idx[-1])
