"""Token samplers (oracle side).  TEST INFRASTRUCTURE ONLY.

The paper samples rollouts from the policy (Eq. 1, a ~ pi(theta_k)) with a
temperature (appendix, rollout configuration table) and states nothing else, so
the samplers are the textbook ones in the build's documented reading:

greedy : arg-max of the logits, the lowest index winning ties.
top-k  : keep the k largest logits (ties: lower index first), in descending
         order; p = softmax(logit / temperature) over those k in float64; the
         token is the first kept entry whose inclusive cumulative probability
         exceeds u (the last entry if rounding leaves none).

top-p  : (nucleus, on top of top-k) of the k kept candidates in that order, keep the
         shortest prefix whose probabilities - renormalised over the k candidates - sum to
         at least top_p; renormalise over the prefix and sample as above.  The paper lists
         only the value (appendix, evaluation top_p 0.7); applying it after the top-k cut
         and on the renormalised distribution is the build's reading.
categorical : the plain temperature sampling of the paper's rollouts (appendix, rollout
         temperature 0.8; no truncation): p = softmax(logit / temperature) over the whole
         vocabulary in float64, cumulative sum in INDEX order, token = first index whose
         inclusive cumulative probability exceeds u (the last index if rounding leaves none).
log-probability of a token: log softmax(logit / temperature) over the whole vocabulary, the
         quantity a trainer's importance ratio needs (Section 2.2, mixed-policy rollouts),
         whatever truncation the sampler applied.

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


def nucleus_size(p, top_p):
    """Length of the shortest prefix of the (already ordered) probabilities p whose sum is
    at least top_p; at least 1, at most len(p)."""
    c = 0.0
    for j in range(len(p)):
        c += p[j]
        if c >= top_p:
            return j + 1
    return len(p)


def top_k_top_p_probs(logits, k, temperature, top_p):
    """Candidates and probabilities after the top-k cut and the nucleus cut."""
    idx, p = top_k_probs(logits, k, temperature)
    if top_p >= 1.0:
        return idx, p
    n = nucleus_size(p, float(top_p))
    q = p[:n]
    return idx[:n], q / np.sum(q)


def top_k_top_p_sample(logits, k, temperature, top_p, u):
    idx, p = top_k_top_p_probs(logits, k, temperature, top_p)
    c = 0.0
    for j in range(idx.shape[0]):
        c += p[j]
        if c > u:
            return int(idx[j])
    return int(idx[-1])


def categorical_sample(logits, temperature, u):
    """Temperature sampling over the whole vocabulary, cumulative sum in index order."""
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    e = np.exp(z - np.max(z))
    p = e / np.sum(e)
    c = 0.0
    for i in range(p.shape[0]):
        c += p[i]
        if c > u:
            return i
    return int(p.shape[0] - 1)


def token_logprob(logits, temperature, token):
    """log softmax(logits / temperature)[token] over the whole vocabulary."""
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    m = np.max(z)
    return float(z[token] - m - np.log(np.sum(np.exp(z - m))))
