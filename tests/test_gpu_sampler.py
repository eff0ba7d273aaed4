"""The device sampler alone, on identical logits rows and identical uniforms."""
import numpy as np
import pytest

import april_inputs as ai
from gpu_common import have_gpu
from oracle import sampler as osampler
from oracle.philox import uniform_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not have_gpu():
        pytest.skip("no GPU")


def engine(vocab, sampler, top_k, temperature, seed, top_p=0.0):
    import paper_2509_18521_amd as ap
    shape = ai.ModelShape(1, 32, 1, 1, 32, 32, vocab, dtype=ai.DTYPE_FP32)
    cfg = ap.make_cfg(shape, max_inflight=4, max_ctx=32, sampler=sampler, top_k=top_k, temperature=temperature,
                      seed=seed, top_p=top_p)
    return ap, ap.april_init(cfg, ap.pack_weights(shape, ai.make_weights(shape, 0)))


@pytest.mark.parametrize("vocab,top_k,temperature,quant", [
    (151936, 50, 1.0, None), (151936, 50, 0.75, None), (1000, 50, 1.0, 0.25), (37, 64, 1.0, 0.5),
    (512, 1, 1.0, None), (4096, 7, 0.5, 1.0), (8192, 50, 1.0, 0.5), (65536, 64, 1.0, 2.0), (4160, 50, 1.0, None)])
def test_topk_sampler_matches_oracle(vocab, top_k, temperature, quant):
    import torch
    rng = np.random.default_rng(vocab + top_k)
    n = 48
    logits = (3.0 * rng.standard_normal((n, vocab))).astype(np.float32)
    if quant:                                    # many exact ties, also across the k-th place
        logits = (np.round(logits / quant) * quant).astype(np.float32)
    seed = 1234567 + vocab
    ap, ctx = engine(vocab, ai.SAMPLER_TOPK, top_k, temperature, seed)
    try:
        rid = rng.integers(0, 2 ** 40, size=n)
        gi = rng.integers(0, 9000, size=n)
        d = torch.from_numpy(logits).cuda()
        got = ap.april_sample_rows(ctx, d.data_ptr(), n, rid, gi)
        exact = 0
        for r in range(n):
            u = uniform_for(seed, int(rid[r]), int(gi[r]))
            idx, p = osampler.top_k_probs(logits[r], top_k, float(np.float32(temperature)))
            if np.min(np.abs(np.cumsum(p)[:-1] - u)) < 1e-9 if len(p) > 1 else False:
                continue                         # u on a CDF boundary: either neighbour is right
            assert int(got[r]) == osampler.top_k_sample(logits[r], top_k, float(np.float32(temperature)), u), r
            exact += 1
        assert exact >= n - 2
    finally:
        ap.april_destroy(ctx)


def test_greedy_sampler_lowest_index_on_ties():
    import torch
    rng = np.random.default_rng(5)
    n, vocab = 32, 3001
    logits = np.round(rng.standard_normal((n, vocab)) * 2).astype(np.float32)     # heavy ties at the max
    logits[3] = 0.0
    logits[4] = -0.0
    logits[5, 100] = np.float32(-0.0)
    ap, ctx = engine(vocab, ai.SAMPLER_GREEDY, 1, 1.0, 0)
    try:
        d = torch.from_numpy(logits).cuda()
        got = ap.april_sample_rows(ctx, d.data_ptr(), n, np.arange(n), np.zeros(n, dtype=np.int32))
        for r in range(n):
            assert int(got[r]) == osampler.greedy(logits[r]), r
    finally:
        ap.april_destroy(ctx)


@pytest.mark.parametrize("vocab,top_k,temperature,top_p,quant", [
    (151936, 64, 0.8, 0.7, None),      # the paper's appendix values: temperature 0.8, top_p 0.7
    (4096, 50, 1.0, 0.9, 0.5), (1000, 20, 0.5, 0.3, 0.25), (512, 64, 1.0, 0.999, None), (8192, 8, 1.3, 0.05, None)])
def test_nucleus_sampler_matches_oracle(vocab, top_k, temperature, top_p, quant):
    """top-k then top-p on the device against the oracle on identical logits and uniforms; rows
    where the uniform or top_p lies within 1e-9 of a step of the cumulative distribution are
    not compared (either neighbour is right there)."""
    import torch
    rng = np.random.default_rng(vocab + top_k + 7)
    n = 64
    logits = (3.0 * rng.standard_normal((n, vocab))).astype(np.float32)
    if quant:
        logits = (np.round(logits / quant) * quant).astype(np.float32)
    seed = 99 + vocab
    T, P = float(np.float32(temperature)), float(np.float32(top_p))
    ap, ctx = engine(vocab, ai.SAMPLER_TOPK, top_k, temperature, seed, top_p=top_p)
    try:
        rid = rng.integers(0, 2 ** 40, size=n)
        gi = rng.integers(0, 9000, size=n)
        d = torch.from_numpy(logits).cuda()
        got = ap.april_sample_rows(ctx, d.data_ptr(), n, rid, gi)
        exact, sizes = 0, set()
        for r in range(n):
            u = uniform_for(seed, int(rid[r]), int(gi[r]))
            _, pk = osampler.top_k_probs(logits[r], top_k, T)
            if np.min(np.abs(np.cumsum(pk) - P)) < 1e-9:
                continue
            idx, q = osampler.top_k_top_p_probs(logits[r], top_k, T, P)
            sizes.add(len(idx))
            if len(q) > 1 and np.min(np.abs(np.cumsum(q)[:-1] - u)) < 1e-9:
                continue
            assert int(got[r]) == osampler.top_k_top_p_sample(logits[r], top_k, T, P, u), r
            exact += 1
        assert exact >= n - 3 and (len(sizes) > 1 or top_p < 0.1)
    finally:
        ap.april_destroy(ctx)


@pytest.mark.parametrize("vocab,temperature", [(151936, 0.8), (3001, 1.0), (64, 0.5), (5000, 2.0)])
def test_categorical_sampler_and_logprobs_match_oracle(vocab, temperature):
    """Temperature sampling over the whole vocabulary (index-order inverse CDF) and the
    log-probability of the chosen token, on identical logits and uniforms."""
    import torch
    rng = np.random.default_rng(vocab)
    n = 40
    logits = (2.5 * rng.standard_normal((n, vocab))).astype(np.float32)
    logits[0] = 0.0                                        # uniform row: log-probability -log V
    seed = 5 + vocab
    T = float(np.float32(temperature))
    ap, ctx = engine(vocab, ai.SAMPLER_CATEGORICAL, 1, temperature, seed)
    try:
        rid = rng.integers(0, 2 ** 40, size=n)
        gi = rng.integers(0, 9000, size=n)
        d = torch.from_numpy(logits).cuda()
        got, lp = ap.april_sample_rows_logprobs(ctx, d.data_ptr(), n, rid, gi)
        assert np.array_equal(got, ap.april_sample_rows(ctx, d.data_ptr(), n, rid, gi))
        exact = 0
        for r in range(n):
            u = uniform_for(seed, int(rid[r]), int(gi[r]))
            z = logits[r].astype(np.float64) / T
            p = np.exp(z - z.max()); p /= p.sum()
            assert abs(float(lp[r]) - osampler.token_logprob(logits[r], T, int(got[r]))) < 2e-5, r
            if np.min(np.abs(np.cumsum(p) - u)) < 1e-9:
                continue
            assert int(got[r]) == osampler.categorical_sample(logits[r], T, u), r
            exact += 1
        assert exact >= n - 2
        assert abs(float(lp[0]) + np.log(vocab)) < 2e-5
    finally:
        ap.april_destroy(ctx)


def test_logprobs_of_greedy_and_topk_choices():
    import torch
    rng = np.random.default_rng(77)
    n, vocab = 24, 4160
    logits = (3.0 * rng.standard_normal((n, vocab))).astype(np.float32)
    for sampler, top_k, temperature in ((ai.SAMPLER_GREEDY, 1, 1.0), (ai.SAMPLER_TOPK, 50, 0.8)):
        T = float(np.float32(temperature))
        ap, ctx = engine(vocab, sampler, top_k, temperature, 3)
        try:
            d = torch.from_numpy(logits).cuda()
            got, lp = ap.april_sample_rows_logprobs(ctx, d.data_ptr(), n, np.arange(n), np.arange(n, dtype=np.int32))
            for r in range(n):
                assert abs(float(lp[r]) - osampler.token_logprob(logits[r], T, int(got[r]))) < 2e-5
        finally:
            ap.april_destroy(ctx)
