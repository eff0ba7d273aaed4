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


def engine(vocab, sampler, top_k, temperature, seed):
    import paper_2509_18521_amd as ap
    shape = ai.ModelShape(1, 32, 1, 1, 32, 32, vocab, dtype=ai.DTYPE_FP32)
    cfg = ap.make_cfg(shape, max_inflight=4, max_ctx=32, sampler=sampler, top_k=top_k, temperature=temperature,
                      seed=seed)
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
