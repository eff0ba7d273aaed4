"""The sampler entry point that allocates nothing (its temporaries live in a static device
array) against the allocating entry point, through the C ABI: two calls in a row on one
context, the second with a smaller input, then a third on another context (same GPU, same
array).  Integer outputs: bit-exact."""
import numpy as np
import pytest

import april_inputs as ai
from gpu_common import have_gpu

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


def rows(rng, n, vocab, quant):
    logits = (3.0 * rng.standard_normal((n, vocab))).astype(np.float32)
    if quant:
        logits = (np.round(logits / quant) * quant).astype(np.float32)
    return logits, rng.integers(0, 2 ** 40, size=n), rng.integers(0, 9000, size=n)


@pytest.mark.parametrize("vocab,sampler,top_k,quant", [
    (8192, ai.SAMPLER_TOPK, 50, 0.5),          # group maxima in the scratch, ties across the k-th place
    (151936, ai.SAMPLER_TOPK, 50, None),       # the benchmark vocabulary
    (3001, ai.SAMPLER_GREEDY, 1, 1.0),         # vocabulary not a multiple of 64: no group maxima
])
def test_no_alloc_sampler_equals_the_allocating_one(vocab, sampler, top_k, quant):
    import torch
    rng = np.random.default_rng(vocab)
    ap, ctx = engine(vocab, sampler, top_k, 0.8, 99 + vocab)
    ap2, ctx2 = engine(vocab, sampler, top_k, 0.8, 99 + vocab)
    try:
        for n, c in ((96, ctx), (17, ctx), (40, ctx2)):          # second call smaller; third from another context
            logits, rid, gi = rows(rng, n, vocab, quant)
            d = torch.from_numpy(logits).cuda()
            want = ap.april_sample_rows(c, d.data_ptr(), n, rid, gi)
            got = ap.april_sample_rows_noalloc(c, d.data_ptr(), n, rid, gi)
            assert np.array_equal(got, want), (n, np.nonzero(got != want))
            assert got.min() >= 0 and got.max() < vocab
    finally:
        ap.april_destroy(ctx)
        ap2.april_destroy(ctx2)


def test_no_alloc_sampler_rejects_sizes_beyond_its_scratch():
    import torch
    ap, ctx = engine(151936, ai.SAMPLER_TOPK, 50, 1.0, 1)
    try:
        n = 512                                                   # 512 x 2374 groups > 1048576 floats
        d = torch.zeros((n, 8), device="cuda")                    # never read: the call must fail on the host
        with pytest.raises(ap.AprilError) as e:
            ap.april_sample_rows_noalloc(ctx, d.data_ptr(), n, np.arange(n), np.zeros(n, dtype=np.int32))
        assert e.value.code == ap.APRIL_EINVAL
        with pytest.raises(ap.AprilError) as e:
            ap.april_sample_rows_noalloc(ctx, d.data_ptr(), 1025, np.arange(1025), np.zeros(1025, dtype=np.int32))
        assert e.value.code == ap.APRIL_EINVAL
    finally:
        ap.april_destroy(ctx)
