"""APRIL rollouts with the oracle model: scheduler + decoder + sampler.
TEST INFRASTRUCTURE ONLY.

Glue between oracle/scheduler.py (Section 2.2's step) and oracle/model.py:
every in-flight rollout owns a KV cache; a rollout that is carried over keeps
its cache (the policy does not change between steps in this build, so the
cached state is exact), or drops it and recomputes it from its tokens when
`drop_kv` is asked for (the paper's buffer holds tokens: Section 3.2.3, "tokens
from incomplete trajectories are cached and reused").
"""
import numpy as np

from . import sampler as _sampler
from .philox import uniform_for
from .scheduler import Rollout, rollout_step


class OracleRollouts:
    def __init__(self, decoder, sampler="greedy", top_k=50, temperature=1.0, seed=0,
                 eos_token=-1, keep_logits=False, top_p=1.0):
        """sampler: "greedy", "topk" (top-k, then nucleus top_p when < 1) or "categorical"
        (temperature sampling over the whole vocabulary, the paper's rollout setting)."""
        self.dec = decoder
        self.sampler = sampler
        self.top_k = top_k
        self.temperature = temperature
        self.seed = seed
        self.eos_token = eos_token
        self.keep_logits = keep_logits
        self.top_p = top_p
        self.buffer = []
        self.logits = {}            # (request_id, gen_index) -> logits row, if keep_logits

    def _pick(self, r, logits):
        if self.keep_logits:
            self.logits[(r.request_id, r.gen)] = logits.copy()
        if self.sampler == "greedy":
            tok = _sampler.greedy(logits)
        else:
            u = uniform_for(self.seed, r.request_id, r.gen)
            if self.sampler == "categorical":
                tok = _sampler.categorical_sample(logits, self.temperature, u)
            else:
                tok = _sampler.top_k_top_p_sample(logits, self.top_k, self.temperature, self.top_p, u)
        # log-probability of the chosen token under softmax(logits / temperature) over the whole
        # vocabulary: what the trainer's importance ratio uses (Section 2.2)
        r.user.setdefault("logprobs", []).append(_sampler.token_logprob(logits, self.temperature, tok))
        return tok

    def _next_token(self, r):
        st = r.user
        if st["cache"] is None:                       # new, or carried over without KV
            st["cache"] = self.dec.new_cache()
            fed = list(st["prompt"]) + list(r.tokens)
            logits = self.dec.forward_block(fed, st["cache"])[-1]
        else:                                         # KV resident: feed the last token
            logits = self.dec.decode_step(r.tokens[-1], st["cache"])
        return self._pick(r, logits)

    def make_rollout(self, request_id, prompt, forced_len, group=-1):
        return Rollout(request_id=request_id, prompt_len=len(prompt), forced_len=forced_len, group=group,
                       user={"prompt": np.asarray(prompt), "cache": None})

    def drop_kv(self, pool=None):
        for r in self.buffer:
            r.user["cache"] = None
            if pool is not None:
                pool.free += r.pages
            r.pages = 0
            r.kv = 0

    def update_weights(self, decoder, keep_kv=False, pool=None):
        """The trainer has moved the policy (Eq. 1: theta_k -> theta_{k+1}); buffered rollouts
        go on under the new one (Section 2.2, mixed-policy trajectories).  keep_kv = False: the
        cached keys / values were computed under the old weights, so they are dropped and
        recomputed from the tokens under the new weights when the rollout resumes.  keep_kv =
        True: the stale cache stays and only new positions use the new weights."""
        self.dec = decoder
        if not keep_kv:
            self.drop_kv(pool)

    @staticmethod
    def _forget_cache(r):
        r.user["cache"] = None

    def step(self, new_rollouts, n_target, n_overprovision, max_new, pool=None, group_size=1):
        out = rollout_step(self.buffer, new_rollouts, n_target, n_overprovision, max_new,
                           next_token=self._next_token, eos_token=self.eos_token, pool=pool,
                           on_preempt=self._forget_cache, group_size=group_size)
        self.buffer = out.buffer
        for r in out.completed:
            r.user["cache"] = None                    # finished: its KV is released
        for r in out.buffer:
            if r.done:
                r.user["cache"] = None                # complete, waiting for delivery: no KV either
        return out
