"""APRIL rollout scheduling (oracle side), integers only.  TEST INFRASTRUCTURE ONLY.

One rollout step, following the four-item description of the method
(Section 2.2, "APRIL: Active Partial Rollouts in Reinforcement Learning"):
  * over-provisioned generation: N' > N rollouts are in flight,
  * early termination: generation stops once N rollouts are complete,
  * buffering continuations: unfinished rollouts go to a continuation buffer,
    completed ones are handed to the trainer,
  * prioritized resumption: at the next step buffered rollouts are resumed
    before new ones start.
The wait-for-all baseline (Section 2.2 first paragraph, Section 3.1 "standard
setting") is the same step with N' = N.

Readings where the paper is silent (each listed in the build's design notes):
  - N' counts resumed rollouts too, so a step admits N' - |buffer| new requests;
  - a step is a sequence of iterations; in every executed iteration each
    in-flight rollout gains exactly one token, the stopping iteration included;
  - a rollout is complete when its generated length reaches its limit
    (min(forced length, max_new)) [or, optionally, when it emits the EOS token];
  - exactly N rollouts are returned per step, lowest request id first among
    those that are complete; rollouts completing in the same iteration beyond
    N stay in the buffer flagged done and are returned first at the next step;
  - buffered rollouts are resumed in ascending request id.

Pins (tests/test_oracle_scheduler.py): an order-statistics closed form derived
independently, the method's invariants (exactly N returned, nothing discarded,
N' = N never buffers, buffer size N' - N), and the paper's worked sizes
(N = 256, N' = 512 leaves 256 carried, Section 3.1).
"""
from dataclasses import dataclass, field
from typing import Callable, List, Optional


@dataclass
class Rollout:
    request_id: int
    prompt_len: int
    limit: int = 0                 # fixed at admission: min(forced_len, max_new)
    forced_len: int = 0
    gen: int = 0                   # tokens generated so far
    n_resumes: int = 0
    done: bool = False
    tokens: List[int] = field(default_factory=list)
    user: object = None            # opaque per-rollout state of the sampler (e.g. a KV cache)


@dataclass
class StepOutcome:
    completed: List[Rollout]       # exactly N when the step succeeds
    buffer: List[Rollout]          # surplus-done first kept with partials, ascending request id
    decode_iters: int
    tokens_generated: int
    n_new_consumed: int
    live_per_iter: List[int]


def rollout_step(buffer: List[Rollout], new_requests: List[Rollout], n_target: int,
                 n_overprovision: int, max_new: int,
                 next_token: Optional[Callable[[Rollout], int]] = None,
                 eos_token: int = -1) -> StepOutcome:
    """Run one step.  `buffer` is the previous step's buffer (may be empty);
    `new_requests` are admitted in order as needed.  `next_token(r)` produces the
    next token of rollout r (None: token value 0, scheduling only)."""
    resumed = sorted(buffer, key=lambda r: r.request_id)
    deliver = [r for r in resumed if r.done]
    inflight = [r for r in resumed if not r.done]
    for r in inflight:
        r.n_resumes += 1
    consumed = 0
    while len(inflight) < n_overprovision - len(deliver) and consumed < len(new_requests):
        r = new_requests[consumed]
        consumed += 1
        r.limit = min(r.forced_len, max_new) if r.forced_len > 0 else max_new
        inflight.append(r)
    if len(deliver) + len(inflight) < n_target:
        raise RuntimeError("starved: fewer than N rollouts can ever complete")
    iters = 0
    generated = 0
    live_hist = []
    while len(deliver) < n_target:
        iters += 1
        live_hist.append(len(inflight))
        for r in inflight:
            tok = next_token(r) if next_token is not None else 0
            r.tokens.append(int(tok))
            r.gen += 1
            generated += 1
            if r.gen >= r.limit or (eos_token >= 0 and tok == eos_token):
                r.done = True
        newly = sorted((r for r in inflight if r.done), key=lambda r: r.request_id)
        inflight = [r for r in inflight if not r.done]
        deliver.extend(newly)
    completed = deliver[:n_target]
    new_buffer = sorted(deliver[n_target:] + inflight, key=lambda r: r.request_id)
    return StepOutcome(completed, new_buffer, iters, generated, consumed, live_hist)
