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
  - buffered rollouts are resumed in ascending request id;
  - an exhausted KV pool (optional PagePool): see rollout_step;
  - instance-level completion (Section 3.2.3, the paragraph on instance-level group control;
    Section 3.1: 32 prompts x 8 samples): with group_size G > 1 every input instance is a
    group of G rollouts, N and N' count rollouts in multiples of G, the step stops once N / G
    GROUPS have all their members complete, and it returns exactly those groups (N rollouts);
    complete members of an incomplete group wait in the buffer and leave with their group.

Pins (tests/test_oracle_scheduler.py): an order-statistics closed form derived
independently, the method's invariants (exactly N returned, nothing discarded,
N' = N never buffers, buffer size N' - N), the paper's worked sizes
(N = 256, N' = 512 leaves 256 carried, Section 3.1); for the page pool: an ample
pool changes nothing, pages are conserved, only the youngest are preempted, and
a brute-force replay of the page demand.
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
    kv: int = 0                    # positions whose K/V are cached (0: token-level only)
    pages: int = 0                 # KV pages held (only tracked with a PagePool)
    group: int = -1                # input instance the rollout belongs to (group_size > 1)


@dataclass
class PagePool:
    """KV page accounting (integers only).  A rollout with K/V for c positions holds
    ceil(c / page_tokens) pages; completed rollouts give their pages back at the END of
    the step in which they complete."""
    total: int
    page_tokens: int = 16
    free: int = -1

    def __post_init__(self):
        if self.free < 0:
            self.free = self.total


@dataclass
class StepOutcome:
    completed: List[Rollout]       # exactly N when the step succeeds
    buffer: List[Rollout]          # surplus-done first kept with partials, ascending request id
    decode_iters: int
    tokens_generated: int
    n_new_consumed: int
    live_per_iter: List[int]
    preempted: List[int] = field(default_factory=list)   # request ids preempted in this step, in order


def _pages(n_tokens, page_tokens):
    return -(-n_tokens // page_tokens)


def rollout_step(buffer: List[Rollout], new_requests: List[Rollout], n_target: int,
                 n_overprovision: int, max_new: int,
                 next_token: Optional[Callable[[Rollout], int]] = None,
                 eos_token: int = -1, pool: Optional[PagePool] = None,
                 on_preempt: Optional[Callable[[Rollout], None]] = None,
                 group_size: int = 1) -> StepOutcome:
    """Run one step.  `buffer` is the previous step's buffer (may be empty);
    `new_requests` are admitted in order as needed.  `next_token(r)` produces the
    next token of rollout r (None: token value 0, scheduling only).

    With a PagePool (the build's reading for an exhausted KV pool, integers only):
      * a rollout that needs prefill (new, or resumed without K/V) is admitted only
        if the pages of its tokens fit; the first one that does not fit closes
        admission for the step (it stays buffered / unconsumed);
      * before an iteration, the in-flight rollouts that decode and whose next position
        opens a page each need one page; while they need more than are free, the
        youngest decoding rollout (largest request id) is preempted: its pages are
        freed, it keeps its tokens, stops progressing this step and is re-prefilled
        when resumed;
      * if nothing is left in flight before N rollouts are complete, the step ends
        with fewer than N.

    group_size > 1: instance-level completion, see rollout_step_groups."""
    if group_size > 1:
        return rollout_step_groups(buffer, new_requests, n_target, n_overprovision, max_new, group_size,
                                   next_token=next_token, eos_token=eos_token)
    resumed = sorted(buffer, key=lambda r: r.request_id)
    deliver = [r for r in resumed if r.done]
    inflight: List[Rollout] = []
    stay: List[Rollout] = []
    prefill_ids = set()
    admission_open = True
    for r in resumed:
        if r.done:
            continue
        if pool is not None and r.kv == 0:
            need = _pages(r.prompt_len + r.gen, pool.page_tokens)
            if admission_open and need <= pool.free:
                pool.free -= need
                r.pages = need
            else:
                admission_open = False
                stay.append(r)
                continue
        if r.kv == 0:
            prefill_ids.add(r.request_id)
        r.n_resumes += 1
        inflight.append(r)
    consumed = 0
    while (len(inflight) < n_overprovision - len(deliver) and consumed < len(new_requests)
           and admission_open):
        r = new_requests[consumed]
        if pool is not None:
            need = _pages(r.prompt_len, pool.page_tokens)
            if need > pool.free:
                admission_open = False
                break
            pool.free -= need
            r.pages = need
        consumed += 1
        r.limit = min(r.forced_len, max_new) if r.forced_len > 0 else max_new
        r.kv = 0
        prefill_ids.add(r.request_id)
        inflight.append(r)
    if pool is None and len(deliver) + len(inflight) < n_target:
        raise RuntimeError("starved: fewer than N rollouts can ever complete")
    iters = 0
    generated = 0
    live_hist = []
    preempted: List[Rollout] = []
    finished_now: List[Rollout] = []
    while len(deliver) < n_target:
        if pool is not None:
            decoders = [r for r in inflight if r.request_id not in prefill_ids]
            need = [r for r in decoders if r.kv % pool.page_tokens == 0 and r.kv // pool.page_tokens >= r.pages]
            while len(need) > pool.free:
                victim = max(decoders, key=lambda r: r.request_id)
                decoders.remove(victim)
                inflight.remove(victim)
                if victim in need:
                    need.remove(victim)
                pool.free += victim.pages
                victim.pages = 0
                victim.kv = 0
                if on_preempt is not None:
                    on_preempt(victim)
                preempted.append(victim)
            for r in need:
                pool.free -= 1
                r.pages += 1
        if not inflight:
            break
        iters += 1
        live_hist.append(len(inflight))
        for r in inflight:
            tok = next_token(r) if next_token is not None else 0
            r.tokens.append(int(tok))
            r.gen += 1
            r.kv = r.prompt_len + r.gen - 1
            generated += 1
            if r.gen >= r.limit or (eos_token >= 0 and tok == eos_token):
                r.done = True
        prefill_ids.clear()
        newly = sorted((r for r in inflight if r.done), key=lambda r: r.request_id)
        inflight = [r for r in inflight if not r.done]
        deliver.extend(newly)
        finished_now.extend(newly)
    if pool is not None:
        for r in finished_now:                         # pages of completed rollouts: back at step end
            pool.free += r.pages
            r.pages = 0
            r.kv = 0
    completed = deliver[:n_target]
    new_buffer = sorted(deliver[n_target:] + inflight + preempted + stay, key=lambda r: r.request_id)
    return StepOutcome(completed, new_buffer, iters, generated, consumed, live_hist,
                       [r.request_id for r in preempted])


def rollout_step_groups(buffer: List[Rollout], new_requests: List[Rollout], n_target: int,
                        n_overprovision: int, max_new: int, group_size: int,
                        next_token: Optional[Callable[[Rollout], int]] = None,
                        eos_token: int = -1) -> StepOutcome:
    """One step with instance-level completion (Section 3.2.3; Section 3.1's 32 x 8 and 64 x 8).

    Every rollout carries the id of its input instance (`group`); an instance has exactly
    group_size rollouts, which arrive consecutively in new_requests and are admitted together.
    n_target and n_overprovision count rollouts and are multiples of group_size.
      * groups of the buffer whose members are all complete (surplus of the last step) are
        delivered first, ascending group id;
      * the unfinished members of the other buffered groups resume (ascending request id); their
        complete members wait in the buffer;
      * new groups are admitted until n_overprovision / group_size groups are in flight or
        delivered;
      * every iteration gives each in-flight rollout one token; a group is complete in the
        iteration in which its last member completes; the step stops once n_target / group_size
        groups are complete;
      * returned: exactly those groups, in order of completion (iteration, then group id), the
        members of a group in ascending request id; groups completing in the stopping iteration
        beyond the target stay in the buffer and are delivered first next time.
    KV-pool accounting is not combined with groups here (ample pool)."""
    G = group_size
    assert n_target % G == 0 and n_overprovision % G == 0 and n_target > 0
    want_groups, over_groups = n_target // G, n_overprovision // G
    members = {}
    for r in sorted(buffer, key=lambda r: r.request_id):
        members.setdefault(r.group, []).append(r)
    deliver = []                                   # complete groups, in delivery order
    for gid in sorted(members):
        if len(members[gid]) == G and all(r.done for r in members[gid]):
            deliver.append(gid)
    inflight: List[Rollout] = []
    open_groups = set()
    for gid in sorted(members):
        if gid in deliver:
            continue
        assert len(members[gid]) == G, "a buffered group lost a member"
        open_groups.add(gid)
        for r in members[gid]:
            if not r.done:
                r.n_resumes += 1
                inflight.append(r)
    inflight.sort(key=lambda r: r.request_id)
    consumed = 0
    while len(open_groups) < over_groups - len(deliver) and consumed + G <= len(new_requests):
        grp = new_requests[consumed:consumed + G]
        gid = grp[0].group
        assert all(r.group == gid for r in grp) and gid not in members, "groups arrive whole and once"
        consumed += G
        members[gid] = list(grp)
        open_groups.add(gid)
        for r in grp:
            r.limit = min(r.forced_len, max_new) if r.forced_len > 0 else max_new
            r.kv = 0
            inflight.append(r)
    if len(deliver) + len(open_groups) < want_groups:
        raise RuntimeError("starved: fewer than N / G groups can ever complete")
    iters = generated = 0
    live_hist = []
    while len(deliver) < want_groups:
        iters += 1
        live_hist.append(len(inflight))
        for r in inflight:
            tok = next_token(r) if next_token is not None else 0
            r.tokens.append(int(tok))
            r.gen += 1
            r.kv = r.prompt_len + r.gen - 1
            generated += 1
            if r.gen >= r.limit or (eos_token >= 0 and tok == eos_token):
                r.done = True
        inflight = [r for r in inflight if not r.done]
        newly = sorted(g for g in open_groups if all(r.done for r in members[g]))
        for g in newly:
            open_groups.discard(g)
        deliver.extend(newly)
    completed = [r for g in deliver[:want_groups] for r in sorted(members[g], key=lambda r: r.request_id)]
    for r in completed:
        r.kv = 0
    rest = [r for g in deliver[want_groups:] for r in members[g]] + [r for g in open_groups for r in members[g]]
    for r in rest:
        if r.done:
            r.kv = 0
    new_buffer = sorted(rest, key=lambda r: r.request_id)
    return StepOutcome(completed, new_buffer, iters, generated, consumed, live_hist, [])
