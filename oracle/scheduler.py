"""CPU oracle for the rollout loop under the online length-aware scheduler.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product path never does.

The paper describes the policy in prose only (Sec. 3.1 "Length-aware Rollout
Schedule", "Grouped Rollout", "Selective Batching"; Sec. 3.2 "Controlled
Off-policiness"; Sec. 3.3 rollout state manager and stateful buffer; Sec. 4.4.1
bubble ratio, eq. 4).  This file states it as an algorithm, one global decode
step at a time, in plain Python with no batching tricks:

  oversubscription  -- the queue holds more prompts than there are slots; a slot
                       freed in step s is refilled in step s+1 (phase A);
  early harvest     -- finished rollouts leave the batch at once and are handed
                       out in groups of `group_size` ordered by
                       (completion_step, gen_len, seq_id): shorter responses
                       finish first, so completion order is length order;
  partial mode      -- unfinished rollouts keep their tokens and log-probs across
                       update boundaries; a cache older than `max_staleness`
                       updates is dropped and rebuilt by re-prefilling
                       prompt + generated tokens (nothing is discarded);
  on-policy mode    -- at an update boundary unfinished rollouts are terminated,
                       their generated tokens discarded, prompts re-queued first;
  sync baseline     -- a batch is admitted only when every slot is empty
                       (the canonical pipeline the paper compares against);
  bubble ratio      -- eq. 4 with one decode step as the time unit:
                       sum_s (Q - r_s) / (Q * steps);
  responses/prompt  -- the training recipe draws several responses per prompt
                       (Sec. 4.1); `submit(..., n_responses=k)` makes k rollouts
                       of one prompt that share the KV pages the prompt fills
                       completely (all but the page holding its last token), so
                       only the first of them to be admitted prefills the prompt.

Readings where the paper is silent (slot choice, page allocation order, the
preemption victim, the staleness rule) are this build's and are listed in the
design notes; they are "parity unpinned" against the paper, pinned only by
their definition here and by the invariants in tests/test_oracle_scheduler.py
(exactly-once harvest, group ordering, sum r_s == tokens emitted, closed-form
synchronous bubble 1 - sum L / (Q max L), Q >= n  =>  completion_step = L - 1,
harvest-timing independence, page conservation, the hand-built preemption case).
"""
from __future__ import annotations

from collections import deque
from typing import List, Optional, Sequence

import numpy as np

from .model import greedy_token, log_prob
from .sampling import log_prob_at, sample_token

QUEUED, ACTIVE, FINISHED, HARVESTED = 0, 1, 2, 3
MODE_PARTIAL, MODE_ONPOLICY, MODE_SYNC = 0, 1, 2
EOS_FORCED_ONLY, EOS_NATURAL_OR_FORCED = 0, 1

_M64 = (1 << 64) - 1


def splitmix64_next(state: int):
    """One step of splitmix64 (Steele, Lea, Flood 2014): returns (new state, 64-bit output)."""
    state = (state + 0x9E3779B97F4A7C15) & _M64
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return state, z ^ (z >> 31)


def splitmix64_permutation(n: int, seed: int) -> List[int]:
    """Fisher-Yates shuffle of 0..n-1, from the top down, position i swapped with (next splitmix64 output) mod (i+1)."""
    state = seed & _M64
    perm = list(range(n))
    for i in range(n - 1, 0, -1):
        state, z = splitmix64_next(state)
        j = z % (i + 1)
        perm[i], perm[j] = perm[j], perm[i]
    return perm


class PromptGroup:
    """The k rollouts of one prompt and the KV pages they share: the first `nshared` logical pages, which hold
    prompt positions 0 .. 16*nshared-1 only (the page with the last prompt token is private, every rollout appends
    its own tokens there).  `ref` counts the running rollouts attached; the pages return to the pool with the last."""

    def __init__(self, nshared: int):
        self.nshared = nshared
        self.ref = 0
        self.pages: List[int] = []
        self.version = 0


class Seq:
    """One entry of the stateful rollout buffer (Sec. 3.3): prompt context, partial
    trajectory, log-probs, completion flag (state) and lifecycle indicator (kv_version)."""

    def __init__(self, seq_id: int, prompt: np.ndarray, target_len: int):
        self.seq_id = seq_id
        self.prompt = [int(t) for t in prompt]
        self.target_len = int(target_len)
        self.tokens: List[int] = []
        self.logp: List[float] = []
        self.slot = -1
        self.state = QUEUED
        self.completion_step = -1
        self.policy_version = 0   # policy version under which the last token was produced (set at finish)
        self.kv_version = 0
        self.n_preempt = 0
        self.pages: List[int] = []
        self.needs_prefill = True
        self.last_slot = -1       # slot of the most recent admission (reported at harvest)
        self.group: Optional[PromptGroup] = None
        self.prefill_from = 0     # first position the pending prefill computes (> 0: attached to shared pages)

    @property
    def gen_len(self) -> int:
        return len(self.tokens)


class OracleRollout:
    def __init__(self, *, max_slots: int, page_tokens: int, n_pages: int, max_new_tokens: int,
                 eos_id: int, eos_mode: int = EOS_FORCED_ONLY, mode: int = MODE_PARTIAL,
                 max_staleness: int = -1, page_seed: int = 0, model=None, kv_pool=None,
                 temperature: float = 0.0, sample_seed: int = 0):
        self.Q = max_slots
        self.pt = page_tokens
        self.cap = max_new_tokens
        self.eos_id, self.eos_mode, self.mode = eos_id, eos_mode, mode
        self.max_staleness = max_staleness
        self.model, self.kv_pool = model, kv_pool
        self.temperature, self.sample_seed = temperature, sample_seed   # 0 = greedy
        self.n_pages = n_pages
        self.free = splitmix64_permutation(n_pages, page_seed)  # stack: pop from the end
        self.slots: List[Optional[Seq]] = [None] * max_slots
        self.queue: deque = deque()
        self.seqs: List[Seq] = []
        self.finished: List[Seq] = []      # finished, not yet harvested
        self.step_no = 0
        self.version = 0
        self.n_groups = 0
        # counters (eq. 4 and the rollout_stats record)
        self.busy = 0            # sum_s r_s
        self.idle = 0            # sum_s (Q - r_s)
        self.steps_q = 0         # steps that began with a non-empty queue
        self.idle_q = 0          # idle slot-steps within those
        self.gen_tokens = 0
        self.discarded_tokens = 0
        self.prefill_tokens = 0
        self.n_preempt = 0
        self.n_stale = 0
        self.max_pages_used = 0
        self.last_logits = {}    # slot -> logits row of the last step (teacher-forcing parity)

    # ---- feed prompts (Fig. 2 step 1) ---------------------------------------------------
    def submit(self, prompts: Sequence[np.ndarray], target_len: Sequence[int], n_responses: int = 1) -> int:
        """target_len has len(prompts) * n_responses entries, prompt-major; seq ids follow that order."""
        first = len(self.seqs)
        k = n_responses
        assert len(target_len) == len(prompts) * k
        for i, p in enumerate(prompts):
            nshared = (len(p) - 1) // self.pt
            grp = PromptGroup(nshared) if k > 1 and nshared > 0 else None
            for r in range(k):
                s = Seq(len(self.seqs), p, target_len[i * k + r])
                s.group = grp
                self.seqs.append(s)
                self.queue.append(s)
        return first

    def _pages_for(self, n_tokens: int) -> int:
        return (n_tokens + self.pt - 1) // self.pt

    def _release(self, s: Seq) -> None:
        g = s.group
        keep = 0
        if g is not None:
            g.ref -= 1
            if g.ref > 0:
                keep = g.nshared      # siblings still read the shared pages
            else:
                g.pages = []
        for p in s.pages[keep:]:      # ascending logical-page order
            self.free.append(p)
        s.pages = []
        self.slots[s.slot] = None
        s.slot = -1

    def _next_pos(self, s: Seq) -> int:
        """Position whose K/V the next decode of s writes."""
        return len(s.prompt) + s.gen_len - 1

    # ---- one global decode step -----------------------------------------------------------
    def step(self) -> dict:
        Q = self.Q
        active = [s for s in self.slots if s is not None]
        queue_nonempty = len(self.queue) > 0

        # A. admission: lowest free slot first, FIFO head only, pages for prefix + the token it will emit
        reserve = sum(1 for s in active if (self._next_pos(s) + 1) // self.pt >= len(s.pages))
        admitted = []
        may_admit = not (self.mode == MODE_SYNC and len(active) > 0)
        while may_admit and self.queue:
            free_slots = [i for i in range(Q) if self.slots[i] is None]
            if not free_slots:
                break
            head: Seq = self.queue[0]
            g = head.group
            attach = g is not None and g.ref > 0          # a sibling is running: its prompt pages are reused
            need = self._pages_for(len(head.prompt) + head.gen_len + 1) - (g.nshared if attach else 0)
            if len(self.free) < need + reserve:
                break
            self.queue.popleft()
            head.slot = head.last_slot = free_slots[0]
            self.slots[head.slot] = head
            fresh = [self.free.pop() for _ in range(need)]
            if attach:
                head.pages = list(g.pages) + fresh
                head.kv_version = g.version               # its cache is as old as the shared part
                head.prefill_from = g.nshared * self.pt
            else:
                head.pages = fresh
                head.kv_version = self.version
                head.prefill_from = 0
                if g is not None:
                    g.pages = fresh[:g.nshared]
                    g.version = self.version
            if g is not None:
                g.ref += 1
            head.state = ACTIVE
            head.needs_prefill = True
            admitted.append(head)
        self.max_pages_used = max(self.max_pages_used, self.n_pages - len(self.free))

        # B. forward: prefill for admitted slots, one-token decode for the rest
        ran = [s for s in self.slots if s is not None]
        r = len(ran)
        logits_of = {}
        for s in ran:
            if s.needs_prefill:
                toks = s.prompt + s.tokens
                p0 = s.prefill_from
                self.prefill_tokens += len(toks) - p0
                if self.model is not None:
                    logits_of[s.slot] = self.model.run_tokens(toks[p0:], p0, self.kv_pool.view(s.pages))
                s.needs_prefill = False
            elif self.model is not None:
                pos = self._next_pos(s)
                logits_of[s.slot] = self.model.token_forward(s.tokens[-1], pos, self.kv_pool.view(s.pages))
        self.last_logits = logits_of

        # C. emit one token per slot that ran; finished rollouts leave the batch now
        done = []
        for s in ran:                                     # ascending slot id
            lg = logits_of.get(s.slot)
            forced = s.target_len > 0 and s.gen_len + 1 == s.target_len
            sampling = self.temperature > 0.0 and lg is not None
            if forced:
                tok = self.eos_id
            elif sampling:
                tok = sample_token(lg, self.temperature, self.sample_seed, s.seq_id, s.gen_len)
            else:
                tok = greedy_token(lg) if lg is not None else 0
            s.tokens.append(tok)
            if lg is None:
                s.logp.append(0.0)
            else:
                s.logp.append(log_prob_at(lg, tok, self.temperature) if sampling else log_prob(lg, tok))
            fin = forced or (self.eos_mode == EOS_NATURAL_OR_FORCED and tok == self.eos_id) \
                or s.gen_len >= self.cap
            if fin:
                s.completion_step = self.step_no
                s.policy_version = self.version
                s.state = FINISHED
                self.finished.append(s)
                self._release(s)
                done.append(s)
        self.gen_tokens += r

        # D. page growth for the survivors; an empty pool preempts the shortest rollout
        preempted = []
        for i in range(Q):
            s = self.slots[i]
            if s is None or self._next_pos(s) // self.pt < len(s.pages):
                continue
            while not self.free:
                live = [x for x in self.slots if x is not None]
                victim = min(live, key=lambda x: (x.gen_len, -x.seq_id))
                self._preempt(victim)
                preempted.append(victim)
            if self.slots[i] is s:                        # s itself may have been the victim
                s.pages.append(self.free.pop())
        self.max_pages_used = max(self.max_pages_used, self.n_pages - len(self.free))

        # E. accounting (eq. 4 with dt = 1 step)
        self.busy += r
        self.idle += Q - r
        if queue_nonempty:
            self.steps_q += 1
            self.idle_q += Q - r
        info = dict(step=self.step_no, r=r, n_active=sum(x is not None for x in self.slots),
                    n_finished_unharvested=len(self.finished), n_queued=len(self.queue),
                    free_pages=len(self.free),
                    admitted=[(s.seq_id, s.last_slot) for s in admitted],
                    finished=[s.seq_id for s in done], preempted=[s.seq_id for s in preempted])
        self.step_no += 1
        return info

    def _preempt(self, s: Seq) -> None:
        self._release(s)
        s.state = QUEUED
        s.n_preempt += 1
        self.n_preempt += 1
        self.queue.appendleft(s)

    # ---- harvest length-ordered update groups (Fig. 2 steps 3-4) ----------------------------
    def harvest(self, group_size: int, flush: bool = False) -> List[List[Seq]]:
        F = sorted(self.finished, key=lambda s: (s.completion_step, s.gen_len, s.seq_id))
        k = len(F) // group_size
        groups = [F[j * group_size:(j + 1) * group_size] for j in range(k)]
        rest = F[k * group_size:]
        drained = not self.queue and all(x is None for x in self.slots)
        if flush and drained and rest:
            groups.append(rest)
            rest = []
        for g in groups:
            for s in g:
                s.state = HARVESTED
                s.group_idx = self.n_groups
            self.n_groups += 1
        self.finished = rest
        if groups:                                        # update boundary: one policy update per group
            self.version += len(groups)
            self._boundary()
        return groups

    def _boundary(self) -> None:
        live = [s for s in self.slots if s is not None]
        if self.mode == MODE_ONPOLICY:
            out = live
        elif self.max_staleness >= 0:
            out = [s for s in live if self.version - s.kv_version > self.max_staleness]
        else:
            out = []
        for s in sorted(out, key=lambda x: x.slot):
            self._release(s)
            s.state = QUEUED
            if self.mode == MODE_ONPOLICY:
                self.discarded_tokens += s.gen_len
                s.tokens, s.logp = [], []
            else:
                self.n_stale += 1
        for s in sorted(out, key=lambda x: -x.seq_id):    # queue front ends up in ascending seq_id
            self.queue.appendleft(s)

    # ---- policy update (Sec. 3.2): later tokens come from the new weights; caches and recorded log-probs stay ------
    def update_weights(self, model) -> None:
        self.model = model

    # ---- reporting ---------------------------------------------------------------------------
    def bubble_ratio(self) -> float:
        return self.idle / (self.Q * self.step_no) if self.step_no else 0.0

    def stats(self) -> dict:
        return dict(steps=self.step_no, busy=self.busy, idle=self.idle, steps_q=self.steps_q,
                    idle_q=self.idle_q, gen_tokens=self.gen_tokens,
                    discarded_tokens=self.discarded_tokens, prefill_tokens=self.prefill_tokens,
                    n_preempt=self.n_preempt, n_stale=self.n_stale, version=self.version,
                    max_pages_used=self.max_pages_used)

    def run_to_completion(self, group_size: int, max_steps: int = 10 ** 9):
        """Bench/test driver: harvest after every step that leaves >= group_size finished."""
        groups = []
        while (self.queue or any(x is not None for x in self.slots)) and self.step_no < max_steps:
            self.step()
            if len(self.finished) >= group_size:
                groups += self.harvest(group_size)
        groups += self.harvest(group_size, flush=True)
        return groups
