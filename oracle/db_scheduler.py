"""Plain-Python statement of SeaLLM's doubling-budget (DB) request scheduler (arXiv 2504.15720,
section 4.2 "Latency-Optimized Scheduling", Equation 6 and the DB algorithm of the appendix).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: the product's scheduler is the C++ one behind
include/ukv_sched.h, which shares no code with this file.  Everything here is lists and sorts, in
the paper's notation, so that it can be checked against the text by eye:

  Q_r      budget of request r, initially Q = L_s + Var_s (mean and standard deviation of the
           execution time of the requests of r's service s); it decreases with the time r executes.
  O_r      priority of r, O_r = Q_r * L_s; the smallest O_r is served first.
  doubling when the budget is used up and r is not finished, the budget becomes 2 Q, then 4 Q, ...
           and the priority is reset from the new budget.
  batch    requests of the same service and the same phase (wait_queue = not yet prefilled,
           decoding_queue = prefilled), taken from the queue of the chosen request in priority
           order while EnoughResource() holds.
  starved  a service with queued requests that has not been served for longer than its
           threshold is served first.

Readings where the paper is silent (the same ones the C++ scheduler takes):
  * the execution time of an iteration is charged in full to every request of the batch;
  * EnoughResource(): the batch has fewer than max_batch requests and the pages its next
    iteration needs (the whole prompt for a prefill, the growth by one token for a decode) fit in
    the free pages the caller reports; a candidate that does not fit ends the batch;
  * if the chosen request itself does not fit, the next request in the same order that fits is
    taken instead (otherwise a full pool would stop all work);
  * ties: smaller priority, then earlier arrival, then smaller id;
  * a service's starvation clock starts when it gets its first queued request and restarts
    whenever one of its batches completes; the most overdue starved service goes first.

Pins (tests/test_sched.py): on instances the first theorem of section 4.2 covers (one request per
iteration, equal execution times within a service, everything queued at time 0) the order
attains the minimum of the summed normalized latency over all permutations (brute force); the
budget sequence Q, 2Q, 4Q; starvation; batch invariants; page accounting against a real free list.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

WAIT, DECODING = 0, 1


@dataclass
class ServiceProfile:
    mean_time: float             # L_s
    std_time: float              # Var_s (the paper calls the standard deviation Var)
    starvation_threshold: float
    token_bytes: int


@dataclass
class Request:
    id: int
    service: int
    prompt_len: int
    arrival: float
    queue: int = WAIT
    ctx_len: int = 0             # tokens in the cache
    budget: float = 0.0          # Q_r
    doublings: int = 0
    priority: float = 0.0        # O_r


@dataclass
class DBScheduler:
    services: Sequence[ServiceProfile]
    page_bytes: int
    max_batch: int
    requests: Dict[int, Request] = field(default_factory=dict)
    last_served: Dict[int, float] = field(default_factory=dict)

    # ---- InitBudget / InitPriority / wait_queue.AddRequest
    def add_request(self, rid: int, service: int, prompt_len: int, now: float) -> None:
        assert rid not in self.requests and prompt_len >= 1
        s = self.services[service]
        if not any(r.service == service for r in self.requests.values()):
            self.last_served[service] = now
        q = s.mean_time + s.std_time
        self.requests[rid] = Request(rid, service, prompt_len, now, WAIT, 0, q, 0, q * s.mean_time)

    def _pages(self, service: int, n_tokens: int) -> int:
        return -(-n_tokens * self.services[service].token_bytes // self.page_bytes)

    def pages_needed(self, r: Request) -> int:
        if r.queue == WAIT:
            return self._pages(r.service, r.prompt_len)
        return self._pages(r.service, r.ctx_len + 1) - self._pages(r.service, r.ctx_len)

    @staticmethod
    def _key(r: Request) -> Tuple[float, float, int]:
        return (r.priority, r.arrival, r.id)

    def _starved_service(self, now: float) -> Optional[int]:
        best, best_over = None, 0.0
        for s in sorted({r.service for r in self.requests.values()}):
            over = now - self.last_served[s] - self.services[s].starvation_threshold
            if over > 0.0 and (best is None or over > best_over):
                best, best_over = s, over
        return best

    # ---- "Schedule requests": returns (ids, service, queue)
    def next_batch(self, now: float, free_pages: int) -> Tuple[List[int], int, int]:
        if not self.requests:
            return [], 0, WAIT
        order = sorted(self.requests.values(), key=self._key)
        starved = self._starved_service(now)
        if starved is not None:          # GetHighestPriorityOrStarvedRequest: that service's requests first
            order = [r for r in order if r.service == starved] + [r for r in order if r.service != starved]
        first = next((r for r in order if self.pages_needed(r) <= free_pages), None)
        if first is None:
            return [], order[0].service, order[0].queue
        batch, used = [], 0
        cur_queue = [r for r in sorted(self.requests.values(), key=self._key) if r.queue == first.queue]
        for r in [first] + [x for x in cur_queue if x is not first]:
            if r.service != first.service:
                continue
            need = self.pages_needed(r)
            if len(batch) >= self.max_batch or used + need > free_pages:   # EnoughResource() fails
                break
            batch.append(r.id)
            used += need
        return batch, first.service, first.queue

    # ---- Execute happened outside; UpdateBudget / UpdatePriority
    def complete(self, ids: Sequence[int], finished: Sequence[bool], elapsed: float, now: float) -> None:
        service = None
        for rid, fin in zip(ids, finished):
            r = self.requests[rid]
            service = r.service
            s = self.services[r.service]
            if r.queue == WAIT:
                r.queue, r.ctx_len = DECODING, r.prompt_len
            else:
                r.ctx_len += 1
            if fin:
                del self.requests[rid]
                continue
            r.budget -= elapsed
            if r.budget <= 0.0:
                r.doublings += 1
                r.budget = (s.mean_time + s.std_time) * float(2 ** r.doublings)
            r.priority = r.budget * s.mean_time
        if service is not None:
            self.last_served[service] = now
