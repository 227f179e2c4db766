"""TEST INFRASTRUCTURE ONLY -- plain Python reference of the paper's phase-specific schedulers and of the
iteration loop they drive.

What it follows:

* Sec. 4.3.1, Eq. 10 and Alg. 2: Shortest Prompt First.  Every waiting request gets the score
  remaining - gamma * age; the queue is sorted by score and requests are taken in that order while the batch's
  token total stays within the budget B; the first request that does not fit ends the batch.
* Sec. 4.3.1: FCFS as the policy SPF is compared with (same filling rule, arrival order).
* Sec. 4.3.2: decode is First-Come-First-Serve, one token per running request per iteration.
* Sec. 5: prefill and decode queues are kept independently; chunked prefill with the engine's chunk size.
* Sec. 6.1 metrics: TTFT (arrival to first token), TBT (time between consecutive tokens of a request),
  normalised latency (end-to-end latency over the number of output tokens).

Readings taken where the paper leaves a choice (marked "reading" where they occur in the code):

* Alg. 2 scores `remaining`, Eq. 10 the prompt length: `remaining` is used (they agree until a request has been
  partly prefilled).  Age is in seconds, gamma in tokens per second.  Ties: earlier arrival, then lower id.
* Alg. 2 as printed never schedules a request whose remaining prompt exceeds B.  With chunked prefill (Sec. 5) the
  first request that does not fit takes what is left of the budget as a partial chunk, then the batch ends.
  `chunk_tail=False` gives the printed rule.
* A request emits its first token when its last prompt chunk completes, and joins the decode pool (capacity
  `max_decode`) in the order of those completions; a decode step at context c stores the token at position c.
* A request is admitted to its first chunk only when the pages of its whole lifetime (prompt + output - 1 tokens)
  can be reserved, so no request ever stalls for KV space in flight; physical pages are taken from the free list
  only as positions get written.  A request that cannot be admitted holds back every not yet admitted request
  behind it in the order (no overtaking), but not the requests that already are.

Nothing here is imported by the product.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

FCFS, SPF = 0, 1


@dataclass
class Request:
    rid: int
    arrival: float
    prompt_len: int
    output_len: int
    prefilled: int = 0
    emitted: int = 0
    pages: List[int] = field(default_factory=list)
    reserved: int = 0
    admitted: bool = False
    ready_time: Optional[float] = None
    in_pool: bool = False
    first_token_time: Optional[float] = None
    last_token_time: Optional[float] = None
    finish_time: Optional[float] = None
    tbt: List[float] = field(default_factory=list)

    @property
    def remaining(self) -> int:
        return self.prompt_len - self.prefilled


def spf_score(remaining: int, age: float, gamma: float) -> float:
    """Alg. 2, the score line."""
    return remaining - gamma * age


def order_queue(queue: Sequence[Request], now: float, policy: int, gamma: float) -> List[Request]:
    if policy == FCFS:
        return sorted(queue, key=lambda r: (r.arrival, r.rid))
    return sorted(queue, key=lambda r: (spf_score(r.remaining, now - r.arrival, gamma), r.arrival, r.rid))


def fill_batch(ordered: Sequence[Request], budget: int, chunk_tail: bool = True,
               max_reqs: Optional[int] = None) -> List[Tuple[Request, int]]:
    """The greedy filling loop of Alg. 2 on an already ordered queue: (request, tokens taken) pairs."""
    batch: List[Tuple[Request, int]] = []
    total = 0
    for r in ordered:
        if max_reqs is not None and len(batch) == max_reqs:
            break
        if total + r.remaining <= budget:
            batch.append((r, r.remaining))
            total += r.remaining
        else:
            if chunk_tail and budget - total > 0:
                batch.append((r, budget - total))
            break
    return batch


def pages_for(tokens: int, page_size: int) -> int:
    return (tokens + page_size - 1) // page_size


@dataclass
class Iteration:
    now: float
    prefill: List[Tuple[int, int, int]]   # (request id, prefix length, chunk length)
    decode: List[Tuple[int, int]]         # (request id, context length before the step)
    page_tables: Dict[int, List[int]]     # request id -> pages it holds during the step
    kv_used_pages: int


class Loop:
    """The iteration loop: submit() requests, then alternate next(now) and commit(end)."""

    def __init__(self, policy: int, budget: int, max_decode: int, page_size: int, n_pages: int, gamma: float = 15.0,
                 chunk_tail: bool = True, max_prefill_reqs: Optional[int] = None,
                 priority: Optional[Callable[[Sequence[Request], float], List[Request]]] = None):
        self.policy, self.budget, self.max_decode, self.page_size = policy, budget, max_decode, page_size
        self.gamma, self.chunk_tail, self.max_prefill_reqs = gamma, chunk_tail, max_prefill_reqs
        self.priority = priority            # test hook: an arbitrary ordering instead of FCFS / SPF
        self.n_pages = n_pages
        self.free = list(range(n_pages - 1, -1, -1))   # pop() hands out 0, 1, 2, ...
        self.reserved_total = 0
        self.reqs: List[Request] = []
        self.pool: List[Request] = []
        self._pending_prefill: Optional[List[Tuple[Request, int]]] = None
        self._pending_decode: Optional[List[Request]] = None
        self.prefill_tokens = 0
        self.decode_tokens = 0

    def submit(self, arrival: float, prompt_len: int, output_len: int) -> int:
        assert prompt_len >= 1 and output_len >= 1
        assert pages_for(prompt_len + output_len - 1, self.page_size) <= self.n_pages, "can never be admitted"
        r = Request(len(self.reqs), arrival, prompt_len, output_len)
        self.reqs.append(r)
        return r.rid

    def _grow(self, r: Request, tokens: int) -> None:
        while len(r.pages) < pages_for(tokens, self.page_size):
            r.pages.append(self.free.pop())

    # ---- the two phases tick independently (Sec. 5: separate coroutines, each with its own scheduler); the
    # ---- coupled iteration below is one tick of each
    def next_prefill(self, now: float) -> List[Tuple[int, int, int]]:
        assert self._pending_prefill is None
        waiting = [r for r in self.reqs if r.arrival <= now and r.remaining > 0]
        ordered = self.priority(waiting, now) if self.priority else order_queue(waiting, now, self.policy, self.gamma)
        # admission, in priority order: once a request's lifetime does not fit, no new request is admitted in this
        # iteration (nothing passes it), while requests admitted earlier keep their place in the order
        admitted: List[Request] = []
        blocked = False
        for r in ordered:
            if not r.admitted:
                need = pages_for(r.prompt_len + r.output_len - 1, self.page_size)
                if blocked or self.reserved_total + need > self.n_pages:
                    blocked = True
                    continue
                r.admitted, r.reserved = True, need
                self.reserved_total += need
            admitted.append(r)
        batch = fill_batch(admitted, self.budget, self.chunk_tail, self.max_prefill_reqs)
        prefill = []
        for r, take in batch:
            self._grow(r, r.prefilled + take)
            prefill.append((r.rid, r.prefilled, take))
        self._pending_prefill = batch or None       # an empty batch is not an iteration: nothing to commit
        return prefill

    def next_decode(self, now: float) -> List[Tuple[int, int]]:
        assert self._pending_decode is None
        # decode pool: first come (first prefilled), first served
        ready = sorted((r for r in self.reqs if r.ready_time is not None and not r.in_pool and r.finish_time is None),
                       key=lambda r: (r.ready_time, r.arrival, r.rid))
        for r in ready:
            if len(self.pool) == self.max_decode:
                break
            r.in_pool = True
            self.pool.append(r)
        decode = []
        for r in self.pool:
            ctx = r.prompt_len + r.emitted - 1
            self._grow(r, ctx + 1)
            decode.append((r.rid, ctx))
        self._pending_decode = list(self.pool) or None
        return decode

    def page_table(self, rid: int) -> List[int]:
        return list(self.reqs[rid].pages)

    @property
    def kv_used_pages(self) -> int:
        return self.n_pages - len(self.free)

    def _finish(self, r: Request, end: float) -> None:
        r.finish_time = end
        self.free.extend(reversed(r.pages))
        r.pages = []
        self.reserved_total -= r.reserved
        r.reserved = 0

    def commit_decode(self, end: float) -> None:
        assert self._pending_decode is not None
        for r in self._pending_decode:
            r.emitted += 1
            self.decode_tokens += 1
            r.tbt.append(end - r.last_token_time)
            r.last_token_time = end
            if r.emitted == r.output_len:
                self.pool.remove(r)
                r.in_pool = False
                self._finish(r, end)
        self._pending_decode = None

    def commit_prefill(self, end: float) -> None:
        assert self._pending_prefill is not None
        for r, take in self._pending_prefill:
            r.prefilled += take
            self.prefill_tokens += take
            if r.remaining == 0:
                r.emitted = 1
                r.first_token_time = r.last_token_time = end
                if r.output_len == 1:
                    self._finish(r, end)
                else:
                    r.ready_time = end
        self._pending_prefill = None

    # ---- the coupled iteration: both phases start together and the iteration ends when both have
    def next(self, now: float) -> Iteration:
        prefill = self.next_prefill(now)
        decode = self.next_decode(now)
        tables = {rid: self.page_table(rid) for rid, _, _ in prefill}
        tables.update({rid: self.page_table(rid) for rid, _ in decode})
        return Iteration(now, prefill, decode, tables, self.kv_used_pages)

    def commit(self, end: float) -> None:
        if self._pending_decode is not None:
            self.commit_decode(end)
        if self._pending_prefill is not None:
            self.commit_prefill(end)

    # ---- metrics (Sec. 6.1)
    def ttft(self) -> List[float]:
        return [r.first_token_time - r.arrival for r in self.reqs if r.first_token_time is not None]

    def tbt(self) -> List[float]:
        return [x for r in self.reqs for x in r.tbt]

    def normalized_latency(self) -> List[float]:
        return [(r.finish_time - r.arrival) / r.output_len for r in self.reqs if r.finish_time is not None]


def run_virtual(loop: Loop, n_iterations: int, dt: float) -> List[Iteration]:
    """Fixed-duration iterations: iteration i starts at i dt and ends at (i + 1) dt."""
    out = []
    for i in range(n_iterations):
        out.append(loop.next(i * dt))
        loop.commit((i + 1) * dt)
    return out
