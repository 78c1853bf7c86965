"""Request batching: variable-length requests into micro-batches of balanced token counts
(the paper's appendix A.2, Algorithm 2).  Host logic only; it decides the token count T
that each kernel execution of the MoE layer sees.

What is computed, in this module's own words.  Requests are taken longest prompt first.
Each goes to the OPEN micro-batch that currently holds the fewest prompt tokens (ties: the
lowest index).  A micro-batch must be able to hold the KV cache of its requests until the
end of generation: if prompt tokens plus gen_len tokens for every request, including the new
one, would exceed cache_size, the request is not placed but returned as aborted, to be
offered again with the next batch.  A micro-batch that reaches ubs requests is closed and
emitted; once all n_ub micro-batches are closed the remaining requests are aborted too.
Micro-batches that are still open at the end are emitted as they are (the listing in the
paper returns only the closed ones; keeping the partly filled ones is this module's
reading, since otherwise requests would be lost without being reported as aborted).
"""
from __future__ import annotations

import dataclasses
import heapq
from typing import List, Sequence, Tuple


@dataclasses.dataclass(frozen=True)
class Request:
    rid: int
    input_len: int


@dataclasses.dataclass
class MicroBatch:
    requests: List[Request]

    @property
    def prompt_tokens(self) -> int:
        """Tokens one prefill kernel execution sees."""
        return sum(r.input_len for r in self.requests)

    @property
    def decode_tokens(self) -> int:
        """Tokens one decode kernel execution sees: one per request."""
        return len(self.requests)


class _OpenBatch:
    """A micro-batch that still takes requests.  It keeps its own running totals and answers the two
    questions of appendix A.2 itself: would one more request overflow the cache, and is it full."""

    __slots__ = ("slot", "tokens", "members")

    def __init__(self, slot: int):
        self.slot, self.tokens, self.members = slot, 0, []

    def load(self) -> Tuple[int, int]:
        return (self.tokens, self.slot)                    # lightest first, the older slot on a tie

    def cache_after(self, req: Request, gen_len: int) -> int:
        """KV-cache entries at the end of generation if req joined: all prompts plus gen_len per request."""
        return self.tokens + req.input_len + (len(self.members) + 1) * gen_len

    def add(self, req: Request) -> None:
        self.members.append(req)
        self.tokens += req.input_len

    def full(self, ubs: int) -> bool:
        return len(self.members) >= ubs


def batch_requests(requests: Sequence[Request], n_ub: int, ubs: int, gen_len: int,
                   cache_size: int) -> Tuple[List[MicroBatch], List[Request]]:
    """-> (micro_batches, aborted).  n_ub micro-batches of at most ubs requests each."""
    if n_ub < 1 or ubs < 1 or gen_len < 0 or cache_size < 0:
        raise ValueError("n_ub, ubs >= 1 and gen_len, cache_size >= 0 are required")
    heap = [(b.load(), b) for b in map(_OpenBatch, range(n_ub))]      # already a valid heap: all loads (0, slot)
    closed: List[_OpenBatch] = []
    aborted: List[Request] = []
    by_length = sorted(requests, key=lambda r: r.input_len, reverse=True)   # stable: equal lengths keep arrival order
    for pos, req in enumerate(by_length):
        if not heap:                                       # every micro-batch is closed: the rest waits for the next batch
            aborted.extend(by_length[pos:])
            break
        lightest = heap[0][1]
        if lightest.cache_after(req, gen_len) > cache_size:
            aborted.append(req)
            continue
        lightest.add(req)
        if lightest.full(ubs):
            heapq.heappop(heap)
            closed.append(lightest)
        else:
            heapq.heapreplace(heap, (lightest.load(), lightest))
    still_open = sorted((b for _, b in heap if b.members), key=lambda b: b.slot)
    return [MicroBatch(b.members) for b in closed + still_open], aborted
