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


def batch_requests(requests: Sequence[Request], n_ub: int, ubs: int, gen_len: int,
                   cache_size: int) -> Tuple[List[MicroBatch], List[Request]]:
    """-> (micro_batches, aborted).  n_ub micro-batches of at most ubs requests each."""
    if n_ub < 1 or ubs < 1 or gen_len < 0 or cache_size < 0:
        raise ValueError("n_ub, ubs >= 1 and gen_len, cache_size >= 0 are required")
    open_batches: List[List[Request]] = [[] for _ in range(n_ub)]
    open_tokens: List[int] = [0] * n_ub
    done: List[MicroBatch] = []
    aborted: List[Request] = []
    # longest first; equal lengths keep their arrival order (stable sort)
    for req in sorted(requests, key=lambda r: -r.input_len):
        if not open_batches:
            aborted.append(req)
            continue
        idx = min(range(len(open_batches)), key=lambda i: (open_tokens[i], i))
        need = open_tokens[idx] + req.input_len + (len(open_batches[idx]) + 1) * gen_len
        if need > cache_size:
            aborted.append(req)
            continue
        open_batches[idx].append(req)
        open_tokens[idx] += req.input_len
        if len(open_batches[idx]) == ubs:
            done.append(MicroBatch(open_batches.pop(idx)))
            open_tokens.pop(idx)
    done.extend(MicroBatch(b) for b in open_batches if b)
    return done, aborted
