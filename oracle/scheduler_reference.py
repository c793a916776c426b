"""TEST INFRASTRUCTURE ONLY -- one iteration of stall-free batching (paper Algorithm 3, section 4.2).

The scheduler fills the next batch in three passes under a token budget tau:
first every running decode (one token each), then the next chunk of every request whose
prefill is under way, then new requests in arrival order while memory and budget last.
The chunk given to a prefill is the largest that the leftover budget admits.

Readings where the paper's listing is silent or garbled (each is also listed in the design notes):

* the chunk is ``min(prompt tokens left, chunk_size, tau - n_t)`` and 0 once ``n_t >= tau``;
  ``chunk_size`` is a separate cap (the listing has only tau);
* decodes count against tau but are never dropped because of it (the text: decodes never
  stall); only ``max_batch_size`` bounds them, and exceeding it is reported as an error;
* the admission loop adds the new request to the batch (the listing prints an assignment)
  and fetches the next waiting request after each admission (as Algorithm 2 does);
* ``can_allocate_request`` = the whole prompt's pages fit into ``free_pages``; admitted
  prompts reserve their pages at once; parity for this policy is unpinned by the paper;
* at most one chunk per request per iteration; batch order = decodes, running prefills, new.

A request is ``(id, prompt_len, num_prefilled, num_decoded)``:
``num_prefilled`` prompt tokens already have their K/V cached; a request with a complete
prefill has ``num_decoded`` generated tokens cached and feeds one more this iteration.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

Request = Tuple[int, int, int, int]  # id, prompt_len, num_prefilled, num_decoded


@dataclass
class Batch:
    seq_id: List[int]
    q_start: List[int]
    q_len: List[int]
    ctx_len: List[int]
    num_decodes: int
    num_prefill_chunks: int
    num_admitted: int
    free_pages_left: int

    @property
    def num_tokens(self) -> int:
        return sum(self.q_len)


def next_chunk_size(prompt_len: int, num_prefilled: int, chunk_size: int, token_budget: int, n_t: int) -> int:
    if n_t >= token_budget:
        return 0
    return max(0, min(prompt_len - num_prefilled, chunk_size, token_budget - n_t))


def build_stall_free_batch(token_budget: int, chunk_size: int,
                           running_decodes: Sequence[Request],
                           running_prefills: Sequence[Request],
                           waiting_prefills: Sequence[Request],
                           free_pages: int, page_size: int, max_batch_size: int) -> Batch:
    if len(running_decodes) > max_batch_size:
        raise OverflowError("more running decodes than max_batch_size")
    ids, q_len, ctx_len = [], [], []
    n_t = 0
    # pass 1: every running decode, one token each
    for (rid, prompt_len, num_prefilled, num_decoded) in running_decodes:
        assert num_prefilled == prompt_len
        n_t += 1
        ids.append(rid)
        q_len.append(1)
        ctx_len.append(prompt_len + num_decoded + 1)
    n_dec = len(ids)
    # pass 2: requests whose prefill is under way
    n_chunks = 0
    for (rid, prompt_len, num_prefilled, _nd) in running_prefills:
        if len(ids) >= max_batch_size:
            break
        c = next_chunk_size(prompt_len, num_prefilled, chunk_size, token_budget, n_t)
        if c > 0:
            n_t += c
            ids.append(rid)
            q_len.append(c)
            ctx_len.append(num_prefilled + c)
            n_chunks += 1
    # pass 3: new requests, first come first served
    admitted = 0
    for (rid, prompt_len, num_prefilled, _nd) in waiting_prefills:
        pages = (prompt_len + page_size - 1) // page_size
        if not (pages <= free_pages and n_t < token_budget and len(ids) < max_batch_size):
            break
        c = next_chunk_size(prompt_len, num_prefilled, chunk_size, token_budget, n_t)
        if c <= 0:
            break
        n_t += c
        free_pages -= pages
        ids.append(rid)
        q_len.append(c)
        ctx_len.append(num_prefilled + c)
        n_chunks += 1
        admitted += 1
    q_start = [0] * len(ids)
    for i in range(1, len(ids)):
        q_start[i] = q_start[i - 1] + q_len[i - 1]
    return Batch(ids, q_start, q_len, ctx_len, n_dec, n_chunks, admitted, free_pages)
