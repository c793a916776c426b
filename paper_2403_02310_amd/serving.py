"""Serving loop around the hot path: many scheduling iterations over a request trace.

Each iteration builds a batch (stall-free batching, Algorithm 3 of section 4.2, through
``sarathi_build_stall_free_batch``), grows the paged KV cache of the scheduled sequences,
appends their new K/V rows and runs hybrid-batch attention (``sarathi_kv_append``,
``sarathi_hybrid_attention``).  Only attention runs (there is no model around it), so iteration
times are a PROXY for the paper's time-between-tokens: they show how the cost of an iteration
varies with what the scheduler put into it, not end-to-end latency.

Two scheduling policies can drive the same kernels:

* ``stall_free``: Algorithm 3 (decodes first, prefills chunked into the leftover token budget).
* ``prefill_first``: a toy stand-in for prefill-prioritising iteration-level schedulers (section
  3.2): while any request waits for (the rest of) its prefill, an iteration holds whole prompts
  only and the running decodes stall.  It exists to contrast iteration times, nothing more.

Query/key/value rows are synthetic: every request owns pre-drawn rows for all its positions
(prompt and generated tokens), so a request's attention outputs can be checked afterwards
against a one-shot computation over its whole sequence, whatever batches it travelled in.

A ``backend`` supplies device memory and runs the two device calls; ``DryBackend`` (no GPU)
only keeps the books and is what the host-logic tests use.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from .workloads import AttnShape


@dataclass
class Request:
    id: int
    arrival_s: float
    prompt_len: int
    output_len: int            # generated tokens wanted; the first comes out of the prefill
    token_base: int = 0        # first row of this request in the per-token tensors
    num_prefilled: int = 0
    num_decoded: int = 0       # generated tokens whose K/V are cached
    slot: int = -1             # row of the block table
    pages: List[int] = field(default_factory=list)
    first_token_s: float = -1.0
    last_token_s: float = -1.0
    finish_s: float = -1.0

    @property
    def total_rows(self) -> int:
        return self.prompt_len + max(0, self.output_len - 1)

    @property
    def prefill_done(self) -> bool:
        return self.num_prefilled == self.prompt_len

    @property
    def finished(self) -> bool:
        return self.prefill_done and self.num_decoded >= self.output_len - 1


def synthetic_trace(seed: int, n_requests: int, qps: float, prompt_median: float = 1730, prompt_p90: float = 5696,
                    output_median: float = 415, output_p90: float = 834, max_prompt: int = 8192,
                    max_output: int = 1024) -> List[Request]:
    """Poisson arrivals; prompt and output lengths log-normal with the given median and 90th percentile
    (defaults: the conversation trace's statistics in the paper's Table 2), clipped."""
    rng = np.random.default_rng([seed, 0x5E])
    z90 = 1.2815515655446004
    def draw(median, p90, lo, hi):
        sigma = np.log(p90 / median) / z90
        x = np.exp(np.log(median) + sigma * rng.standard_normal(n_requests))
        return np.clip(np.rint(x), lo, hi).astype(np.int64)
    prompts = draw(prompt_median, prompt_p90, 1, max_prompt)
    outputs = draw(output_median, output_p90, 1, max_output)
    arrivals = np.cumsum(rng.exponential(1.0 / qps, size=n_requests))
    reqs, base = [], 0
    for i in range(n_requests):
        r = Request(i, float(arrivals[i]), int(prompts[i]), int(outputs[i]), token_base=base)
        base += r.total_rows
        reqs.append(r)
    return reqs


class PagePool:
    """Free list of cache pages (handed out in a seeded random order: pages of a sequence are scattered)."""

    def __init__(self, num_pages: int, seed: int = 0):
        self.num_pages = num_pages
        self._free = np.random.default_rng([seed, 0x9A]).permutation(num_pages).tolist()

    @property
    def free(self) -> int:
        return len(self._free)

    def take(self, n: int) -> List[int]:
        if n > len(self._free):
            raise RuntimeError("page pool exhausted: %d wanted, %d free" % (n, len(self._free)))
        out = self._free[-n:] if n else []
        del self._free[len(self._free) - n:]
        return out

    def give(self, pages: Sequence[int]) -> None:
        self._free.extend(pages)


@dataclass
class IterationRecord:
    start_s: float
    duration_s: float
    num_tokens: int
    num_decodes: int
    num_prefill_tokens: int
    num_seqs: int
    num_running_decodes: int   # requests in their decode phase when the iteration was scheduled


class DryBackend:
    """No device: iteration time from a cost model ``cost(q_len, ctx_len) -> seconds``."""

    def __init__(self, cost: Optional[Callable[[np.ndarray, np.ndarray], float]] = None):
        self.cost = cost or (lambda q_len, ctx_len: 20e-6 + 1e-9 * float((q_len.astype(np.float64) * ctx_len).sum()))

    def setup(self, loop: "ServingLoop") -> None:
        pass

    def set_block_entries(self, slot: int, first_block: int, pages: Sequence[int]) -> None:
        pass

    def run(self, loop: "ServingLoop", slots, token_rows, q_start, q_len, ctx_len) -> float:
        return self.cost(np.asarray(q_len), np.asarray(ctx_len))


class GpuBackend:
    """Device memory (torch) + the two device entry points.  Fails loudly if the library is missing."""

    def __init__(self, seed: int = 0, keep_outputs: bool = True, options: Optional[Dict[str, int]] = None,
                 linear_model: Optional[str] = None):
        """``linear_model`` (a key of ``linear_layers.MODELS``): every iteration also runs the four linear layers of
        one transformer layer of that model over the iteration's tokens (random weights, outputs unused), so that the
        timed iteration holds the operators that dominate a real one (section 3.1), not attention alone."""
        import torch
        from . import binding
        self.torch, self.binding = torch, binding
        self.seed, self.keep_outputs, self.options = seed, keep_outputs, dict(options or {})
        self.linear_model = linear_model
        self.linear = []

    def setup(self, loop: "ServingLoop") -> None:
        torch, s = self.torch, loop.shape
        total = sum(r.total_rows for r in loop.requests)
        g = torch.Generator(device="cuda").manual_seed(self.seed)
        draw = lambda heads: torch.randn(total, heads, s.head_dim, device="cuda", generator=g).to(torch.bfloat16)
        self.q_all, self.k_all, self.v_all = draw(s.num_q_heads), draw(s.num_kv_heads), draw(s.num_kv_heads)
        self.out_all = torch.zeros_like(self.q_all) if self.keep_outputs else None
        self.k_cache = torch.zeros(loop.pool.num_pages, s.num_kv_heads, s.page_size, s.head_dim, device="cuda", dtype=torch.bfloat16)
        self.v_cache = torch.zeros(loop.pool.num_pages, s.num_kv_heads, s.head_dim, s.page_size, device="cuda", dtype=torch.bfloat16)
        self.bt_all = torch.full((loop.max_seqs, loop.max_blocks), -1, device="cuda", dtype=torch.int32)
        self.handle = self.binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=loop.max_tokens,
                                          max_seqs=loop.max_seqs, max_blocks_per_seq=loop.max_blocks)
        for k, v in self.options.items():
            self.handle.set_option(k, v)
        self.sm_scale = 1.0 / float(np.sqrt(s.head_dim))
        self._ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        if self.linear_model:
            from . import linear_layers as ll
            scratch = 16
            for _, n, k in ll.layer_shapes(ll.MODELS[self.linear_model]):
                w = torch.randn(n, k, device="cuda", generator=g).to(torch.bfloat16)
                x = torch.randn(loop.max_tokens, k, device="cuda", generator=g).to(torch.bfloat16)
                y = torch.empty(loop.max_tokens, n, device="cuda", dtype=torch.bfloat16)
                self.linear.append((x, w, y))
                scratch = max([scratch] + [self.binding.linear_workspace_bytes(t, n, k)
                                           for t in (16, 32, 64, 128, 256, 512, loop.max_tokens) if t <= loop.max_tokens])
            self.linear_scratch = torch.empty(scratch, dtype=torch.uint8, device="cuda")

    def set_block_entries(self, slot: int, first_block: int, pages: Sequence[int]) -> None:
        t = self.torch.tensor(list(pages), dtype=self.torch.int32)
        self.bt_all[slot, first_block:first_block + len(pages)] = t.cuda()

    def run(self, loop: "ServingLoop", slots, token_rows, q_start, q_len, ctx_len) -> float:
        torch = self.torch
        rows = torch.from_numpy(np.asarray(token_rows, dtype=np.int64)).cuda()
        bt = self.bt_all.index_select(0, torch.from_numpy(np.asarray(slots, dtype=np.int64)).cuda())
        q, k_new, v_new = self.q_all.index_select(0, rows), self.k_all.index_select(0, rows), self.v_all.index_select(0, rows)
        out = torch.empty_like(q)
        q_start, q_len, ctx_len = (np.asarray(a, dtype=np.int32) for a in (q_start, q_len, ctx_len))
        self._ev[0].record()
        self.handle.kv_append(k_new, v_new, self.k_cache, self.v_cache, bt, q_start, q_len, ctx_len)
        self.handle.hybrid_attention(q, self.k_cache, self.v_cache, bt, q_start, q_len, ctx_len, self.sm_scale, out)
        n_tok = int(q.shape[0])
        for x, w, y in self.linear:   # a smaller workspace than a token count would like only means fewer pieces
            self.binding.linear(x[:n_tok], w, y[:n_tok], self.linear_scratch)
        self._ev[1].record()
        self._ev[1].synchronize()
        if self.out_all is not None:
            self.out_all.index_copy_(0, rows, out)
        return self._ev[0].elapsed_time(self._ev[1]) * 1e-3


class ServingLoop:
    def __init__(self, shape: AttnShape, requests: Sequence[Request], backend, num_pages: int, token_budget: int = 512,
                 chunk_size: int = 512, max_batch_size: int = 256, policy: str = "stall_free", seed: int = 0):
        if policy not in ("stall_free", "prefill_first"):
            raise ValueError("unknown policy %r" % policy)
        self.shape, self.backend, self.policy = shape, backend, policy
        self.requests = [Request(r.id, r.arrival_s, r.prompt_len, r.output_len, r.token_base) for r in requests]
        self.token_budget, self.chunk_size, self.max_batch_size = token_budget, chunk_size, max_batch_size
        self.pool = PagePool(num_pages, seed)
        longest = max(r.total_rows for r in self.requests)
        self.max_blocks = (longest + shape.page_size - 1) // shape.page_size
        self.max_seqs = max_batch_size
        self.max_tokens = max(token_budget + max_batch_size, max(r.prompt_len for r in self.requests) if policy == "prefill_first" else 0)
        self._free_slots = list(range(self.max_seqs - 1, -1, -1))
        self.now = 0.0
        self.iterations: List[IterationRecord] = []
        self.tbt_s: List[float] = []          # gaps between consecutive generated tokens of a request
        self.waiting: List[Request] = []
        self.prefilling: List[Request] = []
        self.decoding: List[Request] = []
        self.done: List[Request] = []
        self._next_arrival = 0
        backend.setup(self)

    # ---- scheduling -----------------------------------------------------------------
    def _admit_arrivals(self) -> None:
        while self._next_arrival < len(self.requests) and self.requests[self._next_arrival].arrival_s <= self.now:
            self.waiting.append(self.requests[self._next_arrival])
            self._next_arrival += 1

    def _lifetime_pages(self, r: Request) -> int:
        return (r.total_rows + self.shape.page_size - 1) // self.shape.page_size

    def _admissible(self):
        """Pages that new requests may claim, and the first-come-first-served prefix of the waiting list that fits.

        The scheduler's own memory test looks at a prompt's pages only (Algorithm 3 leaves ``can_allocate_request``
        open; the library reserves the prompt).  A running request keeps growing by one page every 16 generated
        tokens, and decodes must never stall (section 4.2), least of all on memory: so this loop sets aside, at
        admission, the pages a request will need over its whole life, and only offers the scheduler the waiting
        requests whose lifetime need fits into what is neither in use nor set aside."""
        set_aside = sum(self._lifetime_pages(r) - len(r.pages) for r in self.prefilling + self.decoding)
        avail = self.pool.free - set_aside
        n_ok, claimed = 0, 0
        for r in self.waiting:
            need = self._lifetime_pages(r)
            if claimed + need > avail:
                break
            claimed += need
            n_ok += 1
        return max(avail, 0), n_ok

    def _schedule(self):
        """Returns [(request, q_len)] in batch order and how many waiting requests entered."""
        by_id = {r.id: r for r in self.waiting + self.prefilling + self.decoding}
        avail, n_ok = self._admissible()
        if self.policy == "stall_free":
            from . import binding
            tup = lambda r: (r.id, r.prompt_len, r.num_prefilled, r.num_decoded)
            b = binding.build_stall_free_batch(self.token_budget, self.chunk_size, [tup(r) for r in self.decoding],
                                               [tup(r) for r in self.prefilling], [tup(r) for r in self.waiting[:n_ok]],
                                               avail, self.shape.page_size, min(self.max_batch_size, len(self._free_slots) + len(self.prefilling) + len(self.decoding)))
            return [(by_id[i], n) for i, n in zip(b["seq_id"], b["q_len"])], b["num_admitted"]
        # prefill_first: whole prompts of waiting requests while any wait (decodes stall), else all decodes
        batch, admitted, tokens, pages_left = [], 0, 0, avail
        for r in self.waiting[:n_ok]:
            pages = self._lifetime_pages(r)
            if pages > pages_left or len(batch) >= len(self._free_slots) or (batch and tokens + r.prompt_len > self.max_tokens):
                break
            batch.append((r, r.prompt_len))
            tokens += r.prompt_len
            pages_left -= pages
            admitted += 1
        if not batch:
            batch = [(r, 1) for r in self.decoding]
        return batch, admitted

    # ---- one iteration ----------------------------------------------------------------
    def step(self) -> Optional[IterationRecord]:
        self._admit_arrivals()
        if not (self.waiting or self.prefilling or self.decoding):
            if self._next_arrival >= len(self.requests):
                return None
            self.now = self.requests[self._next_arrival].arrival_s  # idle until the next request
            self._admit_arrivals()
        running_decodes = len(self.decoding)
        batch, admitted = self._schedule()
        if not batch:
            raise RuntimeError("scheduler produced an empty batch with work pending (the pool cannot hold the next request's "
                               "prompt and generated tokens even when nothing else runs?)")
        page = self.shape.page_size
        for r in self.waiting[:admitted]:     # admission reserves the whole prompt's pages
            r.slot = self._free_slots.pop()
            r.pages = self.pool.take((r.prompt_len + page - 1) // page)
            self.backend.set_block_entries(r.slot, 0, r.pages)
            self.prefilling.append(r)
        del self.waiting[:admitted]
        slots, rows, q_start, q_len, ctx_len, n_dec = [], [], [], [], [], 0
        for r, n in batch:
            pos = r.num_prefilled if not r.prefill_done else r.prompt_len + r.num_decoded
            need = (pos + n + page - 1) // page - len(r.pages)
            if need > 0:                      # a generated token crosses into a new page
                new = self.pool.take(need)
                self.backend.set_block_entries(r.slot, len(r.pages), new)
                r.pages.extend(new)
            slots.append(r.slot)
            q_start.append(len(rows))
            q_len.append(n)
            ctx_len.append(pos + n)
            rows.extend(range(r.token_base + pos, r.token_base + pos + n))
            n_dec += int(r.prefill_done)
        dt = self.backend.run(self, slots, rows, q_start, q_len, ctx_len)
        rec = IterationRecord(self.now, dt, len(rows), n_dec, len(rows) - n_dec, len(batch), running_decodes)
        self.iterations.append(rec)
        self.now += dt
        for r, n in batch:                    # every scheduled sequence but an unfinished prefill emits a token now
            if r.prefill_done:
                r.num_decoded += 1
            else:
                r.num_prefilled += n
                if not r.prefill_done:
                    continue
                self.prefilling.remove(r)
                self.decoding.append(r)
                r.first_token_s = self.now
            if r.last_token_s >= 0:
                self.tbt_s.append(self.now - r.last_token_s)
            r.last_token_s = self.now
            if r.finished:
                r.finish_s = self.now
                self.decoding.remove(r)
                self.pool.give(r.pages)
                r.pages = []
                self._free_slots.append(r.slot)
                self.done.append(r)
        return rec

    def run(self, max_iterations: int = 10 ** 9) -> "ServingLoop":
        for _ in range(max_iterations):
            if self.step() is None:
                break
        return self

    # ---- summaries ----------------------------------------------------------------------
    def summary(self) -> dict:
        it = np.array([r.duration_s for r in self.iterations]) * 1e6
        with_dec = np.array([r.duration_s for r in self.iterations if r.num_decodes > 0]) * 1e6
        tbt = np.array(self.tbt_s) * 1e6
        ttft = np.array([r.first_token_s - r.arrival_s for r in self.done]) * 1e6
        pct = lambda a, p: float(np.percentile(a, p)) if len(a) else 0.0
        return {"policy": self.policy, "iterations": len(self.iterations), "requests_done": len(self.done),
                "makespan_s": self.now, "generated_tokens": int(sum(r.output_len for r in self.done)),
                "iteration_us": {"p50": pct(it, 50), "p99": pct(it, 99), "max": pct(it, 100)},
                "iteration_with_decodes_us": {"p50": pct(with_dec, 50), "p99": pct(with_dec, 99), "max": pct(with_dec, 100)},
                "tbt_proxy_us": {"p50": pct(tbt, 50), "p99": pct(tbt, 99), "max": pct(tbt, 100)},
                "ttft_proxy_us": {"p50": pct(ttft, 50), "p99": pct(ttft, 99)}}
