"""Token-budget profiling (section 4.3, "Determining Token Budget").

The budget is found by a one-time profile: time batches with different numbers of tokens and take
the largest count whose iteration stays within the latency target.  Here an "iteration" is KV append
+ hybrid-batch attention, optionally plus the four linear layers of one transformer layer of a named
model (``gpu_timer(linear_model=...)``); there is no whole model around it, so the times are a PROXY for
the paper's time-between-tokens target and the budgets only mean something relative to each other.

A profiled batch for budget tau = the given running decodes (one token each) plus the prefill chunk that
``sarathi_build_stall_free_batch`` gives a request in mid-prefill under that budget (tau - #decodes tokens on
top of its cached prefix; none when the decodes use the budget up): the fullest batch stall-free batching
builds under that budget (Algorithm 3, section 4.2).

The section's second consideration, tile quantisation (a chunk one token past a tile edge costs a
whole further tile), is measured by ``tile_quantization_probe``: chunk sizes around the kernels'
128-column query tile.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from .workloads import AttnShape, HybridBatch, _make


def budget_batch(shape: AttnShape, token_budget: int, decode_ctx: Sequence[int], chunk_prefix: int, seed: int = 0) -> HybridBatch:
    """The fullest batch stall-free batching builds under ``token_budget``: the running decodes (contexts
    ``decode_ctx``, the new token included) and a request in mid-prefill with ``chunk_prefix`` tokens done and more
    than a budget's worth to go.  The batch comes from ``sarathi_build_stall_free_batch`` (Algorithm 3): the chunk is
    what the decodes leave of the budget, and none at all when they leave nothing."""
    from . import binding
    n_dec = len(decode_ctx)
    decodes = [(i, int(c) - 1, int(c) - 1, 0) for i, c in enumerate(decode_ctx)]       # ctx = prompt + 0 decoded + the new token
    prefill = [(n_dec, chunk_prefix + 2 * token_budget + 1, chunk_prefix, 0)]
    b = binding.build_stall_free_batch(token_budget, token_budget, decodes, prefill, [], free_pages=0,
                                       page_size=shape.page_size, max_batch_size=n_dec + 1)
    assert b["num_decodes"] == n_dec and b["num_tokens"] <= max(token_budget, n_dec)
    return _make("budget_%d" % token_budget, shape, b["q_len"], b["ctx_len"], seed, slack=1.0)


def profile(time_batch: Callable[[HybridBatch], float], shape: AttnShape, budgets: Sequence[int], decode_ctx: Sequence[int],
            chunk_prefix: int, seed: int = 0) -> List[Dict[str, float]]:
    """``time_batch(batch) -> seconds`` per candidate budget; returns rows sorted by budget."""
    rows = []
    for tau in sorted(set(int(b) for b in budgets)):
        b = budget_batch(shape, tau, decode_ctx, chunk_prefix, seed)
        rows.append({"token_budget": tau, "tokens": int(b.num_tokens), "seconds": float(time_batch(b))})
    return rows


def compute_token_budget(rows: Sequence[Dict[str, float]], target_seconds: float) -> Optional[int]:
    """Largest profiled budget whose iteration time, and that of every smaller profiled budget, meets the target
    (None if even the smallest does not).  Requiring the smaller ones too makes the answer robust against a noisy
    dip in the profile."""
    best = None
    for r in sorted(rows, key=lambda r: r["token_budget"]):
        if r["seconds"] > target_seconds:
            break
        best = int(r["token_budget"])
    return best


def gpu_timer(options: Optional[Dict[str, int]] = None, reps: int = 20, warmup: int = 3,
              linear_model: Optional[str] = None, on_batch: Optional[Callable] = None) -> Callable[[HybridBatch], float]:
    """Times append + attention of a batch on the GPU (median of ``reps``), values drawn on the device.
    ``linear_model`` (a key of ``linear_layers.MODELS``): the four linear layers of one transformer layer of that
    model run over the batch's tokens inside the timed region too.  ``on_batch(batch, tensors)`` is called after
    a batch has been timed with its device tensors (q, k_cache, v_cache, block_table, out), e.g. by a test that
    checks what the profiled launches computed."""
    import torch
    from . import binding
    linear = []   # (weight, scratch bytes wanted) per layer, drawn once

    def linear_operands(T: int):
        from . import linear_layers as ll
        if not linear:
            g = torch.Generator(device="cuda").manual_seed(12345)
            for _, n, k in ll.layer_shapes(ll.MODELS[linear_model]):
                linear.append(torch.randn(n, k, device="cuda", generator=g).to(torch.bfloat16))
        ops = []
        for w in linear:
            n, k = w.shape
            ops.append((torch.ones(T, k, device="cuda", dtype=torch.bfloat16), w,
                        torch.empty(T, n, device="cuda", dtype=torch.bfloat16),
                        torch.empty(max(16, binding.linear_workspace_bytes(T, n, k)), dtype=torch.uint8, device="cuda")))
        return ops

    def time_batch(b: HybridBatch) -> float:
        s = b.shape
        h = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=max(2048, b.num_tokens),
                           max_seqs=max(128, b.num_seqs), max_blocks_per_seq=b.max_blocks_per_seq)
        for k, v in (options or {}).items():
            h.set_option(k, v)
        g = torch.Generator(device="cuda").manual_seed(b.seed)
        rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=g).to(torch.bfloat16)
        kc = rnd(b.num_pages, s.num_kv_heads, s.page_size, s.head_dim)
        vc = rnd(b.num_pages, s.num_kv_heads, s.head_dim, s.page_size)
        q, kn, vn = rnd(b.num_tokens, s.num_q_heads, s.head_dim), rnd(b.num_tokens, s.num_kv_heads, s.head_dim), rnd(b.num_tokens, s.num_kv_heads, s.head_dim)
        out = torch.empty_like(q)
        bt = torch.from_numpy(b.block_table).cuda()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        lin_ops = linear_operands(b.num_tokens) if linear_model else []
        times = []
        for i in range(warmup + reps):
            ev[0].record()
            h.kv_append(kn, vn, kc, vc, bt, b.q_start, b.q_len, b.ctx_len)
            h.hybrid_attention(q, kc, vc, bt, b.q_start, b.q_len, b.ctx_len, b.sm_scale, out)
            for x, w, y, scratch in lin_ops:
                binding.linear(x, w, y, scratch)
            ev[1].record()
            ev[1].synchronize()
            if i >= warmup:
                times.append(ev[0].elapsed_time(ev[1]) * 1e-3)
        if on_batch is not None:
            on_batch(b, {"q": q, "k_cache": kc, "v_cache": vc, "block_table": bt, "out": out})
        return float(np.median(times))
    return time_batch


def tile_quantization_probe(time_batch: Callable[[HybridBatch], float], shape: AttnShape, prefix: int = 2048,
                            chunks: Sequence[int] = (255, 256, 257, 288), seed: int = 0) -> List[Dict[str, float]]:
    """Chunk-only batches around a multiple of the 128-column query tile (128 / G rows)."""
    rows = []
    for c in chunks:
        b = _make("quant_%d" % c, shape, [c], [prefix + c], seed, slack=1.0)
        rows.append({"chunk": int(c), "seconds": float(time_batch(b))})
    return rows
