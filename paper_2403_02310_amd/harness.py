"""Device-side plumbing shared by the GPU tests, ``bench.py`` and the smoke run.

Everything here moves bytes between numpy and device memory or calls the C ABI through
``binding``; no step of the attention path is computed here and nothing here imports the
CPU checker.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding
from .workloads import HybridBatch

POISON_NAN = 0x7FC1    # a quiet NaN
POISON_PINF = 0x7F80   # +inf
POISON_NINF = 0xFF80   # -inf


def bits_to_device(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 device tensor holding exactly those bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def device_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def make_handle(batch: HybridBatch, max_tokens: Optional[int] = None, max_seqs: Optional[int] = None) -> binding.Handle:
    s = batch.shape
    return binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim,
                          max_tokens=max(max_tokens or 0, batch.num_tokens, 4096),
                          max_seqs=max(max_seqs or 0, batch.num_seqs, 64),
                          max_blocks_per_seq=batch.max_blocks_per_seq, page_size=s.page_size)


def make_pools(batch: HybridBatch, poison: Optional[int] = POISON_NAN, device="cuda", num_pages: Optional[int] = None):
    """K pool [pages, Hkv, page, d] and V pool [pages, Hkv, d, page]; optionally filled with a poison pattern."""
    s = batch.shape
    pages = num_pages or batch.num_pages
    if poison is None:
        k = torch.empty((pages, s.num_kv_heads, s.page_size, s.head_dim), dtype=torch.bfloat16, device=device)
        v = torch.empty((pages, s.num_kv_heads, s.head_dim, s.page_size), dtype=torch.bfloat16, device=device)
    else:
        val = int(np.array([poison], dtype=np.uint16).view(np.int16)[0])
        k = torch.full((pages, s.num_kv_heads, s.page_size, s.head_dim), val, dtype=torch.int16, device=device).view(torch.bfloat16)
        v = torch.full((pages, s.num_kv_heads, s.head_dim, s.page_size), val, dtype=torch.int16, device=device).view(torch.bfloat16)
    return k, v


def append_ranges(handle: binding.Handle, batch: HybridBatch, k_cache, v_cache, bt_dev: torch.Tensor,
                  ranges: Sequence[Tuple[int, int, int]], kv_host: Optional[dict] = None) -> None:
    """Appends positions [start, end) of the listed sequences through sarathi_kv_append.

    ``ranges`` = (sequence, start, end); long ranges are cut to the handle's max_tokens and
    several sequences share a call.  ``kv_host`` optionally caches ``batch.kv_bits``.
    """
    cap_t, cap_s = handle.config.max_tokens, handle.config.max_seqs
    pieces: List[Tuple[int, int, int]] = []
    for (s, a, b) in ranges:
        while a < b:
            e = min(b, a + cap_t)
            pieces.append((s, a, e))
            a = e
    i = 0
    while i < len(pieces):
        group, used, seen = [], 0, set()
        while i < len(pieces) and len(group) < cap_s:
            s, a, e = pieces[i]
            if used + (e - a) > cap_t or s in seen:
                break
            group.append(pieces[i]); used += e - a; seen.add(s); i += 1
        ks, vs = [], []
        for (s, a, e) in group:
            if kv_host is not None and s in kv_host:
                k, v = kv_host[s]
            else:
                k, v = batch.kv_bits(s)
                if kv_host is not None:
                    kv_host[s] = (k, v)
            ks.append(k[a:e]); vs.append(v[a:e])
        k_new = bits_to_device(np.concatenate(ks)); v_new = bits_to_device(np.concatenate(vs))
        q_len = np.array([e - a for (_, a, e) in group], np.int32)
        ctx = np.array([e for (_, _, e) in group], np.int32)
        q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int32)
        rows = torch.as_tensor([s for (s, _, _) in group], device=bt_dev.device, dtype=torch.long)
        bt = bt_dev.index_select(0, rows).contiguous()
        handle.kv_append(k_new, v_new, k_cache, v_cache, bt, q_start, q_len, ctx)
        torch.cuda.synchronize()


def fill_prefixes(handle, batch, k_cache, v_cache, bt_dev, kv_host: Optional[dict] = None, upto: str = "prefix"):
    """Brings the cache to the state before this iteration (``prefix``) or after it (``all``)."""
    ranges = []
    for s in range(batch.num_seqs):
        end = int(batch.prefix_len[s]) if upto == "prefix" else int(batch.ctx_len[s])
        if end > 0:
            ranges.append((s, 0, end))
    append_ranges(handle, batch, k_cache, v_cache, bt_dev, ranges, kv_host)


def new_token_kv(batch: HybridBatch, kv_host: Optional[dict] = None):
    """This iteration's K/V rows in batch order, ``[T, Hkv, d]`` bf16 bits each."""
    ks, vs = [], []
    for s in range(batch.num_seqs):
        if kv_host is not None and s in kv_host:
            k, v = kv_host[s]
        else:
            k, v = batch.kv_bits(s)
            if kv_host is not None:
                kv_host[s] = (k, v)
        p = int(batch.prefix_len[s])
        ks.append(k[p:]); vs.append(v[p:])
    return np.concatenate(ks), np.concatenate(vs)


def run_iteration(handle, batch: HybridBatch, k_cache, v_cache, bt_dev, q_dev, k_new_dev, v_new_dev, out_dev=None):
    """One iteration of the hot path: append the new K/V rows, then attention over the batch."""
    if out_dev is None:
        out_dev = torch.empty_like(q_dev)
    handle.kv_append(k_new_dev, v_new_dev, k_cache, v_cache, bt_dev, batch.q_start, batch.q_len, batch.ctx_len)
    handle.hybrid_attention(q_dev, k_cache, v_cache, bt_dev, batch.q_start, batch.q_len, batch.ctx_len,
                            batch.sm_scale, out_dev)
    return out_dev


def setup_and_run(batch: HybridBatch, poison: Optional[int] = POISON_NAN, handle=None, q_copy: int = 0,
                  kv_host: Optional[dict] = None, q_bits: Optional[np.ndarray] = None):
    """Full flow on fresh pools: poison, fill prefixes, run the iteration.  Returns a dict of device state.

    ``kv_host`` ({sequence: (k_bits, v_bits)}) and ``q_bits`` replace the batch's own seeded draws
    (tests with hand-made values)."""
    handle = handle or make_handle(batch)
    k_cache, v_cache = make_pools(batch, poison)
    bt_dev = torch.from_numpy(batch.block_table).cuda()
    kv_host = {} if kv_host is None else kv_host
    fill_prefixes(handle, batch, k_cache, v_cache, bt_dev, kv_host)
    k_new, v_new = new_token_kv(batch, kv_host)
    q_dev = bits_to_device(batch.q_bits(q_copy) if q_bits is None else q_bits)
    out = run_iteration(handle, batch, k_cache, v_cache, bt_dev, q_dev, bits_to_device(k_new), bits_to_device(v_new))
    torch.cuda.synchronize()
    return {"handle": handle, "k_cache": k_cache, "v_cache": v_cache, "bt": bt_dev, "q": q_dev, "out": out,
            "kv_host": kv_host}
