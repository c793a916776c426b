"""TEST INFRASTRUCTURE ONLY -- what the paged K/V pools must hold, written as plain loops.

The paper keeps the keys and values of every processed token in a KV cache so that later
iterations can read them (section 2.2), organised in fixed-size pages addressed through
per-sequence block tables (paged cache, section 2.2 / 4.4).  The paper fixes neither page
size nor in-page layout; the library's header fixes them and this file restates them so a
byte-for-byte comparison is possible:

* token at absolute position ``p`` of sequence ``s`` lives in page ``block_table[s][p // page]``,
  slot ``p % page``;
* ``k_cache[page, kv_head, slot, c]``  -- slot-major rows of ``d`` channels;
* ``v_cache[page, kv_head, c, slot]``  -- channel-major (each page stores V transposed).

Everything here is integer indexing and byte copies: the comparison bar is bit-exact.
"""
from __future__ import annotations

import numpy as np


def empty_pools(num_pages: int, num_kv_heads: int, head_dim: int, page_size: int, fill: int = 0):
    k = np.full((num_pages, num_kv_heads, page_size, head_dim), fill, dtype=np.uint16)
    v = np.full((num_pages, num_kv_heads, head_dim, page_size), fill, dtype=np.uint16)
    return k, v


def kv_append(k_cache: np.ndarray, v_cache: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
              block_table: np.ndarray, q_start, q_len, ctx_len) -> None:
    """Write this iteration's K/V rows (``[T, Hkv, d]`` bf16 bits, batch order) into the pools, in place."""
    page_size = k_cache.shape[2]
    for s in range(len(q_len)):
        prefix = int(ctx_len[s]) - int(q_len[s])
        for j in range(int(q_len[s])):
            pos = prefix + j
            page = int(block_table[s, pos // page_size])
            slot = pos % page_size
            t = int(q_start[s]) + j
            k_cache[page, :, slot, :] = k_new[t]
            v_cache[page, :, :, slot] = v_new[t]


def gather_sequence(k_cache: np.ndarray, v_cache: np.ndarray, block_table_row: np.ndarray, ctx_len: int):
    """Read positions 0..ctx_len-1 of one sequence back as contiguous ``[ctx_len, Hkv, d]`` K and V."""
    page_size = k_cache.shape[2]
    n_kv, d = k_cache.shape[1], k_cache.shape[3]
    k = np.empty((ctx_len, n_kv, d), dtype=k_cache.dtype)
    v = np.empty((ctx_len, n_kv, d), dtype=v_cache.dtype)
    for pos in range(ctx_len):
        page = int(block_table_row[pos // page_size])
        slot = pos % page_size
        k[pos] = k_cache[page, :, slot, :]
        v[pos] = v_cache[page, :, :, slot]
    return k, v
