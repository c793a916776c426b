"""Seeded synthetic hybrid batches (inputs only; none of the method's arithmetic lives here).

A hybrid batch is what one scheduling iteration hands to the attention path
(paper section 4.2, Algorithm 3): some sequences contribute a prefill chunk of
``q_len > 1`` new tokens on top of an already cached prefix, the others contribute a
single decode token.  Every tensor is drawn from N(0, 1) with a counter-free seeded
numpy generator and rounded once to bf16 (round-to-nearest-even); the values are handed
around as raw ``uint16`` bit patterns so that both the fp64 checker and the GPU library
see exactly the same inputs.

Shapes follow the serving workloads of the paper's evaluation (section 5: prompts of
thousands of tokens, token budgets 512 / 2048, tens to hundreds of running decodes) at
the attention shapes of the models in its Table 1.  The datasets themselves are not
used: lengths are drawn from the simple distributions stated per recipe below.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

PAGE_SIZE = 16


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64 (used by tests to inspect inputs)."""
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def normal_bf16(seed_words: Sequence[int], shape: Tuple[int, ...]) -> np.ndarray:
    """N(0,1) samples of ``shape`` as bf16 bit patterns, fully determined by ``seed_words``."""
    rng = np.random.default_rng(list(seed_words))
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 22
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        out[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))
    return out.reshape(shape)


@dataclass
class AttnShape:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int = PAGE_SIZE

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


MISTRAL_7B = AttnShape(32, 8, 128)
YI_34B = AttnShape(56, 8, 128)
LLAMA2_70B = AttnShape(64, 8, 128)
TINY = AttnShape(4, 1, 64)


@dataclass
class HybridBatch:
    """Lengths, block tables and seeds of one iteration's batch; tensors are made on demand."""

    name: str
    shape: AttnShape
    q_len: np.ndarray            # int32 [S] new tokens this iteration
    ctx_len: np.ndarray          # int32 [S] KV length after this iteration's append
    block_table: np.ndarray      # int32 [S, max_blocks]; unused entries are -1
    num_pages: int               # pages in the pool
    seed: int
    sm_scale: float = field(default=0.0)
    kv_ids: Optional[np.ndarray] = None   # per-sequence seed word for K/V (default: the sequence index)

    def __post_init__(self):
        self.q_len = np.asarray(self.q_len, dtype=np.int32)
        self.ctx_len = np.asarray(self.ctx_len, dtype=np.int32)
        if self.kv_ids is None:
            self.kv_ids = np.arange(self.q_len.shape[0], dtype=np.int64)
        if self.sm_scale == 0.0:
            self.sm_scale = 1.0 / float(np.sqrt(self.shape.head_dim))

    # ---- derived lengths -------------------------------------------------
    @property
    def num_seqs(self) -> int:
        return int(self.q_len.shape[0])

    @property
    def num_tokens(self) -> int:
        return int(self.q_len.sum())

    @property
    def q_start(self) -> np.ndarray:
        out = np.zeros(self.num_seqs, dtype=np.int32)
        np.cumsum(self.q_len[:-1], out=out[1:])
        return out

    @property
    def prefix_len(self) -> np.ndarray:
        return (self.ctx_len - self.q_len).astype(np.int32)

    @property
    def kv_start(self) -> np.ndarray:
        out = np.zeros(self.num_seqs, dtype=np.int64)
        np.cumsum(self.ctx_len[:-1].astype(np.int64), out=out[1:])
        return out

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_table.shape[1])

    # ---- tensors ---------------------------------------------------------
    def q_bits(self, copy: int = 0) -> np.ndarray:
        """Query rows ``[T, Hq, d]``; ``copy`` selects an independent draw (timing rotation)."""
        s = self.shape
        return normal_bf16((self.seed, 0x51, copy), (self.num_tokens, s.num_q_heads, s.head_dim))

    def kv_bits(self, seq: int) -> Tuple[np.ndarray, np.ndarray]:
        """All keys and values of one sequence, ``[ctx_len, Hkv, d]`` each, positions 0..ctx_len-1."""
        s = self.shape
        n = int(self.ctx_len[seq])
        sid = int(self.kv_ids[seq])
        k = normal_bf16((self.seed, 0x4B, sid), (n, s.num_kv_heads, s.head_dim))
        v = normal_bf16((self.seed, 0x56, sid), (n, s.num_kv_heads, s.head_dim))
        return k, v

    def kv_bits_many(self, seqs: Sequence[int], workers: int = 8):
        with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
            return list(ex.map(self.kv_bits, seqs))

    def kv_concat(self, workers: int = 8) -> Tuple[np.ndarray, np.ndarray]:
        """Contiguous ``[sum(ctx_len), Hkv, d]`` K and V with sequence ``s`` at ``kv_start[s]``."""
        parts = self.kv_bits_many(range(self.num_seqs), workers)
        k = np.concatenate([p[0] for p in parts], axis=0)
        v = np.concatenate([p[1] for p in parts], axis=0)
        return k, v

    # ---- algorithmic work (paper section 3.1 roofline terms) --------------
    def kv_bytes(self) -> int:
        s = self.shape
        return int(self.ctx_len.astype(np.int64).sum()) * 2 * s.num_kv_heads * s.head_dim * 2

    def qo_bytes(self) -> int:
        s = self.shape
        return self.num_tokens * s.num_q_heads * s.head_dim * 2 * 2

    def block_table_bytes(self) -> int:
        return int(((self.ctx_len.astype(np.int64) + self.shape.page_size - 1) // self.shape.page_size).sum()) * 4

    def algorithmic_bytes(self) -> int:
        return self.kv_bytes() + self.qo_bytes() + self.block_table_bytes()

    def score_pairs(self) -> int:
        q = self.q_len.astype(np.int64)
        p = self.prefix_len.astype(np.int64)
        return int((q * p + q * (q + 1) // 2).sum())

    def algorithmic_flops(self) -> int:
        s = self.shape
        return 4 * s.head_dim * s.num_q_heads * self.score_pairs()

    def sub_batch(self, seqs: Sequence[int], name: Optional[str] = None) -> "HybridBatch":
        """The same sequences restricted to ``seqs`` (e.g. chunks only, decodes only).

        Keys, values and block tables are those of the parent (so a cache pool filled for the
        parent serves the sub-batch); the query rows are an independent draw.
        """
        idx = np.asarray(list(seqs), dtype=np.int64)
        return HybridBatch(name or (self.name + "/sub"), self.shape, self.q_len[idx], self.ctx_len[idx],
                           self.block_table[idx], self.num_pages, self.seed, self.sm_scale,
                           kv_ids=self.kv_ids[idx])


def reorder(batch: HybridBatch, order: Sequence[int], name: Optional[str] = None) -> HybridBatch:
    """The same batch with its sequences listed in another order (K/V contents follow their sequence)."""
    idx = np.asarray(list(order), dtype=np.int64)
    assert sorted(idx.tolist()) == list(range(batch.num_seqs))
    return HybridBatch(name or batch.name, batch.shape, batch.q_len[idx], batch.ctx_len[idx],
                       batch.block_table[idx], batch.num_pages, batch.seed, batch.sm_scale,
                       kv_ids=batch.kv_ids[idx])


def decodes_first(batch: HybridBatch) -> HybridBatch:
    """Algorithm 3's order: every decode, then the prefill chunks (each group in its original order)."""
    dec = [i for i in range(batch.num_seqs) if batch.q_len[i] == 1]
    pre = [i for i in range(batch.num_seqs) if batch.q_len[i] != 1]
    return reorder(batch, dec + pre)


def pages_needed(ctx_len: np.ndarray, page_size: int = PAGE_SIZE) -> np.ndarray:
    return (np.asarray(ctx_len, dtype=np.int64) + page_size - 1) // page_size


def scatter_block_tables(ctx_len: np.ndarray, num_pages: int, seed: int,
                         page_size: int = PAGE_SIZE, max_blocks: Optional[int] = None) -> np.ndarray:
    """Block tables = consecutive slices of one random draw (without replacement) from the pool."""
    need = pages_needed(ctx_len, page_size)
    total = int(need.sum())
    if total > num_pages:
        raise ValueError("pool too small: need %d pages, have %d" % (total, num_pages))
    rng = np.random.default_rng([seed, 0xB7])
    if num_pages <= 4 * total:
        chosen = rng.permutation(num_pages)[:total]
    else:
        # sparse use of a huge pool: draw, drop duplicates, top up
        chosen = np.unique(rng.integers(0, num_pages, size=int(total * 1.1) + 16))
        while chosen.shape[0] < total:
            extra = rng.integers(0, num_pages, size=total)
            chosen = np.unique(np.concatenate([chosen, extra]))
        chosen = rng.permutation(chosen)[:total]
    width = int(max_blocks if max_blocks is not None else max(1, int(need.max())))
    bt = np.full((len(need), width), -1, dtype=np.int32)
    off = 0
    for s, n in enumerate(need):
        bt[s, : int(n)] = chosen[off: off + int(n)]
        off += int(n)
    return bt


def _make(name, shape, q_len, ctx_len, seed, pool_pages=None, slack=2.0, max_blocks=None, sm_scale=0.0):
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    need = int(pages_needed(ctx_len, shape.page_size).sum())
    num_pages = int(pool_pages if pool_pages is not None else max(need, int(np.ceil(need * slack))))
    bt = scatter_block_tables(ctx_len, num_pages, seed, shape.page_size, max_blocks)
    return HybridBatch(name, shape, np.asarray(q_len, dtype=np.int32), ctx_len, bt, num_pages, seed, sm_scale)


# ---------------------------------------------------------------------------
# The five workload recipes.
# ---------------------------------------------------------------------------

def config1_tiny(seed: int = 1) -> HybridBatch:
    """One 64-token chunk on a 128-token cached prefix plus decodes at context 100/200/300."""
    return _make("c1_tiny", TINY, [64, 1, 1, 1], [192, 100, 200, 300], seed, pool_pages=64)


def config1_prompt(chunk: int, seed: int = 1, prompt_len: int = 192) -> List[HybridBatch]:
    """The same ``prompt_len``-token prompt prefilled in chunks of ``chunk`` tokens: one batch per iteration.

    All iterations share one block table and one seed, so ``kv_bits(0)`` of the last
    iteration holds the whole prompt and earlier iterations see its leading rows.
    """
    full = _make("c1_prompt", TINY, [prompt_len], [prompt_len], seed, pool_pages=32)
    out = []
    done = 0
    while done < prompt_len:
        c = min(chunk, prompt_len - done)
        out.append(HybridBatch("c1_prompt_%d@%d" % (c, done), TINY, [c], [done + c],
                               full.block_table, full.num_pages, seed))
        done += c
    return out


def config2_mistral_hybrid(seed: int = 2, chunk: int = 512, n_decodes: int = 64) -> HybridBatch:
    """Mistral-7B shape: one 512-token chunk at a prefix uniform in [0, 3584] + 64 decodes, ctx uniform in [256, 4096]."""
    rng = np.random.default_rng([seed, 0xC2])
    prefix = int(rng.integers(0, 3584 + 1))
    dec = rng.integers(256, 4096 + 1, size=n_decodes)
    q_len = [chunk] + [1] * n_decodes
    ctx = [prefix + chunk] + [int(x) for x in dec]
    return _make("c2_mistral_hybrid", MISTRAL_7B, q_len, ctx, seed)


def config3_decode_only(seed: int = 3, n_decodes: int = 256, pool_bytes_per_cache: float = 100e9) -> HybridBatch:
    """256 decodes, ctx lognormal (median 1024, sigma 0.8) clipped to [64, 8192], pages scattered over a huge pool."""
    rng = np.random.default_rng([seed, 0xC3])
    z = rng.standard_normal(n_decodes)
    ctx = np.clip(np.rint(np.exp(np.log(1024.0) + 0.8 * z)), 64, 8192).astype(np.int32)
    s = MISTRAL_7B
    page_bytes = s.num_kv_heads * s.page_size * s.head_dim * 2
    pool_pages = int(pool_bytes_per_cache // page_bytes)
    need = int(pages_needed(ctx).sum())
    pool_pages = max(pool_pages, need)
    return _make("c3_decode_only", s, [1] * n_decodes, ctx, seed, pool_pages=pool_pages)


def config4_yi_long(seed: int = 4) -> HybridBatch:
    """Yi-34B shape: chunks of 1024/512/384 at prefixes uniform in [0, 12288] + 128 decodes, ctx uniform in [1024, 16384]."""
    rng = np.random.default_rng([seed, 0xC4])
    chunks = [1024, 512, 384]
    prefixes = rng.integers(0, 12288 + 1, size=3)
    dec = rng.integers(1024, 16384 + 1, size=128)
    q_len = chunks + [1] * 128
    ctx = [int(p) + c for p, c in zip(prefixes, chunks)] + [int(x) for x in dec]
    return _make("c4_yi_long", YI_34B, q_len, ctx, seed)


def config5_llama70b(seed: int = 5, n_decodes: int = 1024) -> HybridBatch:
    """LLaMA2-70B shape: two 512-token chunks (prefix uniform in [0, 3584]) + 1024 decodes, ctx uniform in [512, 4096]."""
    rng = np.random.default_rng([seed, 0xC5])
    prefixes = rng.integers(0, 3584 + 1, size=2)
    dec = rng.integers(512, 4096 + 1, size=n_decodes)
    q_len = [512, 512] + [1] * n_decodes
    ctx = [int(p) + 512 for p in prefixes] + [int(x) for x in dec]
    return _make("c5_llama70b", LLAMA2_70B, q_len, ctx, seed)


def config5_sweep(chunk: int, seed: int = 55, prompt_len: int = 8192, shape: AttnShape = LLAMA2_70B) -> List[HybridBatch]:
    """One ``prompt_len``-token prompt prefilled in chunks of ``chunk``: one single-sequence batch per iteration."""
    full = _make("c5_sweep", shape, [prompt_len], [prompt_len], seed, slack=1.25)
    out = []
    done = 0
    while done < prompt_len:
        c = min(chunk, prompt_len - done)
        out.append(HybridBatch("c5_sweep_%d@%d" % (c, done), shape, [c], [done + c],
                               full.block_table, full.num_pages, seed))
        done += c
    return out


def random_hybrid(seed: int, shape: AttnShape, n_chunks: int, n_decodes: int,
                  max_chunk: int = 96, max_ctx: int = 400, slack: float = 1.5) -> HybridBatch:
    """Small ragged batches for element-by-element parity: odd lengths, mid-page prefixes, shuffled order."""
    rng = np.random.default_rng([seed, 0xAB])
    q_len, ctx = [], []
    for _ in range(n_chunks):
        c = int(rng.integers(2, max_chunk + 1))
        p = int(rng.integers(0, max(1, max_ctx - c) + 1))
        q_len.append(c)
        ctx.append(p + c)
    for _ in range(n_decodes):
        q_len.append(1)
        ctx.append(int(rng.integers(1, max_ctx + 1)))
    order = rng.permutation(len(q_len))
    q_len = [q_len[i] for i in order]
    ctx = [ctx[i] for i in order]
    return _make("random_%d" % seed, shape, q_len, ctx, seed, slack=slack)
