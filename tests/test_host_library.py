"""CPU tests: the C-ABI library loads without a GPU, exports every declared symbol, validates batch
descriptions before touching the device, and plans a work decomposition that covers every
(column, key) pair exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2403_02310_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "sarathi.h")).read()
    declared = set(re.findall(r"\b(sarathi_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(binding.EXPORTED)
    for name in declared:
        assert getattr(binding.lib, name) is not None


def test_create_rejects_bad_shapes():
    for kw, status in [(dict(num_q_heads=6, num_kv_heads=4), binding.ESHAPE),
                       (dict(head_dim=96), binding.ESHAPE), (dict(page_size=32), binding.ESHAPE),
                       (dict(dtype=1), binding.ESHAPE), (dict(max_tokens=0), binding.EINVAL)]:
        args = dict(num_q_heads=8, num_kv_heads=2, head_dim=128, max_tokens=64, max_seqs=8, max_blocks_per_seq=8,
                    page_size=16, dtype=0)
        args.update(kw)
        with pytest.raises(binding.SarathiError) as e:
            binding.Handle(**args)
        assert e.value.status == status


def _call_attention(h, q_start, q_len, ctx_len, num_tokens=None, ws=256, ptr=1, num_pages=100, scale=0.1):
    qs, ql, cl = (np.ascontiguousarray(a, np.int32) for a in (q_start, q_len, ctx_len))
    i32p = ctypes.POINTER(ctypes.c_int32)
    n = int(ql.sum()) if num_tokens is None else num_tokens
    # non-null fake device pointers: validation must fail before anything is dereferenced or enqueued
    return binding.lib.sarathi_hybrid_attention(h._h, ptr, ptr, ptr, ptr, qs.ctypes.data_as(i32p), ql.ctypes.data_as(i32p),
                                                cl.ctypes.data_as(i32p), len(ql), n, num_pages, scale, ptr, ws, None)


def test_validation_errors_are_reported_without_a_gpu():
    h = binding.Handle(8, 2, 128, max_tokens=64, max_seqs=4, max_blocks_per_seq=4)
    assert _call_attention(h, [0], [0], [5]) == binding.EINVAL                 # q_len < 1
    assert _call_attention(h, [0], [6], [5]) == binding.EINVAL                 # q_len > ctx_len
    assert "q_len" in h.last_error()
    assert _call_attention(h, [1], [2], [5]) == binding.EINVAL                 # q_start not the prefix sum
    assert _call_attention(h, [0, 2], [2, 3], [5, 9], num_tokens=6) == binding.EINVAL   # sum q_len != num_tokens
    assert _call_attention(h, [0], [2], [65]) == binding.ECAPACITY             # more pages than max_blocks_per_seq
    assert _call_attention(h, [0], [65], [65]) == binding.ECAPACITY            # more tokens than max_tokens
    assert _call_attention(h, [0, 1, 2, 3, 4], [1] * 5, [3] * 5) == binding.ECAPACITY   # more seqs than max_seqs
    assert _call_attention(h, [0], [2], [5], num_pages=0) == binding.EINVAL
    assert _call_attention(h, [0], [2], [5], ptr=None) == binding.EINVAL       # null tensor
    assert _call_attention(h, [0], [2], [5], ws=None) == binding.EWORKSPACE
    assert _call_attention(h, [0], [2], [5], ws=264) == binding.EWORKSPACE      # not 256-byte aligned
    assert _call_attention(h, [0], [2], [5], scale=float("nan")) == binding.EINVAL
    assert _call_attention(h, [0], [2], [5], scale=-1.0) == binding.EINVAL
    assert _call_attention(h, [], [], [], num_tokens=0) == binding.OK          # empty batch: nothing to do
    with pytest.raises(binding.SarathiError):
        h.set_option("no_such_option", 1)


def _coverage_check(batch, **options):
    s = batch.shape
    h = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=max(2048, batch.num_tokens),
                       max_seqs=max(128, batch.num_seqs), max_blocks_per_seq=batch.max_blocks_per_seq)
    for k, v in options.items():
        h.set_option(k, v)
    info, items = h.plan(batch.q_start, batch.q_len, batch.ctx_len)
    assert len(items) == info.num_items
    G = s.group
    covered = {}
    part_rows = set()
    for idx, it in enumerate(items):
        assert it.kind == (1 if idx < info.num_tile_items else 0)
        assert 1 <= it.n_cols <= (128 if it.kind == 1 else 16)
        assert it.key_begin % 32 == 0 and it.key_begin < it.key_end
        seq, prefix = it.seq, int(batch.ctx_len[it.seq] - batch.q_len[it.seq])
        assert it.col_begin + it.n_cols <= int(batch.q_len[seq]) * G
        last_row = (it.col_begin + it.n_cols - 1) // G
        assert it.key_end <= prefix + last_row + 1          # never past the tile's last visible key
        key = (seq, it.col_begin, it.n_cols)
        covered.setdefault(key, []).append((it.key_begin, it.key_end, it.part_row))
        if it.part_row >= 0:
            rows = set(range(it.part_row, it.part_row + it.n_cols))
            assert not (rows & part_rows), "partial rows overlap"
            part_rows |= rows
    assert len(part_rows) == info.num_part_rows
    # tiles partition every sequence's columns; their pieces partition keys 0 .. last visible key
    for seq in range(batch.num_seqs):
        cols = sorted((c0, nc) for (s_, c0, nc) in covered if s_ == seq)
        pos = 0
        for c0, nc in cols:
            assert c0 == pos
            pos += nc
        assert pos == int(batch.q_len[seq]) * G
    for (seq, c0, nc), pieces in covered.items():
        prefix = int(batch.ctx_len[seq] - batch.q_len[seq])
        pieces.sort()
        window = int(options.get("window", 0))
        first_visible = max(0, prefix + c0 // G - window + 1) if window else 0   # first key of the tile's first row
        assert pieces[0][0] == first_visible // 32 * 32 and pieces[-1][1] == prefix + (c0 + nc - 1) // G + 1
        for a, b in zip(pieces, pieces[1:]):
            assert a[1] == b[0]
        assert all((p[2] >= 0) == (len(pieces) > 1) for p in pieces)
    return info


@pytest.mark.parametrize("make", [wl.config1_tiny, wl.config2_mistral_hybrid, wl.config4_yi_long, wl.config5_llama70b])
def test_plan_covers_every_column_and_key_once(make):
    _coverage_check(make())


def test_plan_coverage_with_forced_options():
    b = wl.random_hybrid(3, wl.AttnShape(14, 2, 128), n_chunks=3, n_decodes=9, max_chunk=200, max_ctx=3000)
    _coverage_check(b, split_keys=32, tile_split_keys=32)
    _coverage_check(b, tile_min_cols=1)
    _coverage_check(b, tile_min_cols=1 << 20, split_keys=1 << 20)


@pytest.mark.parametrize("window", [1, 33, 500, 4096])
def test_plan_coverage_under_a_sliding_window(window):
    """Pieces start at the 32-key tile that holds the first key of the tile's first row's window."""
    b = wl.random_hybrid(4, wl.AttnShape(14, 2, 128), n_chunks=3, n_decodes=9, max_chunk=200, max_ctx=3000)
    _coverage_check(b, window=window)
    _coverage_check(b, window=window, split_keys=32, tile_split_keys=64)
    _coverage_check(wl.config4_yi_long(), window=window)


def test_long_decodes_are_cut_only_where_their_block_would_be_the_tail():
    """A decode's keys go to one block of four wavefronts unless that block would outlast a good part of the time
    the batch's decodes take to stream: the 16,384-key decodes of the long-context recipe stay whole (no partial
    rows, no merge launch), the same decode next to a handful of short ones is cut, and so is a lone long decode."""
    info = _coverage_check(wl.config4_yi_long())
    assert info.num_reduce_items == 0 and info.num_part_rows == 0
    s = wl.AttnShape(56, 8, 128)
    few = wl._make("few", s, [1] * 6, [16384, 300, 900, 50, 1200, 700], 10)
    info = _coverage_check(few)
    assert info.num_reduce_items == 1 and info.num_part_rows > 0          # only the long one, in several pieces
    lone = wl._make("lone", s, [1], [100000], 11)
    info = _coverage_check(lone)
    assert info.num_reduce_items == 1 and info.num_items >= 8


def test_plan_stays_within_the_workspace_when_everything_is_long():
    s = wl.AttnShape(64, 8, 128)
    b = wl._make("long", s, [2048], [16384], 9)
    info = _coverage_check(b, tile_split_keys=32, split_keys=32)
    assert info.num_part_rows <= 32768


def test_linear_refuses_bad_shapes_without_a_gpu():
    """Shape checks come before any device call, so they can be exercised here."""
    for (T, N, K) in [(-1, 128, 64), (4, 0, 64), (4, 100, 64), (4, 128, 32), (4, 128, 96), (4, 128, (1 << 20) + 64)]:
        assert binding.lib.sarathi_linear(None, None, None, T, N, K, None, 0, None) == binding.ESHAPE
        assert binding.linear_workspace_bytes(T, N, K) == 0
    assert binding.lib.sarathi_linear(None, None, None, 0, 128, 64, None, 0, None) == 0          # no tokens: nothing to do
    assert binding.lib.sarathi_linear(None, None, None, 4, 128, 64, None, 0, None) == binding.EINVAL


def test_linear_split_k_workspace_sizes():
    """A small batch on big weights asks for partial tiles; a batch that fills the chip by itself asks for none."""
    assert binding.linear_workspace_bytes(2048, 8192, 4096) == 0
    small = binding.linear_workspace_bytes(128, 4096, 14336)
    assert small > 0 and small % (128 * 4096 * 4) == 0 and small // (128 * 4096 * 4) <= 16
