"""CPU tests: the paged-cache reference (append + gather through the block table)."""
import numpy as np

from oracle import kv_cache_reference as kvref
from paper_2403_02310_amd import workloads as wl


def test_append_then_gather_returns_contiguous_originals_and_touches_nothing_else():
    b = wl.random_hybrid(7, wl.AttnShape(4, 2, 16), n_chunks=2, n_decodes=3, max_chunk=40, max_ctx=90)
    s = b.shape
    POISON = 0xFFFF
    kc, vc = kvref.empty_pools(b.num_pages, s.num_kv_heads, s.head_dim, s.page_size, fill=POISON)
    # whole contexts appended as one "prefill from zero"
    parts = [b.kv_bits(i) for i in range(b.num_seqs)]
    k_new = np.concatenate([p[0] for p in parts]); v_new = np.concatenate([p[1] for p in parts])
    q_start = np.concatenate([[0], np.cumsum(b.ctx_len)[:-1]])
    kvref.kv_append(kc, vc, k_new, v_new, b.block_table, q_start, b.ctx_len, b.ctx_len)
    used = set()
    for i in range(b.num_seqs):
        kg, vg = kvref.gather_sequence(kc, vc, b.block_table[i], int(b.ctx_len[i]))
        np.testing.assert_array_equal(kg, parts[i][0])
        np.testing.assert_array_equal(vg, parts[i][1])
        used.update(int(x) for x in b.block_table[i] if x >= 0)
        # slots past ctx_len in the last page stay untouched
        tail = int(b.ctx_len[i]) % s.page_size
        if tail:
            last = int(b.block_table[i, (int(b.ctx_len[i]) - 1) // s.page_size])
            assert (kc[last, :, tail:, :] == POISON).all()
            assert (vc[last, :, :, tail:] == POISON).all()
    for page in range(b.num_pages):
        if page not in used:
            assert (kc[page] == POISON).all() and (vc[page] == POISON).all()


def test_layout_is_the_documented_flat_offset():
    """k: ((page*Hkv + h)*P + slot)*d + c ;  v: ((page*Hkv + h)*d + c)*P + slot  (elements)."""
    Hkv, d, P, pages = 2, 8, 16, 3
    kc, vc = kvref.empty_pools(pages, Hkv, d, P)
    bt = np.array([[2, 0, -1]], dtype=np.int32)
    k_new = np.arange(20 * Hkv * d, dtype=np.uint16).reshape(20, Hkv, d)
    v_new = (k_new + 1000).astype(np.uint16)
    kvref.kv_append(kc, vc, k_new, v_new, bt, [0], [20], [20])
    kflat, vflat = kc.reshape(-1), vc.reshape(-1)
    for pos in (0, 5, 15, 16, 19):
        page = [2, 0][pos // P]; slot = pos % P
        for h in range(Hkv):
            for c in (0, 3, 7):
                assert kflat[((page * Hkv + h) * P + slot) * d + c] == k_new[pos, h, c]
                assert vflat[((page * Hkv + h) * d + c) * P + slot] == v_new[pos, h, c]


def test_decode_append_writes_exactly_one_slot():
    Hkv, d, P = 1, 4, 16
    kc, vc = kvref.empty_pools(4, Hkv, d, P)
    bt = np.array([[3, 1]], dtype=np.int32)
    k_new = np.full((1, Hkv, d), 7, np.uint16); v_new = np.full((1, Hkv, d), 9, np.uint16)
    kvref.kv_append(kc, vc, k_new, v_new, bt, [0], [1], [18])   # position 17 -> page 1, slot 1
    assert (kc[1, 0, 1] == 7).all() and kc.sum() == 7 * d
    assert (vc[1, 0, :, 1] == 9).all() and vc.sum() == 9 * d
