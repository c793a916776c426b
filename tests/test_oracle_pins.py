"""CPU tests: the fp64 checker against facts that do not come from itself."""
import numpy as np
import pytest

import oracle
from oracle import kv_cache_reference as kvref
from paper_2403_02310_amd import workloads as wl
from tests import pin_checks


@pytest.mark.parametrize("check", pin_checks.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(check):
    check(oracle.hybrid_attention)


@pytest.mark.parametrize("check", pin_checks.WINDOW_CHECKS, ids=lambda f: f.__name__)
def test_window_pin(check):
    check(oracle.hybrid_attention)


def test_softmax_weights_sum_to_one_and_lie_in_unit_interval():
    b = wl.config1_tiny()
    q = b.q_bits(); k, v = b.kv_concat()
    for t in (0, 31, 63, 64, 65, 66):
        for h in range(4):
            w = oracle.softmax_weights(q, k, b.kv_start, b.q_start, b.q_len, b.ctx_len, b.sm_scale, t, h)
            s = int(np.searchsorted(b.q_start, t, side="right") - 1)
            pos = int(b.ctx_len[s] - b.q_len[s] + (t - b.q_start[s]))
            assert w.shape[0] == pos + 1            # keys 0..pos, the token itself included
            assert abs(w.sum() - 1.0) < 1e-12
            assert (w > 0).all() and (w <= 1).all()


def test_weights_times_v_is_the_output():
    b = wl.config1_tiny()
    q = b.q_bits(); k, v = b.kv_concat()
    out = oracle.attention_for_batch(b)
    vf = wl.bf16_bits_to_f64(v)
    t, h = 64, 2   # first decode, ctx 100
    w = oracle.softmax_weights(q, k, b.kv_start, b.q_start, b.q_len, b.ctx_len, b.sm_scale, t, h)
    keys = vf[b.kv_start[1]: b.kv_start[1] + 100, 0]
    np.testing.assert_allclose(out[t, h], w @ keys, rtol=1e-12, atol=1e-15)


def test_config1_against_dense_library():
    pin_checks.check_against_dense_library(oracle.hybrid_attention, wl.config1_tiny())


def test_token_subset_matches_full_run():
    b = wl.config1_tiny()
    full = oracle.attention_for_batch(b)
    toks = [66, 0, 63, 5]
    sub = oracle.attention_for_batch(b, tokens=toks)
    np.testing.assert_array_equal(sub, full[toks])


def test_config1_chunking_invariance_outputs_and_cache():
    """192-token prompt as 1x192, 3x64 and 192x1: same rows, same paged cache bytes."""
    outs, caches = [], []
    for chunk in (192, 64, 1):
        iters = wl.config1_prompt(chunk)
        k_all, v_all = iters[-1].kv_bits(0)
        q_all = wl.normal_bf16((1, 0x51, 99), (192, 4, 64))
        kc, vc = kvref.empty_pools(iters[0].num_pages, 1, 64, 16, fill=0x7FC0)
        rows = []
        for it in iters:
            n, ctx = int(it.q_len[0]), int(it.ctx_len[0])
            kvref.kv_append(kc, vc, k_all[ctx - n: ctx], v_all[ctx - n: ctx], it.block_table, it.q_start, it.q_len, it.ctx_len)
            # attention reads what the cache holds for positions 0..ctx-1
            kg, vg = kvref.gather_sequence(kc, vc, it.block_table[0], ctx)
            rows.append(oracle.hybrid_attention(q_all[ctx - n: ctx], kg, vg, [0], [0], [n], [ctx], it.sm_scale))
        outs.append(np.concatenate(rows))
        caches.append((kc.copy(), vc.copy()))
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])
    for kc, vc in caches[1:]:
        np.testing.assert_array_equal(kc, caches[0][0])
        np.testing.assert_array_equal(vc, caches[0][1])


def test_golden_rows_unchanged():
    """Stored rows written by tests/golden/make_golden.py (which calls only the checker)."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "config1_rows.txt")
    data = np.loadtxt(path)
    b = wl.config1_tiny()
    toks = [0, 63, 64, 65, 66]
    out = oracle.attention_for_batch(b, tokens=toks)
    np.testing.assert_allclose(out.reshape(len(toks), -1), data, rtol=1e-12, atol=1e-15)
