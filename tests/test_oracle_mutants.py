"""CPU test: plausible mistakes planted in COPIES of the checker's source each trip a pin.

The mutants are built in a temporary directory from oracle/attention_oracle.c by textual
substitution; the committed checker is never modified.  If a mutant passed every pin, the
pins would be too weak to trust the checker.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from tests import pin_checks

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "attention_oracle.c")

MUTANTS = {
    "exclusive_mask": ("for (int i = lo; i <= pos; ++i) {\n        const uint16_t *k_row",
                       "for (int i = lo; i < pos; ++i) {\n        const uint16_t *k_row"),
    "wrong_group_map": ("const int g = h / group; ", "const int g = h % num_kv_heads; "),
    "scale_dropped": ("x[i] = sm_scale * dot;", "x[i] = dot;"),
    "sign_flipped": ("x[i] = exp(x[i] - m);", "x[i] = exp(m - x[i]);"),
    "no_normalisation": ("for (int i = lo; i <= pos; ++i) x[i] /= z;", ""),
    "v_head_zero": ("const uint16_t *v_row = vs + ((int64_t)i * num_kv_heads + g) * d;",
                    "const uint16_t *v_row = vs + ((int64_t)i * num_kv_heads + 0) * d;"),
    "k_head_zero": ("const uint16_t *k_row = k_seq + ((int64_t)i * num_kv_heads + kv_head) * d;",
                    "const uint16_t *k_row = k_seq + ((int64_t)i * num_kv_heads + 0) * d;"),
    "prefix_ignored": ("const int pos = ctx_len[s] - q_len[s] + j;       /*", "const int pos = ctx_len[s] - 1;       /*"),
    "position_off_by_one": ("const int pos = ctx_len[s] - q_len[s] + j;       /*", "const int pos = ctx_len[s] - q_len[s] + j - (j > 0);       /*"),
    "v_weight_shifted": ("o[c] += w[i] * bf16_to_f64(v_row[c]);", "o[c] += w[pos - i] * bf16_to_f64(v_row[c]);"),
    "q_k_channel_mismatch": ("dot += bf16_to_f64(q_row[c]) * bf16_to_f64(k_row[c]);",
                             "dot += bf16_to_f64(q_row[c]) * bf16_to_f64(k_row[d - 1 - c]);"),
    "wrong_sequence_kv": ("const uint16_t *vs = v_seq + kv_start[s] * num_kv_heads * d;",
                          "const uint16_t *vs = v_seq + kv_start[0] * num_kv_heads * d;"),
    "bf16_low_bits": ("uint32_t u = ((uint32_t)bits) << 16;", "uint32_t u = ((uint32_t)(bits & 0xFFFE)) << 16;"),
}

# mistakes in the sliding window: caught by the window pins
WINDOW_MUTANTS = {
    "window_off_by_one": ("const int lo = pos - window + 1;", "const int lo = pos - window;"),
    "window_ignored": ("if (window <= 0) return 0;", "return 0;"),
    "window_from_sequence_end": ("const int lo = window_first_key(pos, window);", "const int lo = window_first_key(ctx_len[s] - 1, window);"),
    "window_scores_only": ("for (int i = lo; i <= pos; ++i) {\n                    const uint16_t *v_row",
                           "for (int i = 0; i <= pos; ++i) {\n                    const uint16_t *v_row"),
}


def _build(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation anchor for %s must match exactly once" % name
    src = tmp_path / (name + ".c")
    src.write_text(text.replace(old, new))
    lib = tmp_path / (name + ".so")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(lib), str(src), "-lm"], check=True)
    return ctypes.CDLL(str(lib))


def _as_attn(lib):
    u16p = ctypes.POINTER(ctypes.c_uint16); i32p = ctypes.POINTER(ctypes.c_int32)
    i64p = ctypes.POINTER(ctypes.c_int64); f64p = ctypes.POINTER(ctypes.c_double)
    fn = lib.oracle_hybrid_attention
    fn.restype = ctypes.c_int

    fnw = lib.oracle_hybrid_attention_window
    fnw.restype = ctypes.c_int

    def attn(q, k, v, kv_start, q_start, q_len, ctx_len, scale, window=None):
        q = np.ascontiguousarray(q, np.uint16); k = np.ascontiguousarray(k, np.uint16); v = np.ascontiguousarray(v, np.uint16)
        kvs = np.ascontiguousarray(kv_start, np.int64); qs = np.ascontiguousarray(q_start, np.int32)
        ql = np.ascontiguousarray(q_len, np.int32); cl = np.ascontiguousarray(ctx_len, np.int32)
        T, Hq, d = q.shape
        out = np.empty((T, Hq, d), np.float64)
        head = (q.ctypes.data_as(u16p), k.ctypes.data_as(u16p), v.ctypes.data_as(u16p), kvs.ctypes.data_as(i64p),
                qs.ctypes.data_as(i32p), ql.ctypes.data_as(i32p), cl.ctypes.data_as(i32p),
                ctypes.c_int(len(ql)), ctypes.c_int(T), ctypes.c_int(Hq), ctypes.c_int(k.shape[1]), ctypes.c_int(d),
                ctypes.c_double(scale))
        tail = (None, ctypes.c_int(T), out.ctypes.data_as(f64p), ctypes.c_int(1))
        rc = fn(*head, *tail) if window is None else fnw(*head, ctypes.c_int(window), *tail)
        assert rc == 0
        return out
    return attn


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(tmp_path, name):
    old, new = MUTANTS[name]
    attn = _as_attn(_build(tmp_path, name, old, new))
    tripped = []
    for check in pin_checks.ALL_CHECKS:
        try:
            with np.errstate(all="ignore"):
                check(attn)
        except AssertionError:
            tripped.append(check.__name__)
    assert tripped, "mutant %s passed every pin" % name


@pytest.mark.parametrize("name", sorted(WINDOW_MUTANTS))
def test_window_mutant_is_caught(tmp_path, name):
    old, new = WINDOW_MUTANTS[name]
    attn = _as_attn(_build(tmp_path, name, old, new))
    tripped = []
    for check in pin_checks.WINDOW_CHECKS:
        try:
            with np.errstate(all="ignore"):
                check(attn)
        except AssertionError:
            tripped.append(check.__name__)
    assert tripped, "window mutant %s passed every window pin" % name


def test_unmutated_copy_passes(tmp_path):
    attn = _as_attn(_build(tmp_path, "identity", "int oracle_max_threads(void)", "int oracle_max_threads(void)"))
    for check in pin_checks.ALL_CHECKS + pin_checks.WINDOW_CHECKS:
        check(attn)
