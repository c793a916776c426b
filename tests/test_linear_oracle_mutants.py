"""CPU test: plausible mistakes planted in COPIES of the linear-layer checker each trip a pin.

The mutants are built in a temporary directory from oracle/linear_oracle.c by textual substitution;
the committed checker is never modified."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from tests import linear_pin_checks

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "linear_oracle.c")

MUTANTS = {
    "weight_read_transposed": ("const uint16_t *w_row = w + (int64_t)n * K;\n            double sum = 0.0;\n            for (int k = 0; k < K; ++k) sum += bf16_to_f64(x_row[k]) * bf16_to_f64(w_row[k]);",
                               "double sum = 0.0;\n            for (int k = 0; k < K; ++k) sum += bf16_to_f64(x_row[k]) * bf16_to_f64(w[(int64_t)k * N + n]);"),
    "last_term_dropped": ("for (int k = 0; k < K; ++k) sum +=", "for (int k = 0; k < K - 1; ++k) sum +="),
    "first_term_dropped": ("for (int k = 0; k < K; ++k) sum +=", "for (int k = 1; k < K; ++k) sum +="),
    "single_precision_sum": ("double sum = 0.0;", "float sum = 0.0f;"),
    "token_row_zero": ("const uint16_t *x_row = x + (int64_t)t * K;", "const uint16_t *x_row = x + (int64_t)0 * K;"),
    "row_list_ignored": ("const int t = rows ? rows[r] : r;", "const int t = r;"),
    "column_list_ignored": ("const int n = cols ? cols[c] : c;", "const int n = c;"),
    "output_stride_is_N": ("out[(int64_t)r * C + c] = sum;", "out[(int64_t)r * N + c] = sum;"),
    "bf16_low_bit": ("uint32_t u = ((uint32_t)bits) << 16;", "uint32_t u = ((uint32_t)(bits & 0xFFFE)) << 16;"),
    "sign_of_weight": ("bf16_to_f64(x_row[k]) * bf16_to_f64(w_row[k]);", "bf16_to_f64(x_row[k]) * -bf16_to_f64(w_row[k]);"),
}


def _build(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation anchor for %s must match exactly once" % name
    src = tmp_path / (name + ".c")
    src.write_text(text.replace(old, new))
    lib = tmp_path / (name + ".so")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(lib), str(src)], check=True)
    return ctypes.CDLL(str(lib))


def _as_linear(lib):
    u16p = ctypes.POINTER(ctypes.c_uint16); i32p = ctypes.POINTER(ctypes.c_int32); f64p = ctypes.POINTER(ctypes.c_double)
    fn = lib.oracle_linear
    fn.restype = ctypes.c_int

    def lin(x, w, rows=None, cols=None):
        x = np.ascontiguousarray(x, np.uint16); w = np.ascontiguousarray(w, np.uint16)
        T, K = x.shape; N = w.shape[0]
        r = None if rows is None else np.ascontiguousarray(rows, np.int32)
        c = None if cols is None else np.ascontiguousarray(cols, np.int32)
        R = T if r is None else len(r); C = N if c is None else len(c)
        # room for a mutant that writes with the wrong stride; the result is the leading [R, C] block
        out = np.full(R * max(C, N) + N, np.nan)
        rc = fn(x.ctypes.data_as(u16p), w.ctypes.data_as(u16p), ctypes.c_int(T), ctypes.c_int(N), ctypes.c_int(K),
                None if r is None else r.ctypes.data_as(i32p), ctypes.c_int(R),
                None if c is None else c.ctypes.data_as(i32p), ctypes.c_int(C),
                out.ctypes.data_as(f64p), ctypes.c_int(1))
        assert rc == 0
        return out[:R * C].reshape(R, C)
    return lin


def test_unmodified_copy_passes_every_pin(tmp_path):
    lin = _as_linear(_build(tmp_path, "clean", "double sum = 0.0;", "double sum = 0.0; "))
    for check in linear_pin_checks.ALL_CHECKS:
        check(lin)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_trips_a_pin(tmp_path, name):
    old, new = MUTANTS[name]
    lin = _as_linear(_build(tmp_path, name, old, new))
    tripped = []
    for check in linear_pin_checks.ALL_CHECKS:
        try:
            check(lin)
        except AssertionError:
            tripped.append(check.__name__)
    assert tripped, "no pin noticed the mutant %s" % name
