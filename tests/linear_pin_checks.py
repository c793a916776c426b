"""Checks that pin the fp64 linear-layer checker to facts it does not compute itself.

Every check takes ``lin(x_bits, w_bits, rows=None, cols=None) -> float64 [rows, cols]`` so that the
same list runs against the committed checker (test_linear_oracle_pins.py) and against deliberately
broken copies of it (test_linear_oracle_mutants.py).  Inputs are bf16 bit patterns (uint16).
"""
from fractions import Fraction

import numpy as np


def bf16_bits(a) -> np.ndarray:
    """Round-to-nearest-even bf16 bit patterns of float values (independent of the checker's decoder)."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def bits_to_f64(b) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _normal(seed, shape):
    return bf16_bits(np.random.default_rng(seed).standard_normal(shape))


def check_against_float64_library_product(lin):
    """Section 2.1's linear transformation is a matrix product: numpy's float64 matmul on the same values."""
    for seed, (T, N, K) in enumerate([(5, 7, 3), (33, 20, 129), (64, 96, 512), (3, 130, 1000)]):
        x, w = _normal((seed, 1), (T, K)), _normal((seed, 2), (N, K))
        want = bits_to_f64(x) @ bits_to_f64(w).T
        got = lin(x, w)
        assert got.shape == (T, N)
        scale = np.abs(bits_to_f64(x)) @ np.abs(bits_to_f64(w)).T        # rounding-order slack only
        assert np.all(np.abs(got - want) <= 1e-13 * scale + 1e-300), (T, N, K)


def check_exact_rational_arithmetic_on_small_integers(lin):
    """Small integers: every product and partial sum is exact in double, so the result must equal the
    exact rational value, not just approximate it."""
    rng = np.random.default_rng(11)
    T, N, K = 4, 6, 9
    xi = rng.integers(-8, 9, size=(T, K)); wi = rng.integers(-8, 9, size=(N, K))
    got = lin(bf16_bits(xi), bf16_bits(wi))
    for t in range(T):
        for n in range(N):
            exact = sum(Fraction(int(xi[t, k])) * Fraction(int(wi[n, k])) for k in range(K))
            assert Fraction(got[t, n]) == exact, (t, n)


def check_identity_weight_returns_the_input(lin):
    K = 24
    x = _normal(21, (5, K))
    got = lin(x, bf16_bits(np.eye(K)))
    assert np.array_equal(got, bits_to_f64(x))


def check_one_hot_row_selects_a_weight_column(lin):
    """x = e_k0 picks w[n][k0] for every feature n; tells w[n][k] from w[k][n] when N != K."""
    N, K, k0 = 10, 6, 4
    w = _normal(31, (N, K))
    x = np.zeros((1, K)); x[0, k0] = 1.0
    got = lin(bf16_bits(x), w)
    assert np.array_equal(got[0], bits_to_f64(w)[:, k0])


def check_last_and_first_terms_count(lin):
    """Only the first (or only the last) k carries weight: an off-by-one in the k loop loses it."""
    K = 17
    for k0 in (0, K - 1):
        x = np.zeros((2, K)); x[:, k0] = [2.0, -3.0]
        w = np.zeros((3, K)); w[:, k0] = [0.5, 4.0, -1.0]
        got = lin(bf16_bits(x), bf16_bits(w))
        assert np.array_equal(got, np.outer([2.0, -3.0], [0.5, 4.0, -1.0]))


def check_sum_that_single_precision_would_lose(lin):
    """65536 + 64 * 2^-8: each small term is below half an ulp of 65536 in single precision, so a
    float accumulator returns 65536; double returns 65536.25 exactly."""
    K = 65
    x = np.full((1, K), 2.0 ** -4); w = np.full((1, K), 2.0 ** -4)
    x[0, 0] = 256.0; w[0, 0] = 256.0
    got = lin(bf16_bits(x), bf16_bits(w))
    assert got[0, 0] == 65536.25


def check_bf16_values_are_decoded_in_full(lin):
    """1.0078125 = 1 + 2^-7 uses the lowest mantissa bit of bf16."""
    x = bf16_bits(np.array([[1.0078125]])); w = bf16_bits(np.array([[1.0078125]]))
    assert bits_to_f64(x)[0, 0] == 1.0078125
    assert lin(x, w)[0, 0] == 1.0078125 ** 2


def check_additivity_on_exact_inputs(lin):
    """lin(x1 + x2) = lin(x1) + lin(x2) exactly when all values are small integers."""
    rng = np.random.default_rng(41)
    x1 = rng.integers(-4, 5, size=(3, 12)); x2 = rng.integers(-4, 5, size=(3, 12)); w = rng.integers(-4, 5, size=(5, 12))
    a = lin(bf16_bits(x1), bf16_bits(w)); b = lin(bf16_bits(x2), bf16_bits(w)); c = lin(bf16_bits(x1 + x2), bf16_bits(w))
    assert np.array_equal(a + b, c)


def check_row_and_column_subsets(lin):
    x, w = _normal(51, (9, 40)), _normal(52, (13, 40))
    full = lin(x, w)
    rows, cols = [8, 0, 3], [12, 1, 1, 7]
    assert np.array_equal(lin(x, w, rows=rows), full[rows])
    assert np.array_equal(lin(x, w, cols=cols), full[:, cols])
    assert np.array_equal(lin(x, w, rows=rows, cols=cols), full[np.ix_(rows, cols)])


def check_tokens_do_not_mix(lin):
    """A token's output depends on its own row only (the batch dimension is a plain loop)."""
    x, w = _normal(61, (6, 32)), _normal(62, (8, 32))
    full = lin(x, w)
    for t in (0, 5):
        assert np.array_equal(lin(x[t:t + 1], w)[0], full[t])


ALL_CHECKS = [
    check_against_float64_library_product,
    check_exact_rational_arithmetic_on_small_integers,
    check_identity_weight_returns_the_input,
    check_one_hot_row_selects_a_weight_column,
    check_last_and_first_terms_count,
    check_sum_that_single_precision_would_lose,
    check_bf16_values_are_decoded_in_full,
    check_additivity_on_exact_inputs,
    check_row_and_column_subsets,
    check_tokens_do_not_mix,
]
