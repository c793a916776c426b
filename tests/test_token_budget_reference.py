"""CPU pins of oracle/token_budget_reference.py (section 4.3: the largest token count whose iteration, and
every smaller batch's, meets the latency target), and the product's compute_token_budget against it."""
import itertools
import os
import types

import numpy as np
import pytest

from oracle import token_budget_reference as ref
from paper_2403_02310_amd import token_budget as tb

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "token_budget_reference.py")


def check_closed_form_on_a_linear_profile(fn):
    """time(tau) = a + b*tau grows with tau, so the answer is the largest profiled tau <= (T - a) / b."""
    a, b = 40e-6, 0.25e-6
    grid = [64, 128, 256, 512, 1024, 2048, 4096]
    prof = {t: a + b * t for t in grid}
    for target in (a + b * 512, a + b * 512 * 1.0001, a + b * 511.9, 1.0, a + b * 64, a + b * 63.9, 0.0):
        bound = (target - a) / b
        fits = [t for t in grid if t <= bound * (1 + 1e-12)]
        assert fn(prof, target) == (max(fits) if fits else None), target


def check_equality_meets_the_target(fn):
    prof = {100: 1.0, 200: 2.0, 300: 3.0}
    assert fn(prof, 2.0) == 200            # exactly T_max is within the objective
    assert fn(prof, np.nextafter(2.0, 0.0)) == 100
    assert fn(prof, 3.0) == 300 and fn(prof, 0.5) is None


def check_smaller_batches_must_meet_it_too(fn):
    # the 256-token batch misses a 3.0 target, so no budget above 128 is acceptable although 512 "fits"
    prof = {64: 1.0, 128: 2.0, 256: 5.0, 512: 2.5}
    assert fn(prof, 3.0) == 128
    assert fn(prof, 5.0) == 512
    assert fn({64: 9.0, 128: 1.0}, 2.0) is None     # the smallest batch already misses it


def check_order_of_the_rows_is_irrelevant(fn):
    prof = {64: 1.0, 128: 2.0, 256: 3.0, 512: 4.0, 1024: 5.0}
    for perm in itertools.permutations(prof.items()):
        assert fn(dict(perm), 3.5) == 256


def check_brute_force_on_random_profiles(fn):
    """Against the definition spelled out a second way: sort, walk up, stop at the first miss."""
    rng = np.random.default_rng(5)
    for _ in range(300):
        n = int(rng.integers(1, 8))
        taus = rng.choice(np.arange(1, 5000), size=n, replace=False).tolist()
        times = rng.uniform(0.0, 10.0, size=n).round(1).tolist()     # coarse values: ties with the target happen
        target = float(rng.choice(times + [0.0, 5.0, 10.0]))
        expect = None
        for t, s in sorted(zip(taus, times)):
            if s > target:
                break
            expect = t
        assert fn(dict(zip(taus, times)), target) == expect


PINS = [check_closed_form_on_a_linear_profile, check_equality_meets_the_target, check_smaller_batches_must_meet_it_too,
        check_order_of_the_rows_is_irrelevant, check_brute_force_on_random_profiles]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_reference_meets_its_pins(pin):
    pin(ref.compute_token_budget)


def _product(profile, t_max):
    rows = [{"token_budget": t, "tokens": t, "seconds": s} for t, s in profile.items()]
    return tb.compute_token_budget(rows, t_max)


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_product_meets_the_same_pins(pin):
    pin(_product)


def test_product_equals_reference_on_random_profiles():
    rng = np.random.default_rng(6)
    for _ in range(500):
        n = int(rng.integers(1, 9))
        taus = rng.choice(np.arange(1, 9000), size=n, replace=False).tolist()
        times = rng.uniform(0.0, 10.0, size=n).round(1).tolist()
        target = float(rng.choice(times + [0.0, 5.0, 10.0]))
        prof = dict(zip(taus, times))
        assert _product(prof, target) == ref.compute_token_budget(prof, target)


MUTANTS = {
    "strict_comparison": ("not (seconds <= t_max)", "not (seconds < t_max)"),
    "larger_batches_checked_instead": ("if other <= tau and", "if other >= tau and"),
    "own_time_only": ("if other <= tau and", "if other == tau and"),
    "smallest_safe_count": ("tau > best", "tau < best"),
    "strictly_smaller_batches_only": ("if other <= tau and", "if other < tau and"),
    "target_ignored": ("not (seconds <= t_max)", "not (seconds <= seconds)"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_of_the_reference_trips_a_pin(name):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1
    mod = types.ModuleType("token_budget_mutant_" + name)
    exec(compile(text.replace(old, new), name + ".py", "exec"), mod.__dict__)
    tripped = []
    for pin in PINS:
        try:
            pin(mod.compute_token_budget)
        except AssertionError:
            tripped.append(pin.__name__)
    assert tripped, "mutant %s passed every pin" % name
