"""CPU test: plausible mistakes planted in COPIES of the scheduler reference each trip a pin.

The mutants are made from the text of oracle/scheduler_reference.py by substitution and run from a
module object of their own; the committed reference is never modified.  A mutant that passed every pin of
tests/scheduler_pin_checks.py would show that the pins are too weak to trust the reference (and, through it,
the library's host scheduler, which must equal the reference state by state).
"""
import os
import types

import pytest

from tests import scheduler_pin_checks as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "scheduler_reference.py")

DECODE_PASS = """    for (rid, prompt_len, num_prefilled, num_decoded) in running_decodes:
        assert num_prefilled == prompt_len
        n_t += 1
        ids.append(rid)
        q_len.append(1)
        ctx_len.append(prompt_len + num_decoded + 1)
    n_dec = len(ids)
"""

MUTANTS = {
    # decodes placed after the prefills of the running requests (a prefill could then use up the budget first)
    "decodes_after_running_prefills": None,   # built below by moving a block
    # the decodes' tokens are not charged to the budget
    "budget_ignores_decodes": ("        assert num_prefilled == prompt_len\n        n_t += 1\n", "        assert num_prefilled == prompt_len\n"),
    # the context of a decode forgets the token fed in this iteration
    "decode_context_without_new_token": ("ctx_len.append(prompt_len + num_decoded + 1)", "ctx_len.append(prompt_len + num_decoded)"),
    # the separate cap on the chunk size is dropped
    "chunk_size_cap_dropped": ("return max(0, min(prompt_len - num_prefilled, chunk_size, token_budget - n_t))",
                               "return max(0, min(prompt_len - num_prefilled, token_budget - n_t))"),
    # a chunk may run past the end of its prompt
    "chunk_ignores_prompt_end": ("return max(0, min(prompt_len - num_prefilled, chunk_size, token_budget - n_t))",
                                 "return max(0, min(chunk_size, token_budget - n_t))"),
    # the leftover budget does not bound the chunk
    "chunk_ignores_leftover_budget": ("return max(0, min(prompt_len - num_prefilled, chunk_size, token_budget - n_t))",
                                      "return max(0, min(prompt_len - num_prefilled, chunk_size))"),
    # a chunk smaller than the leftover budget admits (half of it)
    "chunk_not_the_largest": ("return max(0, min(prompt_len - num_prefilled, chunk_size, token_budget - n_t))",
                              "return max(0, min(prompt_len - num_prefilled, chunk_size, (token_budget - n_t + 1) // 2))"),
    # the chunk's context forgets the tokens prefilled earlier
    "chunk_context_without_prefix": ("            ctx_len.append(num_prefilled + c)\n            n_chunks += 1\n    # pass 3",
                                     "            ctx_len.append(c)\n            n_chunks += 1\n    # pass 3"),
    # a request gets a second chunk in the same iteration
    "two_chunks_per_request": ("            ctx_len.append(num_prefilled + c)\n            n_chunks += 1\n    # pass 3",
                               "            ctx_len.append(num_prefilled + c)\n            n_chunks += 1\n"
                               "            c2 = next_chunk_size(prompt_len, num_prefilled + c, chunk_size, token_budget, n_t)\n"
                               "            if c2 > 0:\n                n_t += c2; ids.append(rid); q_len.append(c2); ctx_len.append(num_prefilled + c + c2); n_chunks += 1\n"
                               "    # pass 3"),
    # a waiting request that cannot be admitted is skipped and a later one taken (not first come first served)
    "admission_past_a_blocked_request": ("        if not (pages <= free_pages and n_t < token_budget and len(ids) < max_batch_size):\n            break",
                                         "        if not (pages <= free_pages and n_t < token_budget and len(ids) < max_batch_size):\n            continue"),
    # admitted prompts do not reserve their pages
    "pages_not_reserved": ("        free_pages -= pages\n", ""),
    # the memory test is dropped
    "memory_never_checked": ("if not (pages <= free_pages and n_t < token_budget", "if not (n_t < token_budget"),
    # only the first chunk's pages are reserved, not the prompt's
    "pages_of_the_chunk_only": ("        free_pages -= pages\n", "        free_pages -= (c + page_size - 1) // page_size\n"),
    # an exact fit is refused (this build's reading admits it)
    "exact_fit_refused": ("if not (pages <= free_pages and", "if not (pages < free_pages and"),
    # the row offsets of the batch are not the running sum of the lengths
    "q_start_not_the_prefix_sum": ("q_start[i] = q_start[i - 1] + q_len[i - 1]", "q_start[i] = q_start[i - 1] + q_len[i]"),
    # only one new request per iteration
    "one_admission_per_iteration": ("        n_chunks += 1\n        admitted += 1\n", "        n_chunks += 1\n        admitted += 1\n        break\n"),
    # running prefills stop at the first one that gets a chunk
    "one_running_prefill_per_iteration": ("            ctx_len.append(num_prefilled + c)\n            n_chunks += 1\n    # pass 3",
                                          "            ctx_len.append(num_prefilled + c)\n            n_chunks += 1\n            break\n    # pass 3"),
}


def _mutant_source(name):
    text = open(SRC).read()
    if name == "decodes_after_running_prefills":
        assert text.count(DECODE_PASS) == 1
        text = text.replace(DECODE_PASS, "")
        anchor = "    # pass 3: new requests, first come first served\n"
        assert text.count(anchor) == 1
        moved = DECODE_PASS.replace("    n_dec = len(ids)\n", "    n_dec = len(running_decodes)\n")
        return text.replace(anchor, moved + anchor)
    old, new = MUTANTS[name]
    assert text.count(old) == 1, "mutation anchor for %s must match exactly once" % name
    return text.replace(old, new)


def _impl_of(source, name):
    mod = types.ModuleType("scheduler_mutant_" + name)
    mod.__dict__["__name__"] = mod.__name__
    import sys
    sys.modules[mod.__name__] = mod          # dataclasses looks the module up while the class is being made
    try:
        exec(compile(source, name + ".py", "exec"), mod.__dict__)
    finally:
        del sys.modules[mod.__name__]

    def impl(tb, cs, dec, pre, wait, free, page=16, maxb=128):
        return pins.as_dict(mod.build_stall_free_batch(tb, cs, dec, pre, wait, free, page, maxb))
    return impl


CHECKS = [pins.check_invariants_on_random_states, pins.check_config_shapes, pins.check_figure_scenario_and_full_drain,
          pins.check_admission_reading]


def test_the_unmodified_reference_passes_every_pin():
    impl = _impl_of(open(SRC).read(), "identity")
    for check in CHECKS:
        check(impl)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_trips_a_pin(name):
    impl = _impl_of(_mutant_source(name), name)
    tripped = []
    for check in CHECKS:
        try:
            check(impl)
        except (AssertionError, KeyError, IndexError, OverflowError, ValueError) as e:
            tripped.append(check.__name__)
    assert tripped, "mutant %s passed every scheduler pin" % name
    print(name, "tripped", tripped)


def test_which_pin_catches_the_admission_edge():
    """The paper leaves can_allocate_request undefined; of the pins only the explicit statement of this build's
    reading (an exact fit is admitted) tells `<=` from `<`: the invariants hold for both."""
    impl = _impl_of(_mutant_source("exact_fit_refused"), "exact_fit_refused")
    pins.check_config_shapes(impl)
    pins.check_figure_scenario_and_full_drain(impl)
    with pytest.raises(AssertionError):
        pins.check_admission_reading(impl)
