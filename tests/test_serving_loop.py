"""Host logic of the serving loop (no GPU): stall-free scheduling over many iterations, page and slot
accounting, and the contrast with the prefill-prioritising toy policy (sections 3.2, 4.2)."""
import numpy as np
import pytest

from paper_2403_02310_amd import serving
from paper_2403_02310_amd import workloads as wl

SHAPE = wl.AttnShape(8, 2, 128)


def _trace(seed=7, n=40, qps=2000.0):
    return serving.synthetic_trace(seed, n, qps, prompt_median=300, prompt_p90=900, output_median=20, output_p90=40,
                                   max_prompt=1500, max_output=64)


def _loop(policy, budget=256, chunk=256, pages=20000, reqs=None, cost=None):
    reqs = reqs if reqs is not None else _trace()
    return serving.ServingLoop(SHAPE, reqs, serving.DryBackend(cost), num_pages=pages, token_budget=budget,
                               chunk_size=chunk, max_batch_size=64, policy=policy, seed=3)


def test_trace_follows_requested_statistics():
    reqs = serving.synthetic_trace(1, 4000, 5.0)
    prompts = np.array([r.prompt_len for r in reqs]); outs = np.array([r.output_len for r in reqs])
    assert abs(np.median(prompts) - 1730) / 1730 < 0.08 and abs(np.percentile(prompts, 90) - 5696) / 5696 < 0.1
    assert abs(np.median(outs) - 415) / 415 < 0.08
    assert all(b.arrival_s >= a.arrival_s for a, b in zip(reqs, reqs[1:]))
    assert [r.token_base for r in reqs[:3]] == [0, reqs[0].total_rows, reqs[0].total_rows + reqs[1].total_rows]


@pytest.mark.parametrize("policy", ["stall_free", "prefill_first"])
def test_every_request_completes_and_memory_returns(policy):
    loop = _loop(policy).run()
    assert len(loop.done) == len(loop.requests)
    assert loop.pool.free == loop.pool.num_pages and len(loop._free_slots) == loop.max_seqs
    for r in loop.done:
        assert r.num_prefilled == r.prompt_len and r.num_decoded == r.output_len - 1
        assert r.arrival_s <= r.first_token_s <= r.finish_s
    # every attention row of every request was scheduled exactly once
    assert sum(it.num_tokens for it in loop.iterations) == sum(r.total_rows for r in loop.requests)


def test_stall_free_never_drops_a_decode_and_respects_the_budget():
    loop = _loop("stall_free", budget=128, chunk=96).run()
    assert any(it.num_prefill_tokens and it.num_decodes for it in loop.iterations)   # hybrid batches do occur
    for it in loop.iterations:
        assert it.num_decodes == it.num_running_decodes                     # section 4.2: decodes never stall
        assert it.num_prefill_tokens <= max(0, 128 - it.num_decodes)         # prefills only get the leftover budget
        assert it.num_tokens == it.num_decodes + it.num_prefill_tokens


def test_prefill_first_stalls_decodes_and_stall_free_does_not():
    """With iteration cost proportional to the work in it, whole-prompt iterations stretch the gap between two
    generated tokens of a running request; stall-free batching bounds it by the budget's cost (section 3.2/4.2)."""
    cost = lambda q_len, ctx_len: 10e-6 + 1e-9 * float((q_len.astype(np.float64) * ctx_len).sum())
    reqs = _trace(seed=11, n=60, qps=30000.0)
    a = _loop("stall_free", budget=128, chunk=128, reqs=reqs, cost=cost).run()
    b = _loop("prefill_first", reqs=reqs, cost=cost).run()
    assert any(it.num_prefill_tokens > 0 and it.num_running_decodes > 0 and it.num_decodes == 0 for it in b.iterations)
    assert max(a.tbt_s) < 0.5 * max(b.tbt_s)
    sa, sb = a.summary(), b.summary()
    assert sa["requests_done"] == sb["requests_done"] == 60 and sa["generated_tokens"] == sb["generated_tokens"]


def test_page_pool_exhaustion_is_an_error_not_a_wild_index():
    pool = serving.PagePool(4, seed=1)
    got = pool.take(3)
    assert len(set(got)) == 3 and pool.free == 1
    with pytest.raises(RuntimeError):
        pool.take(2)
    pool.give(got)
    assert pool.free == 4


def test_admission_waits_for_pages():
    """A prompt enters only when its pages are free (the reading of can_allocate_request): with a pool that holds one
    long prompt at a time, requests are served one after the other and all complete."""
    reqs = [serving.Request(i, 0.0, 400, 3, token_base=i * 402) for i in range(4)]
    loop = _loop("stall_free", budget=128, chunk=128, pages=30, reqs=reqs).run()
    assert len(loop.done) == 4
    starts = sorted(r.first_token_s for r in loop.done)
    assert all(b > a for a, b in zip(starts, starts[1:]))


@pytest.mark.parametrize("policy", ["stall_free", "prefill_first"])
def test_a_pool_barely_larger_than_the_working_set_never_stalls_a_decode(policy):
    """Decodes grow by a page every 16 generated tokens.  If admission looked at prompts only, a pool this tight would
    run dry in the middle of a generation (and the loop would die); setting aside a request's lifetime pages at
    admission makes new requests wait instead, and every running decode still gets its token in every iteration."""
    # prompts of 2 pages that generate 150 tokens (11 pages over their life); the pool holds three such lifetimes
    reqs = [serving.Request(i, 0.0, 32, 150, token_base=i * 181) for i in range(9)]
    pages = 3 * ((32 + 149 + 15) // 16)
    loop = _loop(policy, budget=64, chunk=64, pages=pages, reqs=reqs).run()
    assert len(loop.done) == 9 and loop.pool.free == pages
    assert max(it.num_running_decodes for it in loop.iterations) == 3          # never more than fit for their whole life
    if policy == "stall_free":
        assert all(it.num_decodes == it.num_running_decodes for it in loop.iterations)
    # with prompts alone as the admission test all nine would have entered at once (18 pages of 36) and run dry
    assert sum((r.prompt_len + 15) // 16 for r in reqs) <= pages


def test_a_request_that_can_never_fit_is_reported():
    reqs = [serving.Request(0, 0.0, 64, 400, token_base=0)]
    with pytest.raises(RuntimeError, match="cannot hold"):
        _loop("stall_free", pages=10, reqs=reqs).run()
