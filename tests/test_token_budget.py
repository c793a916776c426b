"""Token-budget selection (section 4.3): host logic with a synthetic timer."""
import numpy as np

from paper_2403_02310_amd import token_budget as tb
from paper_2403_02310_amd import workloads as wl

SHAPE = wl.AttnShape(8, 2, 128)


def test_budget_batch_is_the_fullest_stall_free_batch():
    b = tb.budget_batch(SHAPE, 512, [100, 200, 300], chunk_prefix=1000)
    assert b.q_len.tolist() == [1, 1, 1, 509] and b.ctx_len.tolist() == [100, 200, 300, 1509]
    assert b.num_tokens == 512
    # more decodes than budget: they all stay and no prefill token is added (Algorithm 3 gives a prefill only what
    # the decodes leave of the budget)
    tiny = tb.budget_batch(SHAPE, 2, [50, 60, 70], chunk_prefix=0)
    assert tiny.q_len.tolist() == [1, 1, 1] and tiny.ctx_len.tolist() == [50, 60, 70]
    exact = tb.budget_batch(SHAPE, 3, [50, 60, 70], chunk_prefix=10)    # decodes use the budget up exactly
    assert exact.q_len.tolist() == [1, 1, 1]
    one = tb.budget_batch(SHAPE, 4, [50, 60, 70], chunk_prefix=10)
    assert one.q_len.tolist() == [1, 1, 1, 1] and one.ctx_len.tolist() == [50, 60, 70, 11]
    for tau in (64, 512, 4096):
        assert tb.budget_batch(SHAPE, tau, [500] * 16, chunk_prefix=1000).num_tokens == tau


def test_largest_budget_under_the_target():
    cost = lambda b: 10e-6 + 1e-9 * float((b.q_len.astype(np.float64) * b.ctx_len).sum())
    rows = tb.profile(cost, SHAPE, [64, 128, 256, 512, 1024, 2048], [500] * 16, chunk_prefix=1000)
    assert [r["token_budget"] for r in rows] == [64, 128, 256, 512, 1024, 2048]
    assert all(a["seconds"] < b["seconds"] for a, b in zip(rows, rows[1:]))
    t512 = rows[3]["seconds"]
    assert tb.compute_token_budget(rows, t512) == 512
    assert tb.compute_token_budget(rows, t512 * 0.999) == 256
    assert tb.compute_token_budget(rows, 1.0) == 2048
    assert tb.compute_token_budget(rows, rows[0]["seconds"] * 0.5) is None


def test_a_noisy_dip_does_not_raise_the_budget():
    rows = [{"token_budget": t, "tokens": t, "seconds": s} for t, s in [(64, 1.0), (128, 2.0), (256, 5.0), (512, 2.5)]]
    assert tb.compute_token_budget(rows, 3.0) == 128
