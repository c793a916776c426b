"""Token-budget profile on the GPU (section 4.3): times grow with the budget, the pick honours its target."""
import pytest

torch = pytest.importorskip("torch")

from paper_2403_02310_amd import token_budget as tb
from paper_2403_02310_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_profile_and_pick():
    shape = wl.AttnShape(8, 2, 128)
    timer = tb.gpu_timer(reps=15, warmup=3)
    rows = tb.profile(timer, shape, [64, 512, 2048], [700] * 8, chunk_prefix=1500, seed=3)
    print(rows, flush=True)
    assert rows[0]["seconds"] < rows[2]["seconds"]                      # 56 vs 2040 chunk rows on a 1500-token prefix
    # a target that the two smaller budgets meet whatever the noise between them (both are launch-bound here)
    pick = tb.compute_token_budget(rows, max(rows[0]["seconds"], rows[1]["seconds"]) * 1.05)
    assert pick in (512, 2048)
    assert tb.compute_token_budget(rows, min(r["seconds"] for r in rows) * 0.5) is None   # a target nothing meets
