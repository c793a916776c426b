"""Token-budget profile on the GPU (section 4.3): every profiled batch computes what the fp64 checker computes,
times grow with the budget, and the pick equals the reference rule applied to the same profile."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import kv_cache_reference as kvref
from oracle import token_budget_reference as tbref
from paper_2403_02310_amd import token_budget as tb
from paper_2403_02310_amd import workloads as wl
from tests.parity import compare

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def test_profile_and_pick():
    shape = wl.AttnShape(8, 2, 128)
    checked = []

    def check(batch, dev):
        """The launches that were timed wrote `out`: compare it with the checker on the cache as it stands."""
        kc, vc, bt = _bits(dev["k_cache"]), _bits(dev["v_cache"]), dev["block_table"].cpu().numpy()
        ks, vs = [], []
        for s in range(batch.num_seqs):
            k, v = kvref.gather_sequence(kc, vc, bt[s], int(batch.ctx_len[s]))
            ks.append(k); vs.append(v)
        ref = oracle.hybrid_attention(_bits(dev["q"]), np.concatenate(ks), np.concatenate(vs), batch.kv_start, batch.q_start,
                                      batch.q_len, batch.ctx_len, batch.sm_scale)
        got = dev["out"].to(torch.float32).cpu().numpy().astype(np.float64)
        res = compare(got, ref, batch.name)
        checked.append((batch.name, batch.num_tokens, res))
        print("profiled batch", batch.name, "tokens", batch.num_tokens, "max abs %.2e max row rel %.2e" % res, flush=True)

    timer = tb.gpu_timer(reps=15, warmup=3, on_batch=check)
    budgets = [4, 64, 512, 2048]                                        # 4 < the 8 decodes: no prefill token in that batch
    rows = tb.profile(timer, shape, budgets, [700] * 8, chunk_prefix=1500, seed=3)
    print(rows, flush=True)
    assert [c[1] for c in checked] == [8, 64, 512, 2048]                # decodes are never dropped; otherwise the budget is used up
    assert rows[0]["seconds"] < rows[3]["seconds"]                      # no chunk vs 2040 chunk rows on a 1500-token prefix
    profile = {r["token_budget"]: r["seconds"] for r in rows}
    times = sorted(profile.values())
    for target in (times[0] * 0.5, times[-1] * 2.0, 0.5 * (times[-2] + times[-1]), times[1]):
        assert tb.compute_token_budget(rows, target) == tbref.compute_token_budget(profile, target)
    assert tb.compute_token_budget(rows, times[0] * 0.5) is None        # a target nothing meets
    assert tb.compute_token_budget(rows, times[-1] * 2.0) == 2048
