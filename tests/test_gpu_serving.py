"""Serving loop on the GPU: a request's attention rows, gathered over all the hybrid batches it travelled in,
must equal one one-shot fp64 computation over its whole sequence (chunking invariance at system level,
sections 4.1 and 4.3), under both scheduling policies."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2403_02310_amd import serving
from paper_2403_02310_amd import workloads as wl
from tests.parity import compare

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("policy", ["stall_free", "prefill_first"])
def test_requests_match_one_shot_attention(policy):
    shape = wl.AttnShape(8, 2, 128)
    reqs = serving.synthetic_trace(21, 10, 50000.0, prompt_median=150, prompt_p90=420, output_median=8, output_p90=14,
                                   max_prompt=600, max_output=16)
    backend = serving.GpuBackend(seed=5)
    loop = serving.ServingLoop(shape, reqs, backend, num_pages=600, token_budget=128, chunk_size=96, max_batch_size=16,
                               policy=policy, seed=2)
    print("policy", policy, "prompts", [r.prompt_len for r in reqs], "outputs", [r.output_len for r in reqs], flush=True)
    loop.run()
    assert len(loop.done) == len(reqs) and loop.pool.free == loop.pool.num_pages
    if policy == "stall_free":
        assert any(it.num_prefill_tokens and it.num_decodes for it in loop.iterations)
        assert all(it.num_decodes == it.num_running_decodes for it in loop.iterations)
    scale = 1.0 / np.sqrt(shape.head_dim)
    for r in loop.done:
        a, b = r.token_base, r.token_base + r.total_rows
        ref = oracle.hybrid_attention(_bits(backend.q_all[a:b]), _bits(backend.k_all[a:b]), _bits(backend.v_all[a:b]),
                                      [0], [0], [r.total_rows], [r.total_rows], scale)
        got = backend.out_all[a:b].to(torch.float64).cpu().numpy()
        compare(got, ref, "request %d (%d + %d rows) under %s" % (r.id, r.prompt_len, r.total_rows - r.prompt_len, policy))


def test_iterations_with_linear_layers_leave_attention_unchanged():
    """The backend can run the four linear layers of a transformer layer in every iteration (timing only): the
    attention rows must still match, and the iterations must take longer than without them."""
    shape = wl.AttnShape(8, 2, 128)
    reqs = serving.synthetic_trace(23, 6, 50000.0, prompt_median=150, prompt_p90=420, output_median=8, output_p90=14,
                                   max_prompt=600, max_output=16)
    times = {}
    for model in (None, "mistral-7b"):
        backend = serving.GpuBackend(seed=5, linear_model=model)
        loop = serving.ServingLoop(shape, reqs, backend, num_pages=400, token_budget=128, chunk_size=96, max_batch_size=16,
                                   policy="stall_free", seed=2)
        loop.run()
        assert len(loop.done) == len(reqs)
        times[model] = sum(it.duration_s for it in loop.iterations[2:])
        scale = 1.0 / np.sqrt(shape.head_dim)
        r = loop.done[0]
        a, b = r.token_base, r.token_base + r.total_rows
        ref = oracle.hybrid_attention(_bits(backend.q_all[a:b]), _bits(backend.k_all[a:b]), _bits(backend.v_all[a:b]),
                                      [0], [0], [r.total_rows], [r.total_rows], scale)
        compare(backend.out_all[a:b].to(torch.float64).cpu().numpy(), ref, "request %d, linear layers %s" % (r.id, model))
    print("iteration seconds without / with linear layers:", times, flush=True)
    assert times["mistral-7b"] > times[None]
