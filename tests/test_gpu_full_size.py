"""GPU parity at the full sizes of the workload recipes, in the launch configuration bench.py times
(decodes first, default planner options): EVERY row and head of every batch is compared with one pass
of the fp64 checker over the same inputs (no sampling: the checker needs 1 - 40 s per workload on the
box's host cores).  The chunk-size sweep runs every chunk size the recipe names and one shot against a
single checker result, and also checks that the paged cache bytes do not depend on the chunk size.
"""
import time

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2403_02310_amd import workloads as wl
from tests.parity import compare

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2403_02310_amd import harness
    return harness


def oracle_all_rows(batch, kv_host, q_bits, window=0):
    """fp64 result for every row of the batch (one pass of the checker over contiguous per-sequence K/V)."""
    k = np.concatenate([kv_host[s][0] for s in range(batch.num_seqs)])
    v = np.concatenate([kv_host[s][1] for s in range(batch.num_seqs)])
    return oracle.hybrid_attention(q_bits, k, v, batch.kv_start, batch.q_start, batch.q_len, batch.ctx_len, batch.sm_scale,
                                   window=window)


def run_and_check(hx, batch, window=0):
    print("case", batch.name, "T", batch.num_tokens, "S", batch.num_seqs, "sum ctx", int(batch.ctx_len.sum()), "window", window, flush=True)
    handle = None
    if window:
        handle = hx.make_handle(batch)
        handle.set_option("window", window)
    st = hx.setup_and_run(batch, poison=None, handle=handle)
    got = hx.bf16_tensor_to_f64(st["out"])
    t0 = time.time()
    ref = oracle_all_rows(batch, st["kv_host"], batch.q_bits(0), window)
    res = compare(got, ref, batch.name)
    print("   rows checked %d of %d (checker %.1f s): max abs %.3e max row rel %.3e"
          % (ref.shape[0], batch.num_tokens, time.time() - t0, res[0], res[1]), flush=True)
    return st


def test_config2_mistral_hybrid_all_rows(hx):
    batch = wl.decodes_first(wl.config2_mistral_hybrid())
    run_and_check(hx, batch)


def test_config2_algorithm3_variant_448_plus_64(hx):
    """Token budget 512 read through Algorithm 3: 64 decodes leave a 448-token chunk."""
    run_and_check(hx, wl.decodes_first(wl.config2_mistral_hybrid(chunk=448)))


def test_config3_decode_only_scattered_pool(hx):
    """256 decodes whose pages are scattered over the largest pool the box can give (up to 2 x 100 GB)."""
    free, _ = torch.cuda.mem_get_info()
    per_cache = min(100e9, 0.42 * free)
    batch = wl.config3_decode_only(pool_bytes_per_cache=per_cache)
    print("pool pages", batch.num_pages, "bytes per cache %.1f GB" % (batch.num_pages * 32768 / 1e9), flush=True)
    assert int(batch.block_table.max()) > 0.9 * batch.num_pages      # pages really span the pool
    st = run_and_check(hx, batch)
    del st
    torch.cuda.empty_cache()


def test_config2_mistral_hybrid_sliding_window(hx):
    """The Mistral-shape hybrid batch under sliding windows of 4096 (Mistral's own: contexts reach 4096, so only the
    longest rows lose keys), 1024 and 100 keys."""
    for window in (4096, 1024, 100):
        run_and_check(hx, wl.decodes_first(wl.config2_mistral_hybrid()), window=window)


def test_config4_yi_long_sliding_window(hx):
    """Long contexts (to 16384) under a 4096-key window: chunks and decodes start their key ranges mid-sequence,
    with the run-time role assignment of the hybrid launch."""
    run_and_check(hx, wl.decodes_first(wl.config4_yi_long()), window=4096)
    torch.cuda.empty_cache()


def test_config4_yi_long(hx):
    run_and_check(hx, wl.decodes_first(wl.config4_yi_long()))
    torch.cuda.empty_cache()


def test_config5_llama70b(hx):
    run_and_check(hx, wl.decodes_first(wl.config5_llama70b()))
    torch.cuda.empty_cache()


def test_config5_chunk_size_sweep(hx):
    """One 8192-token prompt prefilled in chunks of 64, 128, 256, 512, 1024 and 2048 tokens and in one shot:
    every run matches the single fp64 result on ALL 8192 rows, and all runs leave identical cache bytes
    (chunking changes nothing in what is computed, sections 4.1 and 4.3)."""
    prompt = 8192
    first = wl.config5_sweep(prompt)[-1]
    k_all, v_all = first.kv_bits(0)
    q_all = wl.normal_bf16((55, 0x51, 7), (prompt, first.shape.num_q_heads, first.shape.head_dim))
    t0 = time.time()
    ref = oracle.hybrid_attention(q_all, k_all, v_all, [0], [0], [prompt], [prompt], first.sm_scale)
    print("checker: all %d rows once, %.1f s" % (prompt, time.time() - t0), flush=True)
    q_dev, k_dev, v_dev = hx.bits_to_device(q_all), hx.bits_to_device(k_all), hx.bits_to_device(v_all)
    bt = torch.from_numpy(first.block_table).cuda()
    pools = None
    for chunk in (8192, 2048, 1024, 512, 256, 128, 64):
        iters = wl.config5_sweep(chunk)
        last = iters[-1]
        handle = hx.make_handle(last, max_tokens=prompt)
        k_cache, v_cache = hx.make_pools(last, 0)
        out = torch.empty_like(q_dev)
        print("chunk", chunk, "iterations", len(iters), flush=True)
        for it in iters:
            n, ctx = int(it.q_len[0]), int(it.ctx_len[0])
            hx.run_iteration(handle, it, k_cache, v_cache, bt, q_dev[ctx - n: ctx], k_dev[ctx - n: ctx], v_dev[ctx - n: ctx],
                             out[ctx - n: ctx])
        torch.cuda.synchronize()
        res = compare(hx.bf16_tensor_to_f64(out), ref, "sweep chunk %d" % chunk)
        print("   rows checked %d of %d: max abs %.3e max row rel %.3e" % (prompt, prompt, res[0], res[1]), flush=True)
        if pools is None:
            pools = (k_cache.clone(), v_cache.clone())
        else:
            assert torch.equal(k_cache.view(torch.int16), pools[0].view(torch.int16))
            assert torch.equal(v_cache.view(torch.int16), pools[1].view(torch.int16))
