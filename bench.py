#!/usr/bin/env python3
"""Benchmark of one iteration's hybrid-batch attention on one MI355X.

A step = one pass of the whole hot path over one synthetic hybrid batch:
  host:   one pass of stall-free batching (Algorithm 3) producing the batch description
  device: KV append of the iteration's new rows, attention over the batch, split-KV merge
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5|c2_chunk|c2_decodes|...]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the attention kernels (fetch + write), from two `rocprofv3 --pmc` runs
# (FETCH_SIZE, WRITE_SIZE) scaled by what the same counters read on a plain copy of known size;
# the runs and the scaling are recorded in the named files under profiles/.  The figures belong to the
# recipe's own seed and the library's default options: a run with another seed, other options or other
# values reports no traffic (null) rather than somebody else's.
MEASURED_TRAFFIC_BYTES = {"c2": (606.4e6, "profiles/attention_c2_mistral_hybrid.md"),
                          "c3": (1480.8e6, "profiles/attn_wave_kernel_c3_decode_only.md"),
                          "c4": (5149.7e6, "profiles/attention_c4_yi_long.md"),
                          "c4_chunks": (345.9e6, "profiles/attn_chunk_kernel_c4_chunks.md"),
                          "c5": (9673.0e6, "profiles/attention_c5_llama70b.md")}


def measured_traffic(args):
    """(bytes, source) of the profiled launch this run repeats, or (None, reason)."""
    if args.seed is not None or args.opt or args.values != "normal":
        return None, "not measured for this seed / these options / these values"
    if args.workload not in MEASURED_TRAFFIC_BYTES:
        return None, "no counter run recorded for this workload"
    return MEASURED_TRAFFIC_BYTES[args.workload]

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
# What a decode-only launch of identical decodes streams on this part (`--workload decode_probe`, 512 blocks and more;
# profiles/decode_streaming_rate_probes.md): the ceiling of this access pattern, reported beside the published peak.
MEASURED_STREAMING_CEILING_GBS = 6650.0


def make_workload(name: str, seed=None):
    from paper_2403_02310_amd import workloads as wl
    base = name.split("_")[0]
    make = {"c1": wl.config1_tiny, "c2": wl.config2_mistral_hybrid, "c3": wl.config3_decode_only,
            "c4": wl.config4_yi_long, "c5": wl.config5_llama70b}[base]
    full = make() if seed is None else make(seed=seed)
    batch = wl.decodes_first(full)
    if name.endswith("_chunk") or name.endswith("_chunks"):
        batch = batch.sub_batch([i for i in range(batch.num_seqs) if batch.q_len[i] > 1], name)
    elif name.endswith("_decodes"):
        batch = batch.sub_batch([i for i in range(batch.num_seqs) if batch.q_len[i] == 1], name)
    desc = {
        "c1": "tiny: 64-token chunk @prefix 128 + 3 decodes (Hq4/Hkv1/d64)",
        "c2": "Mistral-7B shape (Hq32/Hkv8/d128, page 16): 512-token chunk @prefix U[0,3584] + 64 decodes ctx U[256,4096]",
        "c3": "Mistral-7B shape: 256 decodes, ctx lognormal(median 1024, sigma 0.8) in [64,8192], pages scattered over 2x100 GB pools",
        "c4": "Yi-34B shape (Hq56/Hkv8/d128): chunks 1024/512/384 @prefix U[0,12288] + 128 decodes ctx U[1024,16384]",
        "c5": "LLaMA2-70B shape (Hq64/Hkv8/d128): 2x512-token chunks @prefix U[0,3584] + 1024 decodes ctx U[512,4096]",
    }[base]
    if "_" in name:
        desc += " [" + name.split("_", 1)[1] + " only]"
    return batch, desc


def run_sweep(args, binding, harness, torch) -> int:
    """Chunk-size sweep (section 5.4's ablation shape): one 8192-token prompt at the LLaMA2-70B attention shape
    prefilled in chunks of c tokens, N = 8192/c iterations of KV append + attention; total time per c."""
    from paper_2403_02310_amd import workloads as wl
    prompt = 8192
    last = wl.config5_sweep(prompt)[-1]
    s = last.shape
    k_all, v_all = last.kv_bits(0)
    q_all = wl.normal_bf16((55, 0x51, 7), (prompt, s.num_q_heads, s.head_dim))
    q_dev, k_dev, v_dev = (harness.bits_to_device(x) for x in (q_all, k_all, v_all))
    out = torch.empty_like(q_dev)
    bt = torch.from_numpy(last.block_table).cuda()
    k_cache, v_cache = harness.make_pools(last, 0)
    handle = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=prompt, max_seqs=8,
                            max_blocks_per_seq=last.max_blocks_per_seq)
    for kv in args.opt:
        name, value = kv.split("=")
        handle.set_option(name, int(value))
    ws = handle.ensure_workspace()
    stream = torch.cuda.current_stream().cuda_stream
    lib, h = binding.lib, handle._h
    i32 = ctypes.c_int32 * 1
    row_q = s.num_q_heads * s.head_dim * 2
    row_kv = s.num_kv_heads * s.head_dim * 2
    flops = 4.0 * s.head_dim * s.num_q_heads * (prompt * (prompt + 1) / 2)
    reps = max(3, min(args.steps, 10))
    curve = {}
    sizes = [int(x) for x in args.sweep_chunks.split(",")] if args.sweep_chunks else [8192, 2048, 1024, 512, 256, 128, 64]
    for c in sizes:
        if c < 1 or prompt % c:
            raise SystemExit("bench.py: --sweep-chunks takes divisors of %d" % prompt)
        n_it = prompt // c
        qs, ql, cl = i32(0), i32(c), [i32((i + 1) * c) for i in range(n_it)]

        def one_pass():
            for i in range(n_it):
                off = i * c
                st = lib.sarathi_kv_append(h, k_dev.data_ptr() + off * row_kv, v_dev.data_ptr() + off * row_kv,
                                           k_cache.data_ptr(), v_cache.data_ptr(), bt.data_ptr(), qs, ql, cl[i], 1, c,
                                           last.num_pages, ws.data_ptr(), stream)
                if st == 0:
                    st = lib.sarathi_hybrid_attention(h, q_dev.data_ptr() + off * row_q, k_cache.data_ptr(), v_cache.data_ptr(),
                                                      bt.data_ptr(), qs, ql, cl[i], 1, c, last.num_pages,
                                                      float(last.sm_scale), out.data_ptr() + off * row_q, ws.data_ptr(), stream)
                if st != 0:
                    raise RuntimeError("sweep step failed: %s" % handle.last_error())

        one_pass()
        torch.cuda.synchronize()
        # passes run back to back (a serving loop keeps the queue fed); one bracket around all of them
        t0 = time.perf_counter()
        for _ in range(reps):
            one_pass()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / reps
        curve[str(c)] = {"iterations": n_it, "total_us": us, "mfma_frac": flops / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    if "8192" in curve:
        one_shot = curve["8192"]["total_us"]
        for v in curve.values():
            v["overhead_vs_one_shot"] = v["total_us"] / one_shot
    best = curve.get("2048") or curve[str(sizes[0])]
    print(json.dumps({
        "metric": "chunked prefill of one 8192-token prompt (KV append + attention per chunk): prompt tokens/s at chunk %s" % ("2048" if "2048" in curve else sizes[0]),
        "value": prompt / (best["total_us"] * 1e-6), "unit": "tokens/s", "n_gpus": 1, "steps": reps, "warmup": 1,
        "ms_per_step": best["total_us"] * 1e-3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c5_sweep: LLaMA2-70B shape (Hq64/Hkv8/d128), one 8192-token prompt, chunk sizes 64..2048 and one shot",
                   "algorithmic_flops": flops},
        "sweep": curve}))
    return 0


def run_serving(args) -> int:
    """Serving-loop proxy (attention only): a Poisson trace with the conversation trace's length statistics
    (Table 2) at the Mistral-7B attention shape, token budget 512, scheduled by stall-free batching and by the
    prefill-prioritising toy policy, same kernels, same trace."""
    from paper_2403_02310_amd import serving, workloads as wl
    n_req = 96
    seed = 31 if args.seed is None else args.seed
    qps = 8000.0   # attention alone is ~50x faster than a whole model's iteration: arrivals scaled to load it
    opts = {k: int(v) for k, v in (kv.split("=") for kv in args.opt)}
    def run(reqs, policy, budget=512, linear_model=None):
        pages = int(1.3 * sum((r.total_rows + 15) // 16 for r in reqs))
        loop = serving.ServingLoop(wl.MISTRAL_7B, reqs, serving.GpuBackend(seed=seed, keep_outputs=False, options=opts,
                                                                             linear_model=linear_model),
                                   num_pages=pages, token_budget=budget, chunk_size=budget, max_batch_size=128, policy=policy,
                                   seed=seed)
        return loop.run()
    run(serving.synthetic_trace(seed + 1, 6, qps, max_prompt=2048, max_output=16), "stall_free")   # warm-up: first use of every kernel
    run(serving.synthetic_trace(seed + 1, 6, qps, max_prompt=2048, max_output=16), "prefill_first")
    reqs = serving.synthetic_trace(seed, n_req, qps, max_prompt=8192, max_output=256)
    tokens = sum(r.total_rows for r in reqs)
    out = {policy: run(reqs, policy).summary() for policy in ("stall_free", "prefill_first")}
    # the same with the four linear layers of one Mistral-7B transformer layer in every iteration: a longer trace-time
    # scale (arrivals at a quarter of the rate), the operators that dominate a real iteration included
    run(serving.synthetic_trace(seed + 1, 6, qps / 4, max_prompt=2048, max_output=16), "prefill_first", linear_model="mistral-7b")
    reqs_l = serving.synthetic_trace(seed, n_req, qps / 4, max_prompt=8192, max_output=256)
    out_l = {policy: run(reqs_l, policy, linear_model="mistral-7b").summary() for policy in ("stall_free", "prefill_first")}
    sf = out["stall_free"]
    print(json.dumps({
        "metric": "serving-loop proxy (KV append + attention only): generated tokens/s under stall-free batching",
        "value": sf["generated_tokens"] / sf["makespan_s"], "unit": "tokens/s", "n_gpus": 1, "steps": sf["iterations"],
        "warmup": 0, "ms_per_step": sf["iteration_us"]["p50"] * 1e-3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "serve: %d requests, Poisson 8000/s, prompts lognormal(median 1730, p90 5696) <= 8192, outputs "
                               "lognormal(median 415, p90 834) <= 256, Mistral-7B attention shape, token budget 512" % n_req,
                   "attention_rows": tokens, "seed": seed},
        "policies": out,
        "policies_with_linear_layers": out_l}))
    return 0


def run_token_budget(args) -> int:
    """One-time profile of section 4.3: iteration time (KV append + attention only: a proxy) against the token
    budget, at the Mistral-7B attention shape with 64 running decodes, and the chunk sizes around a query-tile edge."""
    from paper_2403_02310_amd import token_budget as tb, workloads as wl
    seed = 41 if args.seed is None else args.seed
    rng = np.random.default_rng([seed, 0x7B])
    decode_ctx = rng.integers(256, 4096 + 1, size=64).tolist()
    timer = tb.gpu_timer({k: int(v) for k, v in (kv.split("=") for kv in args.opt)}, reps=max(5, min(args.steps, 30)))
    rows = tb.profile(timer, wl.MISTRAL_7B, [64, 128, 256, 512, 1024, 2048, 4096], decode_ctx, chunk_prefix=2048, seed=seed)
    targets = [150e-6, 200e-6, 300e-6, 500e-6]
    picks = {"%d us" % round(t * 1e6): tb.compute_token_budget(rows, t) for t in targets}
    quant = tb.tile_quantization_probe(timer, wl.MISTRAL_7B, prefix=2048, chunks=(223, 224, 225, 255, 256, 257, 288), seed=seed)
    t512 = [r for r in rows if r["token_budget"] == 512][0]["seconds"]
    # the same with the four linear layers of one Mistral-7B transformer layer in the iteration (section 3.1: the
    # operators that dominate it); tile quantisation now shows at the linear layers' 128/256-token tiles
    timer_l = tb.gpu_timer({k: int(v) for k, v in (kv.split("=") for kv in args.opt)}, reps=max(5, min(args.steps, 30)),
                           linear_model="mistral-7b")
    rows_l = tb.profile(timer_l, wl.MISTRAL_7B, [64, 128, 256, 512, 1024, 2048, 4096], decode_ctx, chunk_prefix=2048, seed=seed)
    targets_l = [300e-6, 500e-6, 1000e-6, 2000e-6]
    picks_l = {"%d us" % round(t * 1e6): tb.compute_token_budget(rows_l, t) for t in targets_l}
    quant_l = tb.tile_quantization_probe(timer_l, wl.MISTRAL_7B, prefix=2048, chunks=(255, 256, 257, 288, 384, 385, 512, 513), seed=seed)
    print(json.dumps({
        "metric": "token-budget profile (KV append + attention only): tokens/s of the budget-512 batch",
        "value": 512 / t512, "unit": "tokens/s", "n_gpus": 1, "steps": max(5, min(args.steps, 30)), "warmup": 3,
        "ms_per_step": t512 * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "budget: Mistral-7B attention shape, 64 decodes ctx U[256,4096] + one chunk of (budget - 64) tokens "
                               "@prefix 2048", "seed": seed},
        "profile_us": {str(r["token_budget"]): r["seconds"] * 1e6 for r in rows},
        "largest_budget_within": picks,
        "tile_quantization_us": {str(r["chunk"]): r["seconds"] * 1e6 for r in quant},
        "with_linear_layers": {"model": "mistral-7b (one transformer layer's four linear layers per iteration)",
                               "profile_us": {str(r["token_budget"]): r["seconds"] * 1e6 for r in rows_l},
                               "largest_budget_within": picks_l,
                               "tile_quantization_us": {str(r["chunk"]): r["seconds"] * 1e6 for r in quant_l}}}))
    return 0


def run_decode_probe(args) -> int:
    """What bounds the decode path, measured with the library's own kernel on synthetic decode-only batches:
    (a) N identical decodes of CTX keys (N x 8 blocks of equal length): the rate one block reaches alone, the rate per
    compute unit with one and with two blocks on it, and the chip-wide streaming ceiling;
    (b) N decodes of mixed lengths (uniform in [256, 4096] and the lognormal recipe) at one and at two blocks per
    compute unit: where starting blocks longest-first as units fall free beats having all of them resident."""
    import torch
    from paper_2403_02310_amd import binding, workloads as wl
    s = wl.MISTRAL_7B
    reps = max(10, min(args.steps, 30))

    def attention_us(b, opts):
        h = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=2048, max_seqs=max(128, b.num_seqs),
                           max_blocks_per_seq=b.max_blocks_per_seq)
        for k, v in opts.items():
            h.set_option(k, v)
        g = torch.Generator(device="cuda").manual_seed(1)
        rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=g).to(torch.bfloat16)
        pools = [(rnd(b.num_pages, s.num_kv_heads, 16, s.head_dim), rnd(b.num_pages, s.num_kv_heads, s.head_dim, 16)) for _ in range(3)]
        q = rnd(b.num_tokens, s.num_q_heads, s.head_dim)
        out = torch.empty_like(q)
        bt = torch.from_numpy(b.block_table).cuda()
        h.set_option("time_kernels", 1)
        for i in range(5 + reps):
            if i == 5:
                h.kernel_times()
            kc, vc = pools[i % 3]     # three pools in turn: no launch finds its keys in the last-level cache
            h.hybrid_attention(q, kc, vc, bt, b.q_start, b.q_len, b.ctx_len, b.sm_scale, out)
        torch.cuda.synchronize()
        kt = h.kernel_times()
        return kt.attention_ms * 1e3 / kt.attention_launches

    equal = []
    for n, ctx in ((4, 8192), (8, 8192), (16, 8192), (24, 8192), (32, 8192), (48, 8192), (64, 8192), (128, 4096), (256, 2048)):
        b = wl._make("equal", s, [1] * n, [ctx] * n, 5, slack=1.0)
        row = {"decodes": n, "ctx": ctx, "blocks": n * s.num_kv_heads}
        for name, per_cu in (("two_per_cu", 2), ("one_per_cu", 1)):
            us = attention_us(b, {"decode_blocks_per_cu": per_cu, "split_keys": 1 << 20})
            row[name] = {"us": us, "TBps": b.kv_bytes() / us / 1e6, "GBps_per_block": b.kv_bytes() / us / 1e3 / (n * s.num_kv_heads)}
        equal.append(row)
    mixed = []
    for n in (16, 32, 48, 64, 96, 128, 192, 256):
        rng = np.random.default_rng([7, n])
        for kind in ("uniform[256,4096]", "lognormal(1024,0.8)"):
            if kind.startswith("uniform"):
                ctx = rng.integers(256, 4097, size=n)
            else:
                ctx = np.clip(np.rint(np.exp(np.log(1024.0) + 0.8 * rng.standard_normal(n))), 64, 8192).astype(np.int32)
            b = wl._make("mixed", s, [1] * n, ctx, 9, slack=1.0)
            row = {"decodes": n, "lengths": kind, "MB": b.algorithmic_bytes() / 1e6}
            for name, per_cu in (("two_per_cu", 2), ("one_per_cu", 1)):
                us = attention_us(b, {"decode_blocks_per_cu": per_cu})
                row[name] = {"us": us, "hbm_frac": b.algorithmic_bytes() / us / 1e3 / HBM_PEAK_GBS}
            mixed.append(row)
    best = max(r["two_per_cu"]["TBps"] for r in equal)
    print(json.dumps({
        "metric": "decode streaming probe: highest K/V rate of equal-length decode batches", "value": best * 1e3, "unit": "GB/s",
        "n_gpus": 1, "steps": reps, "warmup": 5, "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "decode_probe: Mistral-7B attention shape, decode-only batches, compact pools, three pool copies rotated"},
        "roofline": {"bound": "hbm", "kernel": "attn_wave_kernel", "achieved": best * 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": best * 1e3 / HBM_PEAK_GBS, "traffic": None},
        "equal_length": equal, "mixed_length": mixed}))
    return 0


def run_linear(args) -> int:
    """Linear layers of one transformer layer against the number of tokens in the batch (section 3.1): the four
    models of Table 1, one GPU's share under the paper's tensor-parallel degree."""
    from paper_2403_02310_amd import linear_layers as ll
    tokens = [16, 64, 128, 256, 384, 512, 768, 1024, 1536, 2048]
    timer = ll.gpu_timer(reps=max(5, min(args.steps, 20)), zeros=args.values == "zeros")
    out = {}
    for key, m in ll.MODELS.items():
        shapes = ll.layer_shapes(m)
        rows = ll.profile(timer, shapes, tokens)
        wb = ll.weight_bytes(shapes)
        out[key] = {"model": m.name, "tp": m.tp, "layers": {n: [o, i] for n, o, i in shapes}, "weight_bytes": wb,
                    "us": {str(r["tokens"]): r["seconds"] * 1e6 for r in rows},
                    "weights_GBps": {str(r["tokens"]): wb / r["seconds"] / 1e9 for r in rows},
                    "TFLOPs": {str(r["tokens"]): ll.flops(shapes, r["tokens"]) / r["seconds"] / 1e12 for r in rows},
                    "per_layer_us": {str(r["tokens"]): {n: v * 1e6 for n, v in r["per_layer"].items()} for r in rows
                                     if r["tokens"] in (16, 128, 512, 2048)},
                    "knee_tokens": ll.knee(rows)}
    head = out["llama2-70b"]
    t2048 = head["us"]["2048"] * 1e-6
    ach = head["TFLOPs"]["2048"]
    result = {
        "metric": "linear layers of one transformer layer, tokens/s at 2048 tokens (LLaMA2-70B, one GPU of TP4)",
        "value": 2048 / t2048, "unit": "tokens/s", "n_gpus": 1, "steps": max(5, min(args.steps, 20)), "warmup": 3,
        "ms_per_step": t2048 * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic" if args.values == "normal" else "synthetic, ALL-ZERO values (clock diagnostic, not a reported figure)",
        "config": {"workload": "linear: QKV, attention-output, feed-forward up and down projections of the four models of "
                               "Table 1 at one GPU's tensor-parallel share, 16 ... 2048 tokens, N(0,1) values"},
        "roofline": {"bound": "mfma", "kernel": "linear_kernel", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
        "small_batch_roofline": {"bound": "hbm", "tokens": 128, "achieved": head["weights_GBps"]["128"], "peak": HBM_PEAK_GBS,
                                 "unit": "GB/s", "frac": head["weights_GBps"]["128"] / HBM_PEAK_GBS},
        "models": out}
    if not args.no_cpu_baseline:
        import oracle
        from paper_2403_02310_amd import workloads as wl
        # the fp64 checker on a bounded sample: 64 token rows of LLaMA2-70B's feed-forward down projection
        _, n, k = ll.layer_shapes(ll.MODELS["llama2-70b"])[3]
        xb = wl.normal_bf16((77, 0x58), (64, k)); wb_ = wl.normal_bf16((77, 0x57), (n, k))
        tc = time.perf_counter()
        oracle.linear(xb, wb_)
        dt = time.perf_counter() - tc
        per_token = dt / 64 * (ll.flops(ll.layer_shapes(ll.MODELS["llama2-70b"]), 1) / (2.0 * n * k))
        result["cpu_baseline"] = {"value": 1.0 / per_token, "unit": "tokens/s", "cores": oracle.max_threads(), "kind": "oracle",
                                  "seconds": dt, "sample": "64 token rows of the feed-forward down projection (8192 x 7168), "
                                  "scaled by flops to the four layers"}
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2",
                    help="c2 (default), c3, c4, c5, <cN>_chunks, <cN>_decodes, c5_sweep (one 8192-token prompt prefilled in "
                         "chunks of 64 ... 2048 and in one shot), serve (serving loop over a request trace), budget "
                         "(token-budget profile), linear (linear layers against the number of tokens), decode_probe (what bounds the decode "
                         "path: equal-length and mixed-length decode batches at one and two blocks per compute unit)")
    ap.add_argument("--seed", type=int, default=None, help="seed of the workload recipe (default: the recipe's own)")
    ap.add_argument("--copies", type=int, default=0, help="independent KV-pool/Q copies rotated between steps (0 = auto)")
    ap.add_argument("--values", choices=["normal", "zeros"], default="normal",
                    help="normal: the workloads' N(0,1) values (every reported figure); zeros: all-zero Q/K/V or x/w, a "
                         "diagnostic that shows how far the chip's clock, which falls with the matrix pipes' switching "
                         "power, moves the MFMA-bound kernels (no parity check, no CPU baseline)")
    ap.add_argument("--sweep-chunks", default="", help="c5_sweep only: comma-separated chunk sizes (default: 8192,2048,...,64)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--opt", action="append", default=[], help="library tuning knob name=value (repeatable)")
    args = ap.parse_args()
    if args.values == "zeros":
        args.no_cpu_baseline = True  # the checker's inputs are the workload's own values
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                         "run with --gpus 1\n")
        return 2

    import torch
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        return 3
    torch.cuda.set_device(0)
    from paper_2403_02310_amd import binding, harness

    if args.values == "zeros" and args.workload in ("c5_sweep", "serve", "budget", "decode_probe"):
        sys.stderr.write("bench.py: --values zeros applies to the single-batch workloads and to --workload linear\n")
        return 2
    if args.workload == "c5_sweep":
        return run_sweep(args, binding, harness, torch)
    if args.workload == "serve":
        return run_serving(args)
    if args.workload == "budget":
        return run_token_budget(args)
    if args.workload == "linear":
        return run_linear(args)
    if args.workload == "decode_probe":
        return run_decode_probe(args)
    batch, desc = make_workload(args.workload, args.seed)
    s = batch.shape
    T, S = batch.num_tokens, batch.num_seqs
    kv_bytes_per_copy = 2 * batch.num_pages * s.num_kv_heads * s.page_size * s.head_dim * 2
    copies = args.copies or int(max(1, min(4, (24 << 30) // max(1, kv_bytes_per_copy))))

    # ---- resident inputs --------------------------------------------------------------
    t_setup = time.time()
    fill_handle = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=32768, max_seqs=2048,
                                 max_blocks_per_seq=batch.max_blocks_per_seq)
    kv_host: dict = {}
    for i, kv in enumerate(batch.kv_bits_many(range(S), workers=16)):
        kv_host[i] = kv
    bt_dev = torch.from_numpy(batch.block_table).cuda()
    pools = []
    k0, v0 = harness.make_pools(batch, poison=None)
    harness.fill_prefixes(fill_handle, batch, k0, v0, bt_dev, kv_host, upto="all")
    pools.append((k0, v0))
    for _ in range(copies - 1):
        pools.append((k0.clone(), v0.clone()))
    k_new_bits, v_new_bits = harness.new_token_kv(batch, kv_host)
    k_new, v_new = harness.bits_to_device(k_new_bits), harness.bits_to_device(v_new_bits)
    qs = [harness.bits_to_device(batch.q_bits(c)) for c in range(copies)]
    outs = [torch.empty_like(qs[0]) for _ in range(copies)]
    if args.values == "zeros":
        for t in [k_new, v_new] + qs + [x for kv in pools for x in kv]:
            t.zero_()
    del fill_handle
    torch.cuda.synchronize()

    handle = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=max(T, 2048),
                            max_seqs=max(S, 128), max_blocks_per_seq=batch.max_blocks_per_seq)
    for kv in args.opt:
        name, value = kv.split("=")
        handle.set_option(name, int(value))
    ws = handle.ensure_workspace()
    stream = torch.cuda.current_stream().cuda_stream

    # ---- scheduler state that yields exactly this batch (decodes first, then the chunks) ----
    dec = [i for i in range(S) if batch.q_len[i] == 1]
    pre = [i for i in range(S) if batch.q_len[i] > 1]
    mk = lambda lst: (binding.Request * max(1, len(lst)))(*lst)
    running_decodes = mk([binding.Request(i, int(batch.ctx_len[i]) - 1, int(batch.ctx_len[i]) - 1, 0, 0) for i in dec])
    running_prefills = mk([binding.Request(i, int(batch.ctx_len[i]), int(batch.prefix_len[i]), 0, 0) for i in pre])
    token_budget = T
    chunk_size = int(max([batch.q_len[i] for i in pre], default=1))
    cap = max(S, 1)
    sb_id = np.zeros(cap, np.int64); sb_qs = np.zeros(cap, np.int32); sb_ql = np.zeros(cap, np.int32); sb_cl = np.zeros(cap, np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    sched_out = binding.Batch()
    sched_out.seq_id = sb_id.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    sched_out.q_start, sched_out.q_len, sched_out.ctx_len = (a.ctypes.data_as(i32p) for a in (sb_qs, sb_ql, sb_cl))
    p_qs, p_ql, p_cl = sched_out.q_start, sched_out.q_len, sched_out.ctx_len
    lib = binding.lib
    h = handle._h
    bt_ptr, ws_ptr = bt_dev.data_ptr(), ws.data_ptr()
    k_new_ptr, v_new_ptr = k_new.data_ptr(), v_new.data_ptr()
    pool_ptrs = [(k.data_ptr(), v.data_ptr()) for (k, v) in pools]
    q_ptrs = [q.data_ptr() for q in qs]
    out_ptrs = [o.data_ptr() for o in outs]
    num_pages = batch.num_pages
    sm_scale = float(batch.sm_scale)
    n_dec, n_pre = len(dec), len(pre)

    def step(i: int) -> None:
        st = lib.sarathi_build_stall_free_batch(token_budget, chunk_size, running_decodes, n_dec, running_prefills,
                                                n_pre, None, 0, 0, s.page_size, cap, ctypes.byref(sched_out))
        if st != 0:
            raise RuntimeError("scheduler failed: %d" % st)
        c = i % copies
        kp, vp = pool_ptrs[c]
        st = lib.sarathi_kv_append(h, k_new_ptr, v_new_ptr, kp, vp, bt_ptr, p_qs, p_ql, p_cl, sched_out.num_seqs,
                                   sched_out.num_tokens, num_pages, ws_ptr, stream)
        if st != 0:
            raise RuntimeError("kv_append failed: %s" % handle.last_error())
        st = lib.sarathi_hybrid_attention(h, q_ptrs[c], kp, vp, bt_ptr, p_qs, p_ql, p_cl, sched_out.num_seqs,
                                          sched_out.num_tokens, num_pages, sm_scale, out_ptrs[c], ws_ptr, stream)
        if st != 0:
            raise RuntimeError("hybrid_attention failed: %s" % handle.last_error())

    # the scheduler must reproduce the workload's description exactly
    step(0)
    torch.cuda.synchronize()
    assert sched_out.num_seqs == S and sched_out.num_tokens == T
    assert (sb_ql[:S] == batch.q_len).all() and (sb_cl[:S] == batch.ctx_len).all() and (sb_qs[:S] == batch.q_start).all()
    setup_s = time.time() - t_setup

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # the attention kernel's duration is measured live by HIP events around every TIME_EVERY-th launch of the
    # timed steps (an event record between two kernels holds the second back for ~6 us, so bracketing every
    # launch would slow the very steps that are being timed by ~4 %)
    TIME_EVERY = 8 if args.steps >= 64 else 1
    if not args.no_kernel_timing:
        handle.set_option("time_kernels", 1)
        handle.set_option("time_every", TIME_EVERY)
        handle.kernel_times()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kt = handle.kernel_times() if not args.no_kernel_timing else None
    # the other kernels' durations come from a short pass of their own, outside the timed region
    # (every pair of events costs queue time, so the timed region brackets the attention launch only)
    kt_all = None
    if not args.no_kernel_timing:
        handle.set_option("time_kernels", 2)
        handle.set_option("time_every", 1)
        for i in range(min(args.steps, 50)):
            step(i)
        torch.cuda.synchronize()
        kt_all = handle.kernel_times()
    handle.set_option("time_kernels", 0)

    # host-only cost of a step's CPU side (scheduler + planning), measured separately
    t2 = time.perf_counter()
    for i in range(50):
        lib.sarathi_build_stall_free_batch(token_budget, chunk_size, running_decodes, n_dec, running_prefills, n_pre,
                                           None, 0, 0, s.page_size, cap, ctypes.byref(sched_out))
        info = binding.PlanInfo()
        lib.sarathi_plan_hybrid_attention(h, p_qs, p_ql, p_cl, S, T, ctypes.byref(info), None, 0)
    host_us = (time.perf_counter() - t2) * 1e6 / 50

    alg_bytes = batch.algorithmic_bytes()
    alg_flops = batch.algorithmic_flops()
    result = {
        "metric": "hybrid-batch attention tokens/s (one iteration: stall-free batch build + KV append + paged GQA attention)",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "iter_us": ms_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic" if args.values == "normal" else "synthetic, ALL-ZERO values (clock diagnostic, not a reported figure)",
        "config": {"workload": args.workload + ": " + desc, "num_tokens": T, "num_seqs": S,
                   "sum_ctx_len": int(batch.ctx_len.astype(np.int64).sum()), "seed": batch.seed,
                   "kv_copies_rotated": copies, "plan": {"units": info.num_items, "chunk_tile_units": info.num_tile_items,
                                                         "split_tiles": info.num_reduce_items, "split_keys": info.split_keys,
                                                         "tile_split_keys": info.tile_split_keys}},
        "kv_tokens_per_s": float(batch.ctx_len.astype(np.int64).sum()) / (ms_per_step * 1e-3),
        "algorithmic_bytes": alg_bytes,
        "algorithmic_flops": alg_flops,
        "whole_step": {"GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9, "hbm_frac": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "TFLOPs": alg_flops / (ms_per_step * 1e-3) / 1e12,
                       "mfma_frac": alg_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "host_us_per_step": host_us,
        "setup_s": setup_s,
    }
    if kt is not None and kt.attention_launches > 0:
        attn_us = kt.attention_ms * 1e3 / kt.attention_launches
        result["kernel_us"] = {
            "attention": attn_us,
            "merge": (kt_all.merge_ms * 1e3 / kt_all.merge_launches) if kt_all.merge_launches else 0.0,
            "kv_append": (kt_all.append_ms * 1e3 / kt_all.append_launches) if kt_all.append_launches else 0.0,
            "launches": int(kt.attention_launches),
            "note": "attention: HIP events around every %d-th launch of the timed steps; merge (the part on the caller's "
                    "stream) and kv_append: a separate pass of up to 50 steps" % TIME_EVERY}
        mfma_bound = args.workload.endswith("_chunk") or args.workload.endswith("_chunks")
        # the launch the events bracket: one kernel holding both kinds of block when the batch has both
        has_chunk, has_wave = info.num_tile_items > 0, info.num_items > info.num_tile_items
        attn_kernel = ("attn_hybrid_kernel (chunk-tile and wave-tile blocks in one launch)" if has_chunk and has_wave
                       else "attn_chunk_kernel" if has_chunk else "attn_wave_kernel")
        # The rows whose bytes and flops are counted are complete only after the merge of the tiles that were cut
        # (when there are any): the figure is over the attention launch plus that merge.
        merge_us = result["kernel_us"]["merge"]
        kern_us = attn_us + merge_us
        if merge_us > 0:
            attn_kernel += " + splitkv_reduce_kernel"
        traffic, traffic_src = measured_traffic(args)
        if mfma_bound:
            ach = alg_flops / (kern_us * 1e-6) / 1e12
            result["roofline"] = {"bound": "mfma", "kernel": attn_kernel, "achieved": ach,
                                  "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                                  "traffic": traffic, "traffic_source": traffic_src, "duration_us": kern_us}
        else:
            ach = alg_bytes / (kern_us * 1e-6) / 1e9
            result["roofline"] = {"bound": "hbm", "kernel": attn_kernel, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                                  "traffic": traffic, "traffic_source": traffic_src, "duration_us": kern_us,
                                  "measured_streaming_ceiling": {"GBps": MEASURED_STREAMING_CEILING_GBS, "frac": ach / MEASURED_STREAMING_CEILING_GBS,
                                                                 "source": "profiles/decode_streaming_rate_probes.md"}}

    # ---- CPU baseline: the fp64 checker as it stands, on the host cores, bounded sample ----
    if not args.no_cpu_baseline:
        import oracle
        k_all = np.concatenate([kv_host[i][0] for i in range(S)]); v_all = np.concatenate([kv_host[i][1] for i in range(S)])
        # aim for ~10-30 s of CPU work: whole batch if small, else a strided sample of batch rows
        pairs = batch.score_pairs() * s.num_q_heads
        stride = max(1, int(np.ceil(pairs / 6.0e9)))
        toks = list(range(0, T, stride))
        c = (args.steps - 1) % copies
        tc = time.perf_counter()
        ref = oracle.hybrid_attention(batch.q_bits(c), k_all, v_all, batch.kv_start, batch.q_start, batch.q_len,
                                      batch.ctx_len, batch.sm_scale, tokens=toks)
        cpu_s = time.perf_counter() - tc
        got = harness.bf16_tensor_to_f64(outs[c])[toks]
        err = np.abs(got - ref)
        rel = np.linalg.norm(got - ref, axis=-1) / np.linalg.norm(ref, axis=-1)
        result["cpu_baseline"] = {"value": len(toks) / cpu_s, "unit": "tokens/s", "cores": oracle.max_threads(),
                                  "kind": "oracle", "seconds": cpu_s,
                                  "sample": "every %d-th batch row (%d of %d tokens), all heads" % (stride, len(toks), T)}
        result["parity_vs_oracle"] = {"max_abs_err": float(err.max()), "max_row_rel_err": float(rel.max()),
                                      "rows_checked": len(toks)}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
