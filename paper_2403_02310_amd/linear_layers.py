"""The linear layers of one transformer layer at the shapes of the paper's four models (Table 1), per GPU of the
tensor-parallel degree the paper deploys them with, and the time-against-tokens profile of section 3.1.

Per layer (section 2.1): the fused Q/K/V projection, the output projection, the feed-forward up projection
(gate and up fused where the model has a gate) and the down projection.  Tensor parallelism (section 2.3)
splits the first of each pair by output features and the second by input features, so one GPU holds
``out_features / tp`` rows of the former and ``in_features / tp`` columns of the latter.  The models'
dimensions are their public configurations; the paper does not print them.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Sequence, Tuple


@dataclass(frozen=True)
class ModelDims:
    name: str
    hidden: int
    q_heads: int
    kv_heads: int
    head_dim: int
    ffn: int
    gated: bool     # gate and up projections (SwiGLU) or a single up projection
    tp: int         # tensor-parallel degree of the paper's deployment (Table 1)


MODELS: Dict[str, ModelDims] = {
    "mistral-7b": ModelDims("Mistral-7B", 4096, 32, 8, 128, 14336, True, 1),
    "yi-34b": ModelDims("Yi-34B", 7168, 56, 8, 128, 20480, True, 2),
    "llama2-70b": ModelDims("LLaMA2-70B", 8192, 64, 8, 128, 28672, True, 4),
    "falcon-180b": ModelDims("Falcon-180B", 14848, 232, 8, 64, 59392, False, 4),
}


def layer_shapes(m: ModelDims) -> List[Tuple[str, int, int]]:
    """(layer, out_features, in_features) of one GPU's share of one transformer layer."""
    qkv = (m.q_heads + 2 * m.kv_heads) * m.head_dim // m.tp
    attn_out_in = m.q_heads * m.head_dim // m.tp
    up = (2 if m.gated else 1) * m.ffn // m.tp
    return [("qkv", qkv, m.hidden), ("attn_out", m.hidden, attn_out_in), ("ffn_up", up, m.hidden),
            ("ffn_down", m.hidden, m.ffn // m.tp)]


def weight_bytes(shapes: Sequence[Tuple[str, int, int]]) -> int:
    return sum(2 * n * k for _, n, k in shapes)


def flops(shapes: Sequence[Tuple[str, int, int]], tokens: int) -> int:
    return sum(2 * tokens * n * k for _, n, k in shapes)


def profile(timer: Callable[[int, int, int], float], shapes: Sequence[Tuple[str, int, int]],
            token_counts: Sequence[int]) -> List[dict]:
    """Seconds of every layer for every token count: ``timer(T, N, K) -> seconds``."""
    rows = []
    for t in token_counts:
        per = {name: timer(t, n, k) for name, n, k in shapes}
        rows.append({"tokens": t, "seconds": sum(per.values()), "per_layer": per})
    return rows


def knee(rows: Sequence[dict]) -> float:
    """Token count at which the flat (weight-fetch) regime meets the linear (arithmetic) one: the time of the
    smallest batch divided by the per-token slope over the upper half of the token range (section 3.1's
    critical threshold)."""
    rows = sorted(rows, key=lambda r: r["tokens"])
    b = rows[-1]
    a = min(rows, key=lambda r: abs(r["tokens"] - b["tokens"] / 2))
    slope = (b["seconds"] - a["seconds"]) / (b["tokens"] - a["tokens"]) if b["tokens"] > a["tokens"] else 0.0
    return rows[0]["seconds"] / slope if slope > 0 else float("inf")


def gpu_timer(reps: int = 20, warmup: int = 3, min_weight_bytes: int = 640 << 20, zeros: bool = False):
    """Times sarathi_linear with HIP events; enough weight copies are rotated that a repetition never finds its
    weights in the last-level cache (a model's layers are each read once per iteration).  ``zeros``: all-zero
    operands instead of N(0,1) values (a diagnostic: the chip's clock depends on the data the matrix pipes see)."""
    import torch
    from . import binding

    def time_layer(T: int, N: int, K: int) -> float:
        copies = max(2, -(-min_weight_bytes // (2 * N * K)))
        g = torch.Generator(device="cuda").manual_seed(N * 31 + K)
        ws = [torch.randn(N, K, device="cuda", generator=g).to(torch.bfloat16) for _ in range(copies)]
        x = torch.randn(T, K, device="cuda", generator=g).to(torch.bfloat16)
        if zeros:
            for t in ws + [x]:
                t.zero_()
        y = torch.empty(T, N, device="cuda", dtype=torch.bfloat16)
        nbytes = binding.linear_workspace_bytes(T, N, K)
        scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
        for i in range(warmup):
            binding.linear(x, ws[i % copies], y, scratch)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for i in range(reps):
            binding.linear(x, ws[i % copies], y, scratch)
        ev[1].record()
        ev[1].synchronize()
        return ev[0].elapsed_time(ev[1]) * 1e-3 / reps
    return time_layer
