"""GPU parity of the linear layer (sarathi_linear) against the fp64 checker, element by element.

Tolerance (bf16 inputs, fp32 products and sums, ONE rounding to bf16 at the end): the rounding is at
most 2^-9 relative; fp32 accumulation of K terms of size ~|x||w| adds at most ~K * 2^-24 times the sum
of the absolute products, in practice far less.  A result passes when every element satisfies
|got - ref| <= 2^-8 * |ref| + 2^-20 * sum_k |x w|   and every token row is within 2^-8 relative in the 2-norm.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2403_02310_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2403_02310_amd import binding, harness
    return binding, harness


def bits_to_f64(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check(got, ref, x_bits, w_bits, rows, cols, what):
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref)
    mag = np.abs(bits_to_f64(x_bits[rows])) @ np.abs(bits_to_f64(w_bits[cols])).T
    bound = 2.0 ** -8 * np.abs(ref) + 2.0 ** -20 * mag
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "%s: |err| %.3e > bound %.3e at %s" % (what, err[worst], bound[worst], worst)
    rel = np.linalg.norm(got - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
    assert rel.max() <= 2.0 ** -8, "%s: row rel %.3e" % (what, rel.max())
    return float(rel.max())


def run(hx, T, N, K, seed, workspace="full", rows=None, cols=None, x_bits=None, w_bits=None):
    binding, harness = hx
    print("linear case T", T, "N", N, "K", K, "seed", seed, "workspace", workspace, flush=True)
    x_bits = wl.normal_bf16((seed, 0x58), (T, K)) if x_bits is None else x_bits
    w_bits = wl.normal_bf16((seed, 0x57), (N, K)) if w_bits is None else w_bits
    x = harness.bits_to_device(x_bits); w = harness.bits_to_device(w_bits)
    y = torch.full((T, N), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = None
    if workspace != "none":
        nbytes = binding.linear_workspace_bytes(T, N, K)
        if workspace == "half":
            nbytes //= 2
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    binding.linear(x, w, y, ws)
    torch.cuda.synchronize()
    got = harness.bf16_tensor_to_f64(y)
    rows = list(range(T)) if rows is None else rows
    cols = list(range(N)) if cols is None else cols
    ref = oracle.linear(x_bits, w_bits, rows=rows, cols=cols)
    rel = check(got[np.ix_(rows, cols)], ref, x_bits, w_bits, rows, cols, "T%d N%d K%d" % (T, N, K))
    print("   max row rel %.3e" % rel, flush=True)
    return got


@pytest.mark.parametrize("T,N,K", [(128, 128, 64), (1, 128, 64), (77, 256, 192), (129, 384, 320), (300, 1152, 1024),
                                   (64, 128, 4096), (257, 1280, 64), (16, 512, 1024), (33, 384, 256), (100, 640, 512)])
def test_linear_matches_checker(hx, T, N, K):
    """Several token tiles, a ragged last one, several feature tiles (more and fewer than the XCD count), one and many stages."""
    run(hx, T, N, K, seed=T + N + K)


@pytest.mark.parametrize("workspace", ["full", "half", "none"])
def test_split_k_pieces_agree(hx, workspace):
    """A small batch on a long k range is cut into pieces; with less or no workspace fewer or none: same result to rounding."""
    binding, _ = hx
    T, N, K = 48, 256, 8192
    assert binding.linear_workspace_bytes(T, N, K) > 0
    run(hx, T, N, K, seed=5, workspace=workspace)


def test_result_does_not_depend_on_timing(hx):
    T, N, K = 96, 512, 4096
    a = run(hx, T, N, K, seed=9)
    b = run(hx, T, N, K, seed=9)
    assert np.array_equal(a, b)


def test_exact_on_small_integers(hx):
    """Integer inputs whose sums stay below 2^8 are exact in bf16: the GPU result must equal the checker bit for bit."""
    rng = np.random.default_rng(3)
    T, N, K = 40, 128, 64
    xi = rng.integers(-1, 2, size=(T, K)).astype(np.float32); wi = rng.integers(-1, 2, size=(N, K)).astype(np.float32)
    got = run(hx, T, N, K, seed=0, x_bits=wl.f32_to_bf16_bits(xi), w_bits=wl.f32_to_bf16_bits(wi))
    assert np.array_equal(got, xi.astype(np.float64) @ wi.astype(np.float64).T)


def test_no_tokens_is_a_no_op_and_bad_shapes_are_refused(hx):
    binding, _ = hx
    x = torch.zeros((0, 64), device="cuda", dtype=torch.bfloat16); w = torch.zeros((128, 64), device="cuda", dtype=torch.bfloat16)
    binding.linear(x, w, torch.zeros((0, 128), device="cuda", dtype=torch.bfloat16))
    for (T, N, K) in [(4, 100, 64), (4, 128, 96)]:
        with pytest.raises(binding.SarathiError) as e:
            binding.linear(torch.zeros((T, K), device="cuda", dtype=torch.bfloat16), torch.zeros((N, K), device="cuda", dtype=torch.bfloat16),
                           torch.zeros((T, N), device="cuda", dtype=torch.bfloat16))
        assert e.value.status == binding.ESHAPE


def test_model_shapes_sampled(hx):
    """The layer shapes bench.py times (Mistral-7B feed-forward up/gate and down projections) at two token counts,
    on sampled rows and columns."""
    rng = np.random.default_rng(17)
    # ... and Falcon-180B's QKV (a feature count that is not a multiple of the 256-feature tile) and attention
    # output projection (58 stages of 64 k) under TP4, LLaMA2-70B's QKV under TP4 at a decode-sized batch
    # ... and two decode-sized batches on wide matrices, which take the 128 x 64 tile (enough workgroups without
    # cutting k): Mistral-7B's feed-forward up projection, and a ragged 33-token batch on a shorter k
    for (T, N, K) in [(128, 28672, 4096), (2048, 4096, 14336), (640, 6144, 4096), (200, 3968, 14848), (2048, 14848, 3712),
                      (48, 2560, 8192), (16, 28672, 4096), (33, 28672, 512)]:
        rows = sorted(set([0, T - 1, 127 % T, 128 % T] + rng.integers(0, T, 12).tolist()))
        cols = sorted(set([0, N - 1, 127, 128, 1023, 1024] + rng.integers(0, N, 40).tolist()))
        run(hx, T, N, K, seed=21, rows=rows, cols=cols)
