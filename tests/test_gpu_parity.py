"""GPU parity: the HIP path (through the C ABI) against the fp64 checker, element by element."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import kv_cache_reference as kvref
from paper_2403_02310_amd import workloads as wl
from tests.parity import compare

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2403_02310_amd import harness
    return harness


def _expected_pools(batch, poison):
    s = batch.shape
    kc, vc = kvref.empty_pools(batch.num_pages, s.num_kv_heads, s.head_dim, s.page_size, fill=poison)
    for i in range(batch.num_seqs):
        k, v = batch.kv_bits(i)
        n = int(batch.ctx_len[i])
        kvref.kv_append(kc, vc, k, v, batch.block_table[i:i + 1], [0], [n], [n])
    return kc, vc


def _check_batch(hx, batch, poison=0x7FC1, check_pools=True):
    print("case", batch.name, "seed", batch.seed, "q_len", batch.q_len[:8], "ctx", batch.ctx_len[:8], flush=True)
    st = hx.setup_and_run(batch, poison)
    got = hx.bf16_tensor_to_f64(st["out"])
    ref = oracle.attention_for_batch(batch)
    res = compare(got, ref, batch.name)
    if check_pools:
        kc, vc = _expected_pools(batch, poison)
        np.testing.assert_array_equal(hx.device_to_bits(st["k_cache"]), kc)
        np.testing.assert_array_equal(hx.device_to_bits(st["v_cache"]), vc)
    return st, got, ref, res


def test_config1_tiny(hx):
    _check_batch(hx, wl.config1_tiny())


@pytest.mark.parametrize("poison", [0x7FC1, 0x7F80, 0xFF80, 0x0000])
def test_config1_poisoned_pool_does_not_leak(hx, poison):
    """Unused pages and slots past ctx_len hold NaN / +-inf: outputs stay finite and equal."""
    _, got, _, _ = _check_batch(hx, wl.config1_tiny(), poison)
    base = hx.bf16_tensor_to_f64(hx.setup_and_run(wl.config1_tiny(), 0x0000)["out"])
    np.testing.assert_array_equal(got, base)


SHAPES = {
    "mqa4_d64": wl.AttnShape(4, 1, 64),
    "gqa4_d128": wl.AttnShape(8, 2, 128),
    "gqa7_d128": wl.AttnShape(14, 2, 128),
    "gqa8_d128": wl.AttnShape(16, 2, 128),
    "mha_d64": wl.AttnShape(3, 3, 64),
    "mqa20_d128": wl.AttnShape(20, 1, 128),
}


@pytest.mark.parametrize("shape", sorted(SHAPES))
@pytest.mark.parametrize("seed", [101, 102])
def test_random_ragged_hybrid(hx, shape, seed):
    """Odd chunk sizes, mid-page prefixes, 1-token contexts, shuffled sequence order."""
    b = wl.random_hybrid(seed, SHAPES[shape], n_chunks=3, n_decodes=6, max_chunk=90, max_ctx=420)
    _check_batch(hx, b)


def test_edge_lengths(hx):
    """Contexts of 1, 15, 16, 17, 31, 32, 33 as decodes and as whole prefills (prefix 0)."""
    s = wl.AttnShape(8, 2, 128)
    lens = [1, 15, 16, 17, 31, 32, 33, 64, 65]
    q_len = [1] * len(lens) + lens
    ctx = lens + lens
    b = wl._make("edges", s, q_len, ctx, 77)
    _check_batch(hx, b)


def test_long_decode_uses_splits_and_matches(hx):
    """Decodes of very different lengths: by default each is one block whose four wavefronts quarter the keys and
    merge in LDS; a decode beyond 6144 keys, and any decode under a forced small split size, is also split across
    blocks (partial rows + merge kernel)."""
    s = wl.AttnShape(8, 2, 128)
    b = wl._make("long_decode", s, [1, 1, 1, 5, 1], [3000, 40, 777, 1500, 7000], 78)
    st, got, ref, _ = _check_batch(hx, b, check_pools=False)
    info, items = st["handle"].plan(b.q_start, b.q_len, b.ctx_len)
    assert info.num_reduce_items == 1                     # only the 7000-key decode
    assert sum(1 for it in items if it.seq == 0) == 1     # the 3000-key decode: one block, no partial rows
    h2 = hx.make_handle(b)
    h2.set_option("split_keys", 64)
    st2 = hx.setup_and_run(b, 0x7FC1, handle=h2)
    info2, _ = h2.plan(b.q_start, b.q_len, b.ctx_len)
    assert info2.num_reduce_items >= 4
    got2 = hx.bf16_tensor_to_f64(st2["out"])
    compare(got2, ref, "split64")
    h3 = hx.make_handle(b)
    h3.set_option("split_keys", 1 << 20)   # never split across blocks
    st3 = hx.setup_and_run(b, 0x7FC1, handle=h3)
    compare(hx.bf16_tensor_to_f64(st3["out"]), ref, "nosplit")


@pytest.mark.parametrize("shape", ["gqa7_d128", "gqa4_d128", "mqa4_d64"])
def test_chunk_tiles_with_forced_splits_and_both_paths(hx, shape):
    """A 300-row chunk on a 1000-token prefix + decodes: default plan, chunk tiles split every 64 keys,
    everything through chunk tiles, everything through wave tiles, and the three ways of launching the two
    kinds of tile (in sequence, on two streams, in one launch) -- all within tolerance of the checker."""
    s = SHAPES[shape]
    b = wl._make("chunk300_" + shape, s, [300, 1, 37, 1], [1300, 555, 37, 1], 79)
    st, got, ref, _ = _check_batch(hx, b, check_pools=False)
    info, items = st["handle"].plan(b.q_start, b.q_len, b.ctx_len)
    assert info.num_tile_items > 0 and info.num_items > info.num_tile_items
    for opts in ({"tile_split_keys": 64, "split_keys": 32}, {"tile_min_cols": 1}, {"tile_min_cols": 1 << 20},
                 {"interleave": 0, "tile_split_keys": 128}, {"interleave": 1, "tile_split_keys": 128},
                 {"interleave": 2, "tile_split_keys": 128}, {"interleave": 2, "resident_chunks": 1, "tile_split_keys": 128},
                 {"interleave": 2, "resident_chunks": 1}):
        h = hx.make_handle(b)
        for k, v in opts.items():
            h.set_option(k, v)
        print("options", opts, flush=True)
        out = hx.bf16_tensor_to_f64(hx.setup_and_run(b, 0x7FC1, handle=h)["out"])
        compare(out, ref, str(opts))


def test_small_decode_batches_at_one_and_two_blocks_per_unit(hx):
    """Launches that hold decodes only run one block per compute unit up to 1024 blocks (automatic) and can be forced
    either way: the same bits come out."""
    s = SHAPES["gqa4_d128"]
    b = wl._make("occupancy", s, [1] * 40, [int(x) for x in np.random.default_rng(5).integers(1, 3000, size=40)], 85)
    outs = []
    for per_cu in (-1, 1, 2):
        h = hx.make_handle(b)
        h.set_option("decode_blocks_per_cu", per_cu)
        st = hx.setup_and_run(b, 0x7FC1, handle=h)
        outs.append(hx.device_to_bits(st["out"]))
        if per_cu == -1:
            compare(hx.bf16_tensor_to_f64(st["out"]), oracle.attention_for_batch(b), "occupancy")
    np.testing.assert_array_equal(outs[0], outs[1])
    np.testing.assert_array_equal(outs[0], outs[2])


def test_very_long_contexts(hx):
    """A decode over 131,072 keys (8,192 pages: cut across blocks, partial rows, merge), a 96-row chunk behind a
    100,000-token prefix (chunk tiles cut for balance) and a short decode in one batch: page and key offsets far
    beyond what the recipes reach."""
    s = wl.AttnShape(8, 2, 128)
    b = wl._make("very_long", s, [1, 96, 1], [131072, 100096, 77], 81, slack=1.05)
    st, got, ref, _ = _check_batch(hx, b, check_pools=False)
    info, items = st["handle"].plan(b.q_start, b.q_len, b.ctx_len)
    assert info.num_reduce_items >= 2 and max(it.key_end for it in items) == 131072


@pytest.mark.parametrize("heads", [(32, 32, 128), (64, 16, 64), (40, 40, 64)])
def test_many_kv_heads(hx, heads):
    """Shapes with many KV heads (multi-head attention with as many KV heads as query heads; more KV heads than the
    part has XCDs): default launch, run-time roles asked for, forced cuts, two kernels in sequence."""
    s = wl.AttnShape(*heads)
    b = wl._make("kvh%d" % heads[1], s, [130, 1, 1, 20, 1], [700, 300, 1, 20, 2500], 82)
    _, _, ref, _ = _check_batch(hx, b, check_pools=True)
    for opts in ({"resident_chunks": 1}, {"tile_split_keys": 64, "split_keys": 64}, {"interleave": 0}):
        h = hx.make_handle(b)
        for k, v in opts.items():
            h.set_option(k, v)
        print("options", opts, flush=True)
        compare(hx.bf16_tensor_to_f64(hx.setup_and_run(b, 0x7FC1, handle=h)["out"]), ref, str(opts))


RANDOM_SHAPES = [wl.AttnShape(4, 1, 64), wl.AttnShape(8, 2, 128), wl.AttnShape(14, 2, 128), wl.AttnShape(3, 3, 64),
                 wl.AttnShape(20, 1, 128), wl.AttnShape(32, 8, 128), wl.AttnShape(8, 8, 64), wl.AttnShape(56, 8, 128),
                 wl.AttnShape(12, 4, 64)]
RANDOM_OPTIONS = [{}, {}, {"tile_split_keys": 64, "split_keys": 32}, {"tile_split_keys": 128}, {"split_keys": 64},
                  {"interleave": 0}, {"interleave": 1}, {"interleave": 2, "resident_chunks": 1}, {"decode_blocks_per_cu": 1},
                  {"decode_blocks_per_cu": 2}, {"tile_min_cols": 1}, {"tile_min_cols": 1 << 20}, {"window": 64},
                  {"window": 333}, {"window": 1000, "tile_split_keys": 96}, {"inline_append": 0}, {"stream_kv": 0},
                  {"stream_kv": 1}]


def test_randomized_batches_shapes_and_options(hx):
    """100 seeded draws of (head shape, number and size of chunks, number of decodes, longest context, planner and
    launch options, sliding window): every output row against the checker.  Covers combinations the hand-picked
    cases above do not (e.g. a windowed batch that is cut every 96 keys, decode-only launches forced to either
    occupancy, chunk-only batches, contexts long enough to be cut across blocks)."""
    rng = np.random.default_rng(20240310)
    worst = [0.0, 0.0]
    for case in range(100):
        shape = RANDOM_SHAPES[int(rng.integers(len(RANDOM_SHAPES)))]
        opts = RANDOM_OPTIONS[int(rng.integers(len(RANDOM_OPTIONS)))]
        n_chunks = int(rng.integers(0, 5))
        n_dec = int(rng.integers(0 if n_chunks else 1, 40))
        max_ctx = int(rng.choice([60, 400, 1500, 4000, 9000]))
        max_chunk = min(int(rng.choice([8, 40, 130, 300, 700])), max_ctx)
        print("case", case, shape, "chunks", n_chunks, "decodes", n_dec, "max_chunk", max_chunk, "max_ctx", max_ctx, opts, flush=True)
        b = wl.random_hybrid(9000 + case, shape, n_chunks, n_dec, max_chunk=max_chunk, max_ctx=max_ctx)
        h = hx.make_handle(b)
        for k, v in opts.items():
            h.set_option(k, v)
        st = hx.setup_and_run(b, 0x7FC1, handle=h)
        got = hx.bf16_tensor_to_f64(st["out"])
        k_all = np.concatenate([st["kv_host"][i][0] for i in range(b.num_seqs)])
        v_all = np.concatenate([st["kv_host"][i][1] for i in range(b.num_seqs)])
        ref = oracle.hybrid_attention(b.q_bits(0), k_all, v_all, b.kv_start, b.q_start, b.q_len, b.ctx_len, b.sm_scale,
                                      window=opts.get("window", 0))
        res = compare(got, ref, "random case %d" % case)
        worst = [max(worst[0], res[0]), max(worst[1], res[1])]
    print("worst max abs %.3e, worst row rel %.3e" % tuple(worst), flush=True)


@pytest.mark.parametrize("shape", ["gqa4_d128", "gqa7_d128", "mqa4_d64"])
@pytest.mark.parametrize("window", [1, 17, 64, 300])
def test_sliding_window(hx, shape, window):
    """Sliding-window attention (the query at p sees keys p-window+1 .. p): chunks whose rows start their
    windows at different keys, decodes, a window longer than some contexts; default plan, forced small
    splits, everything through chunk tiles and everything through wave tiles."""
    s = SHAPES[shape]
    b = wl._make("window_" + shape, s, [300, 1, 37, 1, 1, 70], [1300, 555, 37, 1, 2000, 70], 84)
    ref = oracle.attention_for_batch(b, window=window)
    for opts in ({}, {"tile_split_keys": 64, "split_keys": 32}, {"tile_min_cols": 1}, {"tile_min_cols": 1 << 20},
                 {"resident_chunks": 1, "tile_split_keys": 96}):
        h = hx.make_handle(b)
        h.set_option("window", window)
        for k, v in opts.items():
            h.set_option(k, v)
        print("window", window, "options", opts, flush=True)
        out = hx.bf16_tensor_to_f64(hx.setup_and_run(b, 0x7FC1, handle=h)["out"])
        compare(out, ref, "window %d %s" % (window, opts))


def test_window_longer_than_every_context_changes_nothing(hx):
    s = SHAPES["gqa4_d128"]
    b = wl._make("window_inactive", s, [200, 1, 1], [700, 300, 1], 85)
    base = hx.setup_and_run(b, 0x7FC1)["out"]
    h = hx.make_handle(b)
    h.set_option("window", 700)
    out = hx.setup_and_run(b, 0x7FC1, handle=h)["out"]
    assert torch.equal(out.view(torch.int16), base.view(torch.int16))


@pytest.mark.parametrize("shape", ["gqa4_d128", "mqa4_d64"])
def test_peaky_scores_raise_the_softmax_reference_mid_sequence(hx, shape):
    """sm_scale = 1 makes scores ~ N(0, d): tile maxima jump by far more than the kernels' lazy-rescale slack,
    so the running reference is raised again and again in mid-sequence (chunk tiles: while the weights of the
    previous tile still wait for their output MFMAs)."""
    s = SHAPES[shape]
    b = wl._make("peaky_" + shape, s, [260, 1, 1, 40], [1500, 900, 33, 40], 86, sm_scale=1.0)
    _check_batch(hx, b, check_pools=False)
    for opts in ({"tile_split_keys": 96, "split_keys": 64}, {"tile_min_cols": 1}, {"tile_min_cols": 1 << 20}):
        h = hx.make_handle(b)
        for k, v in opts.items():
            h.set_option(k, v)
        out = hx.bf16_tensor_to_f64(hx.setup_and_run(b, 0x7FC1, handle=h)["out"])
        compare(out, oracle.attention_for_batch(b), "peaky %s" % opts)


def _crafted(case, batch, rng):
    """Hand-made Q/K/V (float64, later rounded to bf16) for one value pattern; direction u carries the scores."""
    s = batch.shape
    T, d = batch.num_tokens, s.head_dim
    u = np.zeros(d); u[0] = 1.0
    q = 0.05 * rng.standard_normal((T, s.num_q_heads, d))
    kv = {}
    for i in range(batch.num_seqs):
        n = int(batch.ctx_len[i])
        k = 0.05 * rng.standard_normal((n, s.num_kv_heads, d))
        v = rng.standard_normal((n, s.num_kv_heads, d))
        pos = np.arange(n)[:, None, None]
        if case == "ascending":      # score grows ~0.5 per key: every 32-key tile lifts the maximum by ~23 (base 2)
            k = k + 0.5 * pos * u
        elif case == "descending":   # the first keys dominate, later weights underflow
            k = k - 0.5 * pos * u
        elif case == "spike_at_tile_edges":
            k = k + 40.0 * np.isin(pos, [0, 31, 32, 33, n // 2, n - 2]) * u
        elif case == "v_outliers":
            v = v * np.where(rng.random((n, 1, 1)) < 0.02, 4.0, 1.0)   # larger values would break the absolute bound in bf16 output
        elif case == "huge_equal_scores":   # large |k| orthogonal noise, identical score contribution
            k = 0.0 * k + 30.0 * u
        kv[i] = (k, v)
    if case in ("ascending", "descending", "spike_at_tile_edges", "huge_equal_scores"):
        q = q + 1.0 * u
    if case == "zero_query":
        q = 0.0 * q
    return q, kv


@pytest.mark.parametrize("case", ["ascending", "descending", "spike_at_tile_edges", "v_outliers", "huge_equal_scores", "zero_query"])
def test_crafted_value_patterns(hx, case):
    """Value patterns that N(0,1) draws never produce: maxima that rise or fall along the sequence, spikes on tile
    edges, outliers in V, huge equal scores, all-equal scores; chunk tiles, wave tiles and forced splits."""
    s = SHAPES["gqa4_d128"]
    b = wl._make("crafted_" + case, s, [200, 1, 1, 70], [900, 1500, 40, 70], 87, sm_scale=1.0)
    rng = np.random.default_rng([88, len(case)])
    q, kv = _crafted(case, b, rng)
    q_bits = wl.f32_to_bf16_bits(q.astype(np.float32))
    kv_bits = {i: (wl.f32_to_bf16_bits(k.astype(np.float32)), wl.f32_to_bf16_bits(v.astype(np.float32))) for i, (k, v) in kv.items()}
    k_all = np.concatenate([kv_bits[i][0] for i in range(b.num_seqs)]); v_all = np.concatenate([kv_bits[i][1] for i in range(b.num_seqs)])
    ref = oracle.hybrid_attention(q_bits, k_all, v_all, b.kv_start, b.q_start, b.q_len, b.ctx_len, b.sm_scale)
    assert np.isfinite(ref).all()
    for opts in ({}, {"tile_split_keys": 96, "split_keys": 64}, {"tile_min_cols": 1}, {"tile_min_cols": 1 << 20}):
        h = hx.make_handle(b)
        for k, v in opts.items():
            h.set_option(k, v)
        print("case", case, "options", opts, flush=True)
        st = hx.setup_and_run(b, 0x7FC1, handle=h, kv_host=dict(kv_bits), q_bits=q_bits)
        compare(hx.bf16_tensor_to_f64(st["out"]), ref, "%s %s" % (case, opts))


def test_run_time_roles_repeat_on_one_workspace(hx):
    """Blocks that pick chunk or wave tiles when they start (per-unit flags and queue heads in the workspace):
    several launches in a row on one handle and workspace, each against the checker and equal bit for bit."""
    s = SHAPES["gqa4_d128"]
    b = wl._make("roles", s, [200, 150, 1, 1, 1, 9, 1], [900, 150, 700, 33, 1200, 64, 300], 83)
    h = hx.make_handle(b)
    h.set_option("resident_chunks", 1)
    h.set_option("tile_split_keys", 256)
    st = hx.setup_and_run(b, 0x7FC1, handle=h)
    ref = oracle.attention_for_batch(b)
    first = hx.bf16_tensor_to_f64(st["out"])
    compare(first, ref, "roles launch 0")
    k_new, v_new = hx.new_token_kv(b, st["kv_host"])
    k_new, v_new = hx.bits_to_device(k_new), hx.bits_to_device(v_new)
    for i in range(1, 5):
        out = hx.run_iteration(h, b, st["k_cache"], st["v_cache"], st["bt"], st["q"], k_new, v_new)
        torch.cuda.synchronize()
        got = hx.bf16_tensor_to_f64(out)
        compare(got, ref, "roles launch %d" % i)
        np.testing.assert_array_equal(got, first)


def test_run_time_roles_do_not_depend_on_what_the_workspace_held(hx):
    """The scheduling words of the run-time role assignment live in the caller's workspace; whatever an earlier
    user of that memory left there (all-ones bytes here, then the leftovers of a launch, then all-ones again)
    must not change the result."""
    s = SHAPES["gqa4_d128"]
    b = wl._make("roles_dirty", s, [200, 150, 1, 1, 1, 9, 1], [900, 150, 700, 33, 1200, 64, 300], 84)
    h = hx.make_handle(b)
    h.set_option("resident_chunks", 1)
    h.set_option("tile_split_keys", 256)
    ws = h.ensure_workspace()
    ws.fill_(0xFF)
    torch.cuda.synchronize()
    st = hx.setup_and_run(b, 0x7FC1, handle=h)
    ref = oracle.attention_for_batch(b)
    first = hx.bf16_tensor_to_f64(st["out"])
    compare(first, ref, "roles on a workspace of 0xFF bytes")
    k_new, v_new = hx.new_token_kv(b, st["kv_host"])
    k_new, v_new = hx.bits_to_device(k_new), hx.bits_to_device(v_new)
    for i in range(2):
        if i == 1:
            ws.fill_(0xFF)
        out = hx.run_iteration(h, b, st["k_cache"], st["v_cache"], st["bt"], st["q"], k_new, v_new)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(hx.bf16_tensor_to_f64(out), first)


def test_many_iterations_and_two_streams_on_one_handle(hx):
    """The per-call metadata travels through a ring of pinned buffers that the launches read directly: forty
    iterations in a row (the ring wraps twice) with different batches in turn, then the same on two streams used
    alternately (a stream change inside half a ring takes the library's slow path), every output equal bit for
    bit to that batch's first result, which is checked against the fp64 checker."""
    from paper_2403_02310_amd import binding
    s = SHAPES["gqa4_d128"]
    batches = [wl._make("ring%d" % i, s, [70 + 9 * i, 1, 1, 5], [300 + 40 * i, 500 - 30 * i, 64 + i, 90], 300 + i, max_blocks=40)
               for i in range(3)]  # one block-table width: the handle's
    cap = max(batches, key=lambda b: b.num_tokens)
    h = binding.Handle(s.num_q_heads, s.num_kv_heads, s.head_dim, max_tokens=max(2048, cap.num_tokens), max_seqs=128,
                       max_blocks_per_seq=40)
    states, firsts = [], []
    for b in batches:
        st = hx.setup_and_run(b, 0x7FC1, handle=h)
        compare(hx.bf16_tensor_to_f64(st["out"]), oracle.attention_for_batch(b), b.name)
        k_new, v_new = hx.new_token_kv(b, st["kv_host"])
        st["k_new"], st["v_new"] = hx.bits_to_device(k_new), hx.bits_to_device(v_new)
        states.append(st)
        firsts.append(hx.device_to_bits(st["out"]))
    outs = []
    for i in range(40):  # enqueued back to back, no host wait in between
        b, st = batches[i % 3], states[i % 3]
        outs.append(hx.run_iteration(h, b, st["k_cache"], st["v_cache"], st["bt"], st["q"], st["k_new"], st["v_new"]))
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        np.testing.assert_array_equal(hx.device_to_bits(o), firsts[i % 3])
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    outs = []
    for i in range(24):
        b, st = batches[i % 3], states[i % 3]
        sm = streams[(i // 3) % 2]
        out = torch.empty_like(st["q"])
        # the two streams share the caches and the workspace: keep their iterations apart
        sm.wait_stream(streams[1 - (i // 3) % 2])
        h.kv_append(st["k_new"], st["v_new"], st["k_cache"], st["v_cache"], st["bt"], b.q_start, b.q_len, b.ctx_len, stream=sm)
        h.hybrid_attention(st["q"], st["k_cache"], st["v_cache"], st["bt"], b.q_start, b.q_len, b.ctx_len, b.sm_scale, out, stream=sm)
        outs.append(out)
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        np.testing.assert_array_equal(hx.device_to_bits(o), firsts[i % 3])


def test_kernel_timing_brackets_every_nth_launch(hx):
    """Options time_kernels / time_every: with every 4th attention launch bracketed, 8 iterations report 2 timed
    launches with a positive duration, and the outputs do not depend on the instrumentation."""
    b = wl.random_hybrid(21, wl.AttnShape(8, 2, 128), n_chunks=1, n_decodes=6, max_chunk=80, max_ctx=700)
    h = hx.make_handle(b)
    st = hx.setup_and_run(b, 0x7FC1, handle=h)
    first = hx.device_to_bits(st["out"])
    k_new, v_new = hx.new_token_kv(b, st["kv_host"])
    k_new, v_new = hx.bits_to_device(k_new), hx.bits_to_device(v_new)
    h.set_option("time_kernels", 1)
    h.set_option("time_every", 4)
    h.kernel_times()
    for _ in range(8):
        out = hx.run_iteration(h, b, st["k_cache"], st["v_cache"], st["bt"], st["q"], k_new, v_new)
    torch.cuda.synchronize()
    kt = h.kernel_times()
    assert kt.attention_launches == 2 and kt.attention_ms > 0.0 and kt.append_launches == 0
    np.testing.assert_array_equal(hx.device_to_bits(out), first)
    h.set_option("time_kernels", 2)
    h.set_option("time_every", 1)
    for _ in range(3):
        hx.run_iteration(h, b, st["k_cache"], st["v_cache"], st["bt"], st["q"], k_new, v_new)
    torch.cuda.synchronize()
    kt = h.kernel_times()
    assert kt.attention_launches == 3 and kt.append_launches == 3
    with pytest.raises(Exception):
        h.set_option("time_every", 0)


def test_chunking_invariance_config1(hx):
    """192-token prompt as 1x192, 3x64, 192x1: KV cache bytes identical, outputs within tolerance of the one fp64 result."""
    q_all = wl.normal_bf16((1, 0x51, 99), (192, 4, 64))
    ref = None
    pools = []
    for chunk in (192, 64, 1):
        iters = wl.config1_prompt(chunk)
        last = iters[-1]
        k_all, v_all = last.kv_bits(0)
        if ref is None:
            ref = oracle.hybrid_attention(q_all, k_all, v_all, [0], [0], [192], [192], last.sm_scale)
        handle = hx.make_handle(last)
        k_cache, v_cache = hx.make_pools(last, 0x7FC1)
        bt = torch.from_numpy(last.block_table).cuda()
        rows = []
        for it in iters:
            n, ctx = int(it.q_len[0]), int(it.ctx_len[0])
            q_dev = hx.bits_to_device(q_all[ctx - n: ctx])
            out = hx.run_iteration(handle, it, k_cache, v_cache, bt, q_dev,
                                   hx.bits_to_device(k_all[ctx - n: ctx]), hx.bits_to_device(v_all[ctx - n: ctx]))
            rows.append(hx.bf16_tensor_to_f64(out))
        torch.cuda.synchronize()
        compare(np.concatenate(rows), ref, "chunk%d" % chunk)
        pools.append((hx.device_to_bits(k_cache), hx.device_to_bits(v_cache)))
    for kc, vc in pools[1:]:
        np.testing.assert_array_equal(kc, pools[0][0])
        np.testing.assert_array_equal(vc, pools[0][1])


def test_block_table_permutation_and_rerun_are_bitwise_stable(hx):
    """Physical page placement and repetition must not change a single output bit."""
    b = wl.random_hybrid(5, wl.AttnShape(8, 2, 128), n_chunks=2, n_decodes=4, max_chunk=70, max_ctx=900)
    a = hx.device_to_bits(hx.setup_and_run(b)["out"])
    a2 = hx.device_to_bits(hx.setup_and_run(b)["out"])
    np.testing.assert_array_equal(a, a2)
    rng = np.random.default_rng(9)
    perm = rng.permutation(b.num_pages).astype(np.int32)
    bt2 = np.where(b.block_table >= 0, perm[np.maximum(b.block_table, 0)], -1).astype(np.int32)
    b2 = wl.HybridBatch(b.name + "_perm", b.shape, b.q_len, b.ctx_len, bt2, b.num_pages, b.seed, b.sm_scale)
    c = hx.device_to_bits(hx.setup_and_run(b2)["out"])
    np.testing.assert_array_equal(a, c)


def test_empty_batch_is_a_noop(hx):
    b = wl.config1_tiny()
    h = hx.make_handle(b)
    e = np.zeros(0, np.int32)
    ws = h.ensure_workspace()
    k_cache, v_cache = hx.make_pools(b, 0)
    bt = torch.from_numpy(b.block_table).cuda()
    q = torch.zeros((0, 4, 64), dtype=torch.bfloat16, device="cuda")
    h.kv_append(q[:, :1], q[:, :1], k_cache, v_cache, bt, e, e, e, num_tokens=0)
    h.hybrid_attention(q, k_cache, v_cache, bt, e, e, e, 0.125, q, num_tokens=0)
    torch.cuda.synchronize()
