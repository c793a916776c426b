"""Pins of stall-free batching (paper Algorithm 3, section 4.2), written as functions of an implementation
``impl(token_budget, chunk_size, running_decodes, running_prefills, waiting, free_pages, page_size, max_batch_size)
-> dict`` so that the same checks run on the reference in oracle/, on the library's host code and on mutants of
the reference (tests/test_scheduler_mutants.py).

What the paper fixes and these checks assert: every running decode is in every batch, first, with one token
(decodes never stall); prefill tokens only get the budget the decodes leave; a chunk is the largest the leftover
budget admits; new requests enter first come first served while memory lasts; the worked scenario of the
section's scheduling figure.  The admission test itself (``can_allocate_request``) is undefined in the paper:
``check_admission_reading`` pins THIS BUILD's reading (a prompt is admitted iff all its pages are free, and
reserves them), not the paper.
"""
import numpy as np


def as_dict(b):
    """A ``scheduler_reference.Batch`` (or a mutant's) in the form the library binding returns."""
    return {"seq_id": b.seq_id, "q_start": b.q_start, "q_len": b.q_len, "ctx_len": b.ctx_len,
            "num_tokens": b.num_tokens, "num_decodes": b.num_decodes, "num_prefill_chunks": b.num_prefill_chunks,
            "num_admitted": b.num_admitted, "free_pages_left": b.free_pages_left}


def random_state(rng):
    n_dec = int(rng.integers(0, 40)); n_pre = int(rng.integers(0, 4)); n_wait = int(rng.integers(0, 6))
    dec = [(i, int(p), int(p), int(rng.integers(0, 50))) for i, p in enumerate(rng.integers(1, 3000, n_dec))]
    pre = []
    for i in range(n_pre):
        p = int(rng.integers(2, 9000)); pre.append((100 + i, p, int(rng.integers(0, p)), 0))
    wait = [(200 + i, int(p), 0, 0) for i, p in enumerate(rng.integers(1, 9000, n_wait))]
    return dec, pre, wait


def check_invariants_on_random_states(impl, n_states=200, seed=42):
    rng = np.random.default_rng(seed)
    for _ in range(n_states):
        dec, pre, wait = random_state(rng)
        tb = int(rng.choice([64, 256, 512, 2048])); cs = int(rng.choice([64, 512, 4096]))
        free = int(rng.integers(0, 2000)); maxb = 128
        b = impl(tb, cs, dec, pre, wait, free, 16, maxb)
        n = len(b["seq_id"])
        # every running decode is in the batch exactly once, first, with one token (decodes never stall)
        assert b["seq_id"][: len(dec)] == [d[0] for d in dec]
        assert b["q_len"][: len(dec)] == [1] * len(dec)
        assert b["ctx_len"][: len(dec)] == [d[1] + d[3] + 1 for d in dec]
        assert b["num_decodes"] == len(dec)
        # prefill tokens fit the leftover budget; each chunk within chunk_size and the remaining prompt
        chunks = b["q_len"][len(dec):]
        assert sum(chunks) <= max(0, tb - len(dec))
        by_id = {r[0]: r for r in pre + wait}
        for sid, c, ctx in zip(b["seq_id"][len(dec):], chunks, b["ctx_len"][len(dec):]):
            _, plen, done, _ = by_id[sid]
            assert 1 <= c <= min(cs, plen - done)
            assert ctx == done + c
        # a chunk is the LARGEST the leftover budget admits: every chunk but the last uses up its cap, and so
        # does the last unless the budget ran out there
        left = max(0, tb - len(dec))
        for sid, c in zip(b["seq_id"][len(dec):], chunks):
            _, plen, done, _ = by_id[sid]
            assert c == min(cs, plen - done, left)
            left -= c
        # at most one chunk per request; q_start is the prefix sum; sizes add up
        assert len(set(b["seq_id"])) == n
        assert b["q_start"] == [int(x) for x in np.concatenate([[0], np.cumsum(b["q_len"])[:-1]])] if n else True
        assert b["num_tokens"] == sum(b["q_len"]) and b["num_prefill_chunks"] == len(chunks) and n <= maxb
        # running prefills come before new requests, in the order given, none skipped while budget and room remain
        ids_after = b["seq_id"][len(dec):]
        admitted = [i for i in ids_after if i >= 200]
        assert admitted == [w[0] for w in wait[: b["num_admitted"]]]
        assert ids_after == [i for i in ids_after if i < 200] + admitted
        running_in = [i for i in ids_after if i < 200]
        assert running_in == [p[0] for p in pre[: len(running_in)]]
        if len(running_in) < len(pre):
            assert sum(chunks) == max(0, tb - len(dec)) or n == maxb     # only a spent budget (or a full batch) leaves one out
        # admitted requests are a first-come-first-served prefix of the waiting list and reserve their prompt's pages
        pages = sum((w[1] + 15) // 16 for w in wait[: b["num_admitted"]])
        assert b["free_pages_left"] == free - pages and b["free_pages_left"] >= 0
        # the first request NOT admitted was stopped by something: no budget, no room in the batch, or no pages
        if b["num_admitted"] < len(wait):
            nxt = wait[b["num_admitted"]]
            assert (sum(chunks) >= max(0, tb - len(dec)) or n >= maxb or (nxt[1] + 15) // 16 > b["free_pages_left"])


def check_config_shapes(impl):
    # LLaMA2-70B recipe: 1024 decodes, budget 2048, chunk 512 -> exactly two 512-token chunks from two requests
    dec = [(i, 600, 600, 3) for i in range(1024)]
    pre = [(5000, 4000, 1024, 0), (5001, 3000, 0, 0), (5002, 2000, 0, 0)]
    b = impl(2048, 512, dec, pre, [], 10_000, 16, 2048)
    assert b["q_len"][1024:] == [512, 512] and b["num_tokens"] == 2048
    # Mistral recipe read through Algorithm 3: budget 512 with 64 decodes leaves a 448-token chunk
    dec = [(i, 1000, 1000, 0) for i in range(64)]
    b = impl(512, 512, dec, [(99, 4096, 1000, 0)], [], 0, 16, 128)
    assert b["q_len"][64:] == [448] and b["ctx_len"][64:] == [1448]
    # more decodes than budget: all decodes still run, no prefill token is added
    dec = [(i, 10, 10, 0) for i in range(100)]
    b = impl(64, 64, dec, [(999, 500, 0, 0)], [(1000, 50, 0, 0)], 100, 16, 128)
    assert b["num_decodes"] == 100 and b["num_prefill_chunks"] == 0 and b["num_tokens"] == 100


def check_figure_scenario_and_full_drain(impl):
    """A and B decode; C then D arrive: C's prefill is split into chunks that ride along with A's and B's
    decodes (paper section 4.2, the example of its scheduling figure); iterating drains every prompt."""
    budget, chunk = 256, 256
    state = {"A": [300, 300, 5], "B": [200, 200, 9], "C": [400, 0, 0], "D": [100, 0, 0]}   # prompt, prefilled, decoded
    ids = {"A": 1, "B": 2, "C": 3, "D": 4}
    names = {v: k for k, v in ids.items()}
    running, waiting = ["A", "B"], ["C", "D"]
    seen_chunks = {"C": [], "D": []}
    for it in range(12):
        dec = [(ids[r], state[r][0], state[r][1], state[r][2]) for r in running if state[r][1] == state[r][0]]
        pre = [(ids[r], state[r][0], state[r][1], 0) for r in running if state[r][1] < state[r][0]]
        wait = [(ids[r], state[r][0], 0, 0) for r in waiting]
        b = impl(budget, chunk, dec, pre, wait, 1000, 16, 16)
        # A and B decode in EVERY iteration: no generation stall
        assert set(b["seq_id"][: b["num_decodes"]]) >= {1, 2}
        assert b["num_tokens"] <= budget
        for sid, c in zip(b["seq_id"][b["num_decodes"]:], b["q_len"][b["num_decodes"]:]):
            seen_chunks[names[sid]].append(c)
            state[names[sid]][1] += c
        for sid in b["seq_id"][: b["num_decodes"]]:
            state[names[sid]][2] += 1
        for _ in range(b["num_admitted"]):
            running.append(waiting.pop(0))
    assert seen_chunks["C"] == [254, 146]          # first chunk = budget minus the two decodes, then the rest
    assert seen_chunks["D"] == [100]               # fits the budget left in the iteration of C's second chunk
    assert state["C"][1] == 400 and state["D"][1] == 100


def check_admission_reading(impl):
    """This build's reading of the admission test the paper leaves undefined: a waiting prompt is admitted exactly
    when all of its pages are free (an exact fit is admitted, one page short is not), and the pages are reserved
    for it at once, so a second prompt sees only what the first left."""
    b = impl(512, 512, [], [], [(7, 160, 0, 0)], 10, 16, 8)        # 160 tokens = 10 pages, 10 free: fits exactly
    assert b["num_admitted"] == 1 and b["free_pages_left"] == 0 and b["q_len"] == [160]
    b = impl(512, 512, [], [], [(7, 161, 0, 0)], 10, 16, 8)        # 11 pages, 10 free
    assert b["num_admitted"] == 0 and b["free_pages_left"] == 10 and b["q_len"] == []
    b = impl(512, 512, [], [], [(7, 100, 0, 0), (8, 100, 0, 0)], 13, 16, 8)   # 7 + 7 pages, 13 free: the second waits
    assert b["num_admitted"] == 1 and b["free_pages_left"] == 6 and b["seq_id"] == [7]
    # first come first served: a request that would fit does not overtake one that does not
    b = impl(512, 512, [], [], [(7, 400, 0, 0), (8, 16, 0, 0)], 5, 16, 8)
    assert b["num_admitted"] == 0 and b["seq_id"] == []
