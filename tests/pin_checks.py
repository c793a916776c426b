"""Checks that pin the fp64 attention checker to facts that do not come from itself.

Every check takes ``attn``: a callable with the signature of ``oracle.hybrid_attention``
(q_bits, k_bits, v_bits, kv_start, q_start, q_len, ctx_len, sm_scale) -> [T, Hq, d] float64,
so the same checks can be aimed at deliberately broken copies of the checker
(tests/test_oracle_mutants.py) to show that each plausible mistake trips at least one.
"""
import numpy as np
import mpmath

from paper_2403_02310_amd.workloads import bf16_bits_to_f64, f32_to_bf16_bits, normal_bf16


def _prefix_sums(q_len, ctx_len):
    q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int32)
    kv_start = np.concatenate([[0], np.cumsum(ctx_len)[:-1]]).astype(np.int64)
    return q_start, kv_start


def _small_batch(seed, Hq, Hkv, d, q_len, ctx_len, sigma=1.0):
    T, N = int(np.sum(q_len)), int(np.sum(ctx_len))
    q = normal_bf16((seed, 1), (T, Hq, d))
    k = normal_bf16((seed, 2), (N, Hkv, d))
    v = normal_bf16((seed, 3), (N, Hkv, d))
    if sigma != 1.0:
        q = f32_to_bf16_bits((bf16_bits_to_f64(q) * sigma).astype(np.float32))
    q_start, kv_start = _prefix_sums(q_len, ctx_len)
    return q, k, v, kv_start, q_start, np.asarray(q_len, np.int32), np.asarray(ctx_len, np.int32)


def check_bruteforce_mpmath(attn):
    """Paper section 2.1 written as a direct triple loop in 50-digit arithmetic, no max subtraction."""
    mpmath.mp.dps = 50
    Hq, Hkv, d = 4, 2, 4
    q_len, ctx_len = [3, 1, 2], [5, 6, 2]
    scale = 0.37
    q, k, v, kv_start, q_start, ql, cl = _small_batch(11, Hq, Hkv, d, q_len, ctx_len)
    got = attn(q, k, v, kv_start, q_start, ql, cl, scale)
    qf, kf, vf = bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v)
    G = Hq // Hkv
    for s in range(len(q_len)):
        for j in range(q_len[s]):
            pos = ctx_len[s] - q_len[s] + j
            t = q_start[s] + j
            for h in range(Hq):
                g = h // G
                num = [mpmath.mpf(0)] * d
                den = mpmath.mpf(0)
                for i in range(pos + 1):
                    dot = mpmath.mpf(0)
                    for c in range(d):
                        dot += mpmath.mpf(float(qf[t, h, c])) * mpmath.mpf(float(kf[kv_start[s] + i, g, c]))
                    e = mpmath.exp(mpmath.mpf(scale) * dot)
                    den += e
                    for c in range(d):
                        num[c] = num[c] + e * mpmath.mpf(float(vf[kv_start[s] + i, g, c]))
                want = np.array([float(x / den) for x in num])
                np.testing.assert_allclose(got[t, h], want, rtol=1e-13, atol=1e-14)


def check_single_key_returns_v0(attn):
    """A context of one token: the softmax has one weight, 1, so the output is v_0 exactly."""
    q, k, v, kv_start, q_start, ql, cl = _small_batch(12, 4, 2, 8, [1, 1], [1, 1])
    got = attn(q, k, v, kv_start, q_start, ql, cl, 0.5)
    vf = bf16_bits_to_f64(v)
    for s in range(2):
        for h in range(4):
            np.testing.assert_array_equal(got[s, h], vf[kv_start[s], h // 2])


def check_zero_query_gives_running_mean(attn):
    """q = 0 makes all scores equal: row at position p returns the mean of V[0..p]."""
    q, k, v, kv_start, q_start, ql, cl = _small_batch(13, 2, 1, 8, [6], [9])
    q[:] = 0
    got = attn(q, k, v, kv_start, q_start, ql, cl, 1.0)
    vf = bf16_bits_to_f64(v)
    for j in range(6):
        pos = 3 + j
        want = vf[: pos + 1, 0].mean(axis=0)
        for h in range(2):
            np.testing.assert_allclose(got[j, h], want, rtol=1e-14, atol=1e-15)


def check_identical_keys_give_mean(attn):
    q, k, v, kv_start, q_start, ql, cl = _small_batch(14, 2, 2, 8, [4], [7])
    k[:] = k[0:1]
    got = attn(q, k, v, kv_start, q_start, ql, cl, 0.8)
    vf = bf16_bits_to_f64(v)
    for j in range(4):
        pos = 3 + j
        for h in range(2):
            np.testing.assert_allclose(got[j, h], vf[: pos + 1, h].mean(axis=0), rtol=1e-13, atol=1e-15)


def check_constant_v(attn):
    q, k, v, kv_start, q_start, ql, cl = _small_batch(15, 4, 2, 8, [5, 1], [11, 20])
    v[:] = f32_to_bf16_bits(np.float32([1.5]))[0]
    got = attn(q, k, v, kv_start, q_start, ql, cl, 0.3)
    np.testing.assert_allclose(got, 1.5, rtol=1e-14)


def check_dominant_key(attn):
    """One key aligned with q and huge: the output tends to that key's value."""
    d = 8
    q, k, v, kv_start, q_start, ql, cl = _small_batch(16, 1, 1, d, [1], [10])
    qf = np.zeros((1, 1, d), np.float32); qf[0, 0, 0] = 4.0
    q = f32_to_bf16_bits(qf)
    kf = np.zeros((10, 1, d), np.float32); kf[6, 0, 0] = 32.0
    k = f32_to_bf16_bits(kf)
    got = attn(q, k, v, kv_start, q_start, ql, cl, 1.0)
    np.testing.assert_allclose(got[0, 0], bf16_bits_to_f64(v)[6, 0], rtol=0, atol=1e-40)


def check_score_shift_invariance(attn):
    """Adding the same constant to every score of a row changes nothing (softmax)."""
    d = 4
    q_len, ctx_len = [3], [6]
    q_start, kv_start = _prefix_sums(q_len, ctx_len)
    qf = np.zeros((3, 1, d), np.float32); qf[:, 0, 0] = 2.0
    a = np.float32([0.5, -1.0, 2.0, 0.25, -0.75, 1.5])
    outs = []
    v = normal_bf16((17, 3), (6, 1, d))
    for shift in (0.0, 3.0, -5.0):
        kf = np.zeros((6, 1, d), np.float32); kf[:, 0, 0] = a + np.float32(shift)
        kf[:, 0, 1] = 7.0  # q is zero on this channel: must not matter
        outs.append(attn(f32_to_bf16_bits(qf), f32_to_bf16_bits(kf), v, kv_start, q_start,
                         np.int32(q_len), np.int32(ctx_len), 0.5))
    np.testing.assert_allclose(outs[1], outs[0], rtol=1e-13)
    np.testing.assert_allclose(outs[2], outs[0], rtol=1e-13)
    # and the scale matters: halving sm_scale must change the result
    kf = np.zeros((6, 1, d), np.float32); kf[:, 0, 0] = a
    other = attn(f32_to_bf16_bits(qf), f32_to_bf16_bits(kf), v, kv_start, q_start,
                 np.int32(q_len), np.int32(ctx_len), 0.25)
    assert np.abs(other - outs[0]).max() > 1e-3


def dense_masked_softmax(qf, kf, vf, prefix, scale):
    """Library route for ONE sequence and ONE head pair: softmax(Q K^T scale + mask) V with numpy matmul."""
    s = (qf @ kf.T) * scale
    n_q, n_k = s.shape
    i = np.arange(n_k)[None, :]
    j = np.arange(n_q)[:, None]
    s = np.where(i <= prefix + j, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return p @ vf


def check_against_dense_library(attn, batch=None):
    """Per sequence and head, the result equals a dense masked softmax(QK^T)V done with matmuls."""
    if batch is None:
        Hq, Hkv, d = 6, 2, 16
        q_len, ctx_len = [17, 1, 40, 1, 5], [50, 33, 40, 1, 64]
        q, k, v, kv_start, q_start, ql, cl = _small_batch(18, Hq, Hkv, d, q_len, ctx_len)
        scale = 1.0 / np.sqrt(d)
    else:
        q = batch.q_bits(); k, v = batch.kv_concat()
        kv_start, q_start, ql, cl, scale = batch.kv_start, batch.q_start, batch.q_len, batch.ctx_len, batch.sm_scale
        Hq, Hkv, d = q.shape[1], k.shape[1], q.shape[2]
    got = attn(q, k, v, kv_start, q_start, ql, cl, scale)
    qf, kf, vf = bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v)
    G = Hq // Hkv
    for s in range(len(ql)):
        rows = slice(int(q_start[s]), int(q_start[s] + ql[s]))
        keys = slice(int(kv_start[s]), int(kv_start[s] + cl[s]))
        for h in range(Hq):
            want = dense_masked_softmax(qf[rows, h], kf[keys, h // G], vf[keys, h // G], int(cl[s] - ql[s]), scale)
            np.testing.assert_allclose(got[rows, h], want, rtol=1e-11, atol=1e-13)


def check_gqa_equals_expanded_mha(attn):
    """Copying each K/V head G times (GQA -> MHA) must not change any output."""
    Hq, Hkv, d = 8, 2, 8
    q, k, v, kv_start, q_start, ql, cl = _small_batch(19, Hq, Hkv, d, [7, 1], [19, 12])
    a = attn(q, k, v, kv_start, q_start, ql, cl, 0.4)
    k2 = np.repeat(k, Hq // Hkv, axis=1)
    v2 = np.repeat(v, Hq // Hkv, axis=1)
    b = attn(q, k2, v2, kv_start, q_start, ql, cl, 0.4)
    np.testing.assert_array_equal(a, b)


def check_sequence_permutation(attn):
    """Reordering the sequences of a batch reorders the outputs and changes nothing else."""
    Hq, Hkv, d = 4, 2, 8
    q_len, ctx_len = [5, 1, 3], [9, 14, 3]
    q, k, v, kv_start, q_start, ql, cl = _small_batch(20, Hq, Hkv, d, q_len, ctx_len)
    a = attn(q, k, v, kv_start, q_start, ql, cl, 0.4)
    perm = [2, 0, 1]
    q2 = np.concatenate([q[q_start[s]: q_start[s] + ql[s]] for s in perm])
    k2 = np.concatenate([k[kv_start[s]: kv_start[s] + cl[s]] for s in perm])
    v2 = np.concatenate([v[kv_start[s]: kv_start[s] + cl[s]] for s in perm])
    ql2, cl2 = ql[perm], cl[perm]
    qs2, kvs2 = _prefix_sums(ql2, cl2)
    b = attn(q2, k2, v2, kvs2, qs2, ql2, cl2, 0.4)
    a_perm = np.concatenate([a[q_start[s]: q_start[s] + ql[s]] for s in perm])
    np.testing.assert_array_equal(a_perm, b)


def check_chunking_invariance(attn, prompt_len=48, chunks=(48, 16, 5, 1)):
    """Prefilling a prompt in chunks of any size (size 1 = decode) gives the rows of the one-shot prefill.

    Paper section 4.1/4.3: chunking splits the prefill over iterations; every chunk reads the
    keys and values of all earlier chunks; the computation is unchanged.
    """
    Hq, Hkv, d = 4, 1, 16
    q = normal_bf16((21, 1), (prompt_len, Hq, d))
    k = normal_bf16((21, 2), (prompt_len, Hkv, d))
    v = normal_bf16((21, 3), (prompt_len, Hkv, d))
    results = []
    for c in chunks:
        rows = []
        done = 0
        while done < prompt_len:
            n = min(c, prompt_len - done)
            out = attn(q[done: done + n], k[: done + n], v[: done + n], np.int64([0]), np.int32([0]),
                       np.int32([n]), np.int32([done + n]), 0.25)
            rows.append(out)
            done += n
        results.append(np.concatenate(rows))
    for r in results[1:]:
        np.testing.assert_array_equal(r, results[0])
    # and the rows are not all alike (a prefix-insensitive bug would pass the above otherwise)
    assert np.abs(results[0][0] - results[0][-1]).max() > 1e-3


# ---- sliding window (Table 1 lists Mistral-7B's attention as grouped-query with a sliding window) ----
# These take ``attn`` with a keyword ``window``: the query at position p sees keys p-window+1 .. p.

def check_window_bruteforce_mpmath(attn):
    """The windowed sum written as a direct loop over keys max(0, p-W+1) .. p in 50-digit arithmetic."""
    mpmath.mp.dps = 50
    Hq, Hkv, d = 4, 2, 4
    q_len, ctx_len = [4, 1, 3], [7, 9, 3]
    scale = 0.41
    q, k, v, kv_start, q_start, ql, cl = _small_batch(31, Hq, Hkv, d, q_len, ctx_len)
    qf, kf, vf = bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v)
    G = Hq // Hkv
    for W in (1, 2, 3, 5):
        got = attn(q, k, v, kv_start, q_start, ql, cl, scale, window=W)
        for s in range(len(q_len)):
            for j in range(q_len[s]):
                pos = ctx_len[s] - q_len[s] + j
                t = q_start[s] + j
                for h in range(Hq):
                    g = h // G
                    num = [mpmath.mpf(0)] * d
                    den = mpmath.mpf(0)
                    for i in range(max(0, pos - W + 1), pos + 1):
                        dot = mpmath.mpf(0)
                        for c in range(d):
                            dot += mpmath.mpf(float(qf[t, h, c])) * mpmath.mpf(float(kf[kv_start[s] + i, g, c]))
                        e = mpmath.exp(mpmath.mpf(scale) * dot)
                        den += e
                        for c in range(d):
                            num[c] = num[c] + e * mpmath.mpf(float(vf[kv_start[s] + i, g, c]))
                    want = np.array([float(x / den) for x in num])
                    np.testing.assert_allclose(got[t, h], want, rtol=1e-13, atol=1e-14)


def check_window_of_one_returns_own_v(attn):
    """W = 1: the only visible key is the token itself, so the output is its own V row exactly."""
    q, k, v, kv_start, q_start, ql, cl = _small_batch(32, 4, 2, 8, [5, 1], [9, 6])
    got = attn(q, k, v, kv_start, q_start, ql, cl, 0.5, window=1)
    vf = bf16_bits_to_f64(v)
    for s in range(2):
        for j in range(ql[s]):
            pos = cl[s] - ql[s] + j
            for h in range(4):
                np.testing.assert_array_equal(got[q_start[s] + j, h], vf[kv_start[s] + pos, h // 2])


def check_window_at_least_context_changes_nothing(attn):
    """W >= ctx_len hides no key: bit-identical to no window; W = ctx_len - 1 differs in the last row only."""
    q, k, v, kv_start, q_start, ql, cl = _small_batch(33, 4, 2, 8, [6, 1], [10, 7])
    base = attn(q, k, v, kv_start, q_start, ql, cl, 0.3)
    for W in (10, 11, 1000):
        np.testing.assert_array_equal(attn(q, k, v, kv_start, q_start, ql, cl, 0.3, window=W), base)
    nine = attn(q, k, v, kv_start, q_start, ql, cl, 0.3, window=9)
    np.testing.assert_array_equal(nine[:5], base[:5])       # positions 4..8 of sequence 0 see <= 9 keys anyway
    assert np.abs(nine[5] - base[5]).max() > 1e-6             # position 9 loses key 0
    np.testing.assert_array_equal(nine[6], base[6])         # the decode of sequence 1 (position 6) sees 7 keys


def check_window_equals_attention_over_cut_sequence(attn):
    """Row p under window W = the LAST row of plain attention over the sequence cut to keys p-W+1 .. p."""
    Hq, Hkv, d, W = 4, 2, 8, 5
    q, k, v, kv_start, q_start, ql, cl = _small_batch(34, Hq, Hkv, d, [7], [12])
    got = attn(q, k, v, kv_start, q_start, ql, cl, 0.45, window=W)
    for j in range(7):
        pos = 5 + j
        lo = max(0, pos - W + 1)
        n = pos - lo + 1
        cut = attn(q[j:j + 1], k[lo:pos + 1], v[lo:pos + 1], np.array([0], np.int64), np.array([0], np.int32),
                   np.array([1], np.int32), np.array([n], np.int32), 0.45)
        np.testing.assert_allclose(got[j], cut[0], rtol=1e-14, atol=1e-15)


WINDOW_CHECKS = [
    check_window_bruteforce_mpmath,
    check_window_of_one_returns_own_v,
    check_window_at_least_context_changes_nothing,
    check_window_equals_attention_over_cut_sequence,
]

ALL_CHECKS = [
    check_bruteforce_mpmath,
    check_single_key_returns_v0,
    check_zero_query_gives_running_mean,
    check_identical_keys_give_mean,
    check_constant_v,
    check_dominant_key,
    check_score_shift_invariance,
    check_against_dense_library,
    check_gqa_equals_expanded_mha,
    check_sequence_permutation,
    check_chunking_invariance,
]
