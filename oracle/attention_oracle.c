/*
 * TEST INFRASTRUCTURE ONLY: a plain, slow, fp64 CPU statement of what one iteration's
 * attention over a hybrid batch computes.  Nothing in the product path may call this.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What is computed (paper section 2.1, "self-attention module"): for every query
 * token, the dot product of its Q vector with the K vectors of all tokens of its own
 * sequence up to and including itself, a softmax over those scores, and the average
 * of the matching V vectors weighted by the softmax.  Several heads run side by side;
 * with grouped-query attention (section 2.2) consecutive groups of Hq/Hkv query heads
 * read the same K/V head.
 *
 * A hybrid batch (section 4.1-4.2) holds, per sequence s, q_len[s] new query rows at
 * absolute positions ctx_len[s]-q_len[s] .. ctx_len[s]-1.  A prefill chunk is q_len > 1
 * rows on top of an already processed prefix; a decode is q_len == 1.  Chunking changes
 * which iteration computes a row, never the row's value (section 4.3: a chunk reads the
 * keys and values of all earlier chunks; the cost of the computation is unchanged), so
 * the row result below depends only on (sequence contents, position, head).
 *
 * Sliding-window attention (the paper's Table 1 lists Mistral-7B's attention as grouped-query
 * with a sliding window; the paper does not define it, this file takes the usual meaning):
 * with a window of W tokens the query at position p sees keys p-W+1 .. p only (at most W keys,
 * itself included); W <= 0 means no window.  Nothing else changes.
 *
 * Keys and values arrive CONTIGUOUS per sequence (position-major); this file never sees
 * pages or block tables.  Inputs are bf16 bit patterns widened exactly to double; all
 * arithmetic is double; no blocking, no running-max rescaling, no reordering.
 *
 * Pins (tests/test_oracle_pins.py): brute force in 50-digit arithmetic on tiny inputs,
 * closed forms (one key, equal scores, constant V, dominant key), weights summing to 1,
 * shift invariance, a dense masked-softmax matrix product per sequence, GQA-to-MHA
 * expansion, and chunking invariance; for the window: W >= context equals no window, W = 1
 * returns the token's own V, 50-digit brute force over the window, and equality with plain
 * attention over a sequence cut to the window.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Scores x_i = sm_scale * <q, k_i>, i = lo..pos, for one (query row, head). */
static void scores_for_row(const uint16_t *q_row, const uint16_t *k_seq, int kv_head,
                           int num_kv_heads, int d, int lo, int pos, double sm_scale, double *x) {
    for (int i = lo; i <= pos; ++i) {
        const uint16_t *k_row = k_seq + ((int64_t)i * num_kv_heads + kv_head) * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += bf16_to_f64(q_row[c]) * bf16_to_f64(k_row[c]);
        x[i] = sm_scale * dot;
    }
}

/* Softmax weights over x[lo..pos] written in place; returns nothing, weights sum to 1. */
static void softmax_in_place(double *x, int lo, int pos) {
    double m = x[lo];
    for (int i = lo + 1; i <= pos; ++i) if (x[i] > m) m = x[i];
    double z = 0.0;
    for (int i = lo; i <= pos; ++i) { x[i] = exp(x[i] - m); z += x[i]; }
    for (int i = lo; i <= pos; ++i) x[i] /= z;
}

/* First key position the query at `pos` sees under a window of `window` tokens (<= 0: none). */
static int window_first_key(int pos, int window) {
    if (window <= 0) return 0;
    const int lo = pos - window + 1;
    return lo > 0 ? lo : 0;
}

/*
 * q        [num_tokens, Hq, d]  bf16 bits, batch order (sequence s owns rows q_start[s]..+q_len[s])
 * k_seq    [sum ctx_len, Hkv, d] bf16 bits; sequence s owns rows kv_start[s]..+ctx_len[s], position-major
 * v_seq    same shape
 * tokens   optional list of batch-row indices to compute (NULL = all); n_tokens its length
 * out      [n_rows, Hq, d] double, n_rows = n_tokens if tokens != NULL else num_tokens
 * window   sliding window in tokens, <= 0 for none
 * returns 0, or -1 on an inconsistent description.
 */
int oracle_hybrid_attention_window(const uint16_t *q, const uint16_t *k_seq, const uint16_t *v_seq,
                                   const int64_t *kv_start, const int32_t *q_start, const int32_t *q_len,
                                   const int32_t *ctx_len, int num_seqs, int num_tokens,
                                   int num_q_heads, int num_kv_heads, int d, double sm_scale, int window,
                                   const int32_t *tokens, int n_tokens, double *out, int num_threads) {
    if (num_q_heads % num_kv_heads != 0) return -1;
    const int group = num_q_heads / num_kv_heads;
    const int n_rows = tokens ? n_tokens : num_tokens;

    /* batch row -> owning sequence */
    int32_t *owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)(num_tokens > 0 ? num_tokens : 1));
    for (int t = 0; t < num_tokens; ++t) owner[t] = -1;
    int max_ctx = 1;
    for (int s = 0; s < num_seqs; ++s) {
        if (q_len[s] < 1 || q_len[s] > ctx_len[s] || q_start[s] < 0 || q_start[s] + q_len[s] > num_tokens) {
            free(owner);
            return -1;
        }
        for (int j = 0; j < q_len[s]; ++j) owner[q_start[s] + j] = s;
        if (ctx_len[s] > max_ctx) max_ctx = ctx_len[s];
    }
    int bad = 0;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * (size_t)max_ctx);
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int r = 0; r < n_rows; ++r) {
            for (int h = 0; h < num_q_heads; ++h) {
                const int t = tokens ? tokens[r] : r;
                if (t < 0 || t >= num_tokens || owner[t] < 0) { bad = 1; continue; }
                const int s = owner[t];
                const int j = t - q_start[s];
                const int pos = ctx_len[s] - q_len[s] + j;       /* absolute position of this query */
                const int g = h / group;                          /* K/V head shared by the group */
                const uint16_t *q_row = q + ((int64_t)t * num_q_heads + h) * d;
                const uint16_t *ks = k_seq + kv_start[s] * num_kv_heads * d;
                const uint16_t *vs = v_seq + kv_start[s] * num_kv_heads * d;
                const int lo = window_first_key(pos, window);
                scores_for_row(q_row, ks, g, num_kv_heads, d, lo, pos, sm_scale, w);
                softmax_in_place(w, lo, pos);
                double *o = out + ((int64_t)r * num_q_heads + h) * d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int i = lo; i <= pos; ++i) {
                    const uint16_t *v_row = vs + ((int64_t)i * num_kv_heads + g) * d;
                    for (int c = 0; c < d; ++c) o[c] += w[i] * bf16_to_f64(v_row[c]);
                }
            }
        }
        free(w);
    }
    free(owner);
    return bad ? -1 : 0;
}

/* The same without a window (every query sees all keys up to itself). */
int oracle_hybrid_attention(const uint16_t *q, const uint16_t *k_seq, const uint16_t *v_seq,
                            const int64_t *kv_start, const int32_t *q_start, const int32_t *q_len,
                            const int32_t *ctx_len, int num_seqs, int num_tokens,
                            int num_q_heads, int num_kv_heads, int d, double sm_scale,
                            const int32_t *tokens, int n_tokens, double *out, int num_threads) {
    return oracle_hybrid_attention_window(q, k_seq, v_seq, kv_start, q_start, q_len, ctx_len, num_seqs, num_tokens,
                                          num_q_heads, num_kv_heads, d, sm_scale, 0, tokens, n_tokens, out, num_threads);
}

/* Softmax weights of ONE (batch row t, head h): weights[0..pos], returns pos+1 (or -1). */
int oracle_softmax_weights(const uint16_t *q, const uint16_t *k_seq, const int64_t *kv_start,
                           const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len,
                           int num_seqs, int num_q_heads, int num_kv_heads, int d, double sm_scale,
                           int t, int h, double *weights) {
    const int group = num_q_heads / num_kv_heads;
    for (int s = 0; s < num_seqs; ++s) {
        if (t >= q_start[s] && t < q_start[s] + q_len[s]) {
            const int pos = ctx_len[s] - q_len[s] + (t - q_start[s]);
            const uint16_t *q_row = q + ((int64_t)t * num_q_heads + h) * d;
            const uint16_t *ks = k_seq + kv_start[s] * num_kv_heads * d;
            scores_for_row(q_row, ks, h / group, num_kv_heads, d, 0, pos, sm_scale, weights);
            softmax_in_place(weights, 0, pos);
            return pos + 1;
        }
    }
    return -1;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
