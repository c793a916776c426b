/*
 * TEST INFRASTRUCTURE ONLY: a plain, slow, fp64 CPU statement of a linear layer applied to the
 * tokens of a batch.  Nothing in the product path may call this; it shares no code, header,
 * table or helper with the HIP library.
 *
 * What is computed (paper section 2.1): the Q, K and V vectors of a token come from a linear
 * transformation of its embedding, the heads' outputs are combined by another one, and the
 * feed-forward network is two more around an activation.  Section 3.1 studies exactly these
 * operators (they are most of an iteration's time): every token of the batch meets the same
 * weights, so their cost per token falls as the batch grows until arithmetic, not the fetch of
 * the weights, bounds it.  A linear transformation of the T token rows x[t][0..K) by a weight
 * matrix with N output features is the plain definition
 *
 *     y[t][n] = sum over k < K of  x[t][k] * w[n][k]
 *
 * The paper fixes neither a bias nor a storage order.  Readings taken here: no bias (the models
 * of its Table 1 have none in these layers), and the weight is stored output-feature-major,
 * w[n][k] with k contiguous, so that a token row and a weight row are both read along k.
 *
 * Inputs are bf16 bit patterns widened exactly to double; products and sums are double, in
 * the order k = 0, 1, ..., K-1; no blocking, no reordering.
 *
 * Pins (tests/test_linear_oracle_pins.py): a float64 library matrix product, exact rational
 * arithmetic on small integers, identity and one-hot special cases, a sum that single
 * precision would lose, additivity on exactly representable inputs, row and column subsets.
 */
#include <stdint.h>
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

/*
 * x     [T, K] bf16 bits, row-major (one row per token of the batch)
 * w     [N, K] bf16 bits, row-major (one row per output feature)
 * rows  optional list of token rows to compute (NULL = all T); n_rows its length
 * cols  optional list of output features to compute (NULL = all N); n_cols its length
 * out   [n_rows, n_cols] double
 * returns 0, or -1 on an index outside the matrices.
 */
int oracle_linear(const uint16_t *x, const uint16_t *w, int T, int N, int K,
                  const int32_t *rows, int n_rows, const int32_t *cols, int n_cols,
                  double *out, int num_threads) {
    const int R = rows ? n_rows : T;
    const int C = cols ? n_cols : N;
    int bad = 0;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#else
    (void)num_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int r = 0; r < R; ++r) {
        for (int c = 0; c < C; ++c) {
            const int t = rows ? rows[r] : r;
            const int n = cols ? cols[c] : c;
            if (t < 0 || t >= T || n < 0 || n >= N) { bad = 1; continue; }
            const uint16_t *x_row = x + (int64_t)t * K;
            const uint16_t *w_row = w + (int64_t)n * K;
            double sum = 0.0;
            for (int k = 0; k < K; ++k) sum += bf16_to_f64(x_row[k]) * bf16_to_f64(w_row[k]);
            out[(int64_t)r * C + c] = sum;
        }
    }
    return bad ? -1 : 0;
}
