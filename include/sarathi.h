/*
 * sarathi.h -- C ABI of the hybrid-batch paged attention library for MI355X (gfx950).
 *
 * One scheduling iteration of Sarathi-Serve (arXiv 2403.02310) processes a HYBRID BATCH:
 * every running decode contributes one query token and some prefills contribute a CHUNK
 * of their prompt (chunked-prefills, section 4.1; stall-free batching, section 4.2,
 * Algorithm 3).  This library is the attention of one such iteration for one layer:
 *
 *   sarathi_build_stall_free_batch   host only: one pass of Algorithm 3
 *   sarathi_kv_append                write the iteration's new K/V rows into the paged cache
 *   sarathi_hybrid_attention         softmax attention of every query row of the batch
 *
 * Batch description (host arrays of length num_seqs).  Sequence s contributes q_len[s] new
 * tokens, rows q_start[s] .. q_start[s]+q_len[s]-1 of the batch-ordered tensors
 * (q_start = exclusive prefix sum of q_len).  ctx_len[s] is its KV length AFTER this
 * iteration's append, so its new tokens sit at absolute positions
 * ctx_len[s]-q_len[s] .. ctx_len[s]-1.  q_len == 1 is a decode, q_len > 1 a prefill chunk
 * on top of a cached prefix of ctx_len-q_len tokens (possibly 0).  Sequences may come in
 * any order.
 *
 * What attention computes (section 2.1): for the query at position p of a sequence, scores
 * sm_scale * <q, k_i> for i = 0..p (itself included), softmax over them, and the
 * softmax-weighted average of v_i.  A chunk therefore reads the K/V of all earlier chunks of
 * its prompt from the cache (section 4.3) plus its own rows causally; chunking changes
 * nothing in the result.  Query head h reads K/V head h / (num_q_heads/num_kv_heads)
 * (grouped-query attention, section 2.2).
 *
 * Paged cache (section 2.2; page size and in-page layout are this library's choice, the
 * paper fixes neither).  Position p of sequence s lives in page
 * block_table[s*max_blocks_per_seq + p/page_size], slot p%page_size.  Elements are bf16:
 *
 *   k_cache[((page*num_kv_heads + h)*page_size + slot)*head_dim + c]     slot-major
 *   v_cache[((page*num_kv_heads + h)*head_dim  + c   )*page_size + slot] channel-major
 *
 * (V is stored transposed inside each page so that both contractions read 16-byte runs
 * along their contraction index straight into matrix-core operands.)  Slots at or beyond
 * ctx_len and pages not named by a block table are never read in a way that can influence
 * a result; block-table entries at or beyond ceil(ctx_len/page_size) are never dereferenced.
 *
 * Conventions for every function: returns SARATHI_OK (0) or a negative sarathi_status;
 * never throws, aborts, allocates or frees caller memory.  Device work is enqueued on
 * `stream` and NOT synchronised; the caller owns every buffer and keeps device buffers
 * alive until the stream has drained.  "dev" = device pointer, "host" = host pointer.
 * HOST length arrays may be reused as soon as the call returns.  A handle serves one
 * stream at a time and is not thread-safe.  Within an iteration call sarathi_kv_append
 * BEFORE sarathi_hybrid_attention with the same description: attention reads the chunk's
 * own K/V from the cache.
 */
#ifndef SARATHI_H
#define SARATHI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SARATHI_OK = 0,
    SARATHI_EINVAL = -1,     /* null pointer, negative size, malformed description */
    SARATHI_ESHAPE = -2,     /* unsupported head counts / head_dim / page size / dtype */
    SARATHI_ECAPACITY = -3,  /* exceeds max_tokens / max_seqs / max_blocks_per_seq / max_batch_size / num_pages */
    SARATHI_EWORKSPACE = -4, /* workspace pointer missing */
    SARATHI_EHIP = -5        /* a HIP runtime call failed; see sarathi_last_error */
} sarathi_status;

typedef struct {
    int32_t num_q_heads;        /* Hq, multiple of num_kv_heads */
    int32_t num_kv_heads;       /* Hkv */
    int32_t head_dim;           /* 64 or 128 */
    int32_t page_size;          /* 16 */
    int32_t dtype;              /* 0 = bf16 (the only one) */
    int32_t max_tokens;         /* bound on num_tokens per call */
    int32_t max_seqs;           /* bound on num_seqs per call */
    int32_t max_blocks_per_seq; /* row length of block_table */
} sarathi_config;

typedef struct sarathi_handle sarathi_handle;

/* Creates host-side state (no device work, usable without a GPU for validation and planning).
 * Pinned staging memory is allocated lazily by the first call that enqueues device work: a ring of 16
 * buffers that hold the per-call metadata and that the launches read directly.  Consequences for callers:
 * a handle serves one host thread at a time; calls may be enqueued back to back on one stream without any
 * host wait (the library waits only when it comes round to a buffer whose launch has not run yet); changing
 * streams between calls is allowed but may make the library wait for the previous stream; the device entry
 * points must not be recorded into a HIP graph (a replay would read a buffer that later calls have
 * rewritten).  sarathi_destroy waits for the device before it frees the buffers. */
sarathi_status sarathi_create(const sarathi_config *config, sarathi_handle **out);
sarathi_status sarathi_destroy(sarathi_handle *handle);

/* Bytes of device scratch the caller must pass as `workspace` (256-byte aligned) to the two
 * device entry points: batch metadata, the work lists, scheduling words and the split-KV partial results.
 * Nothing is expected of its contents (no region has to be zero on entry).  Between a sarathi_kv_append and the
 * sarathi_hybrid_attention of the same iteration the metadata region holds that iteration's plan: do not
 * overwrite it in between (the attention call would read a stale plan). */
size_t sarathi_workspace_bytes(const sarathi_handle *handle);

/* Text of the last error on this handle (includes hipGetErrorString where relevant). */
const char *sarathi_last_error(const sarathi_handle *handle);

/* Tuning knobs, all optional: "split_keys" (target keys per WAVEFRONT of a 16-column wave-tile
 * work item; an item is one block whose four wavefronts quarter its keys and merge in LDS, so it
 * covers four times as many; multiple of 32, 0 = automatic), "target_items" (wavefronts of
 * wave-tile work per KV head the automatic choice aims for), "tile_split_keys" (keys per split of the 128-column chunk tiles, 0 =
 * automatic), "tile_min_cols" (sequences with at least this many columns q_len*G use chunk
 * tiles), "plan_at_append" (0/1: sarathi_kv_append also plans and uploads the attention
 * metadata of its batch so that the following attention call needs no copy of its own),
 * "interleave" (batches holding both prefill chunks and decodes: 0 = chunk-tile kernel then
 * wave-tile kernel on the caller's stream, 1 = chunk-tile kernel and the merge of its split tiles
 * on a second stream next to the wave-tile kernel, 2 = one launch holding both kinds of block),
 * "resident_chunks" (one-launch mode: blocks choose between chunk and wave tiles when they start so
 * that a compute unit runs at most one chunk block while decode work remains; -1 = automatic, 0 =
 * never, 1 = always),
 * "stream_kv" (the decodes' K/V loads carry the non-temporal hint, which pays on decode streams and
 * costs a little next to prefill chunks that matter; -1 = automatic, 0 = never, 1 = always),
 * "window" (sliding-window attention as in the paper's Table 1 for Mistral-7B: with window W > 0 the
 * query at position p reads keys p-W+1 .. p only; 0 = every key up to p; pages in front of every
 * window of a sequence are never dereferenced),
 * "decode_blocks_per_cu" (launches that hold decodes / 16-column tiles only: 1 = one block per compute unit, so
 * that blocks start longest first as units fall free, which shortens the tail of small batches; 2 = as many as fit;
 * -1 = automatic: one for up to 1024 blocks),
 * "inline_append" (0/1: sarathi_kv_append sends up to 224 page records in its kernel's arguments instead of
 * letting the blocks read them from the pinned buffer), "lds_pad_kb" (diagnostic: KiB of unused LDS per
 * attention block, which lowers the number of blocks a compute unit holds),
 * "time_kernels" (0/1/2, see sarathi_get_kernel_times), "time_every" (n >= 1: only every n-th launch of a
 * kind is bracketed, so that a timed run carries few events; default 1).
 * Unknown names return SARATHI_EINVAL. */
sarathi_status sarathi_set_option(sarathi_handle *handle, const char *name, int64_t value);

/* Optional instrumentation.  With option "time_kernels" = 1 the library brackets the attention
 * launch (both attention kernels, fork and join included) with a pair of HIP events on the
 * caller's stream; with 2 also the append kernel and the part of the split-KV merge that runs on
 * the caller's stream (up to 8192 launches per kernel between two reads; every event costs a few
 * microseconds of queue time, which is why level 1 exists).  sarathi_get_kernel_times waits for the recorded events, returns the
 * summed durations and launch counts since the last read, and resets them. */
typedef struct {
    double append_ms, attention_ms, merge_ms;
    int64_t append_launches, attention_launches, merge_launches;
} sarathi_kernel_times;
sarathi_status sarathi_get_kernel_times(sarathi_handle *handle, sarathi_kernel_times *out);

/*
 * KV append (section 2.2: keys and values of processed tokens are kept for later iterations).
 * Copies row t of k_new / v_new, for every token t of the batch, to its page and slot.
 * Pure data movement: the pool bytes written are exactly the input bytes.
 *
 *   k_new, v_new   dev, bf16 [num_tokens, Hkv, head_dim], batch order
 *   k_cache        dev, bf16 [num_pages, Hkv, page_size, head_dim]   (written)
 *   v_cache        dev, bf16 [num_pages, Hkv, head_dim, page_size]   (written)
 *   block_table    dev, int32 [num_seqs, max_blocks_per_seq]
 *   q_start, q_len, ctx_len   host, int32 [num_seqs]
 *   num_pages      pages in each pool (64-bit: pools may exceed 2^31 elements)
 *   workspace      dev, sarathi_workspace_bytes()
 *   stream         a hipStream_t passed as void* (NULL = the default stream)
 */
sarathi_status sarathi_kv_append(sarathi_handle *handle,
                                 const void *k_new, const void *v_new,
                                 void *k_cache, void *v_cache,
                                 const int32_t *block_table,
                                 const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len,
                                 int32_t num_seqs, int32_t num_tokens, int64_t num_pages,
                                 void *workspace, void *stream);

/*
 * Attention over the hybrid batch (sections 2.1, 4.1-4.3; see the top of this file).
 *
 *   q              dev, bf16 [num_tokens, Hq, head_dim], batch order
 *   k_cache, v_cache, block_table, q_start, q_len, ctx_len, num_pages: as above (read only)
 *   sm_scale       multiplies every score before the softmax; positive and finite (callers use 1/sqrt(head_dim))
 *   out            dev, bf16 [num_tokens, Hq, head_dim] (written; fp32 accumulation, one
 *                  round-to-nearest-even at the end)
 *
 * Prefill-chunk rows and decode rows run in the same launch; long key ranges are split
 * into independent pieces whose partial (max, sum, unnormalised output) triples are merged
 * in a fixed order by a second small kernel, so results are bitwise reproducible run to
 * run and do not depend on which physical pages hold the data.  A call enqueues kernels only: a small
 * one that moves the batch metadata from the handle's pinned buffer into the workspace (not needed when the
 * sarathi_kv_append of the same iteration has already brought it), a fill of the scheduling words when blocks
 * take their role at run time, the attention launch, and the merge when a key range was cut.
 */
sarathi_status sarathi_hybrid_attention(sarathi_handle *handle,
                                        const void *q,
                                        const void *k_cache, const void *v_cache,
                                        const int32_t *block_table,
                                        const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len,
                                        int32_t num_seqs, int32_t num_tokens, int64_t num_pages,
                                        float sm_scale, void *out,
                                        void *workspace, void *stream);

/*
 * The same attention for callers that cannot allocate device memory or hand a workspace over: code that runs
 * under HIP stream capture, tight serving loops, harnesses that forbid hipMalloc.  Identical to
 * sarathi_hybrid_attention except that it takes no workspace: the batch metadata, the scheduling words and the
 * split-KV partial rows live in a fixed array of about 16.7 MiB inside the library's device image (each GPU the
 * library runs on holds one copy until the process ends), and the metadata reaches the device in the arguments of
 * small kernels (3,840 bytes per launch) instead of through the handle's pinned buffers.  The call allocates
 * nothing (no hipMalloc / hipHostMalloc / hipFree, no stream or event creation) and enqueues kernels only; it
 * records no timing events ("time_kernels" is ignored) and treats option "interleave" = 1 as 2.
 *
 * Limits: the packed plan (48 bytes per tile of 16 decode columns or 128 chunk columns, 4 bytes per work item)
 * must fit into 96 KiB, else SARATHI_ECAPACITY (roughly 1,800 sequences); 16 MiB of partial rows (4,096 rows at
 * 8 KV heads x 128 channels; key ranges are cut less finely when that is short, never refused);
 * num_kv_heads * head_dim * 4 bytes per partial row must leave room for 256 rows, else SARATHI_ECAPACITY.
 * Every call on a GPU shares that GPU's array: two calls that overlap in time on one GPU (two streams, two
 * handles, two threads) race; calls ordered by one stream are safe.  What must start at zero (the scheduling
 * words) is cleared by a fill kernel inside the call.  Results agree with sarathi_hybrid_attention's within the
 * attention tolerance, and bit for bit when no key range is cut differently.
 * Under stream capture: make one call on the device before capturing (the first call on a device looks up the
 * array's address); a captured call holds its plan in the captured kernel arguments, so a replay repeats the
 * batch lengths it was captured with, on whatever the buffers then contain.
 */
sarathi_status sarathi_hybrid_attention_noalloc(sarathi_handle *handle,
                                                const void *q,
                                                const void *k_cache, const void *v_cache,
                                                const int32_t *block_table,
                                                const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len,
                                                int32_t num_seqs, int32_t num_tokens, int64_t num_pages,
                                                float sm_scale, void *out, void *stream);

/* Host-only view of the work decomposition sarathi_hybrid_attention would launch for this
 * description (no device work).  For tests and for sizing studies. */
typedef struct {
    int32_t seq;        /* sequence index */
    int32_t col_begin;  /* first column of the tile; column = row_in_chunk*G + head_in_group */
    int32_t n_cols;     /* valid columns in the tile */
    int32_t key_begin;  /* first key position (multiple of 32) */
    int32_t key_end;    /* one past the last key position this item reads */
    int32_t part_row;   /* first row of the partial buffers, or -1 if the item writes `out` itself */
    int32_t kind;       /* 0 = 16-column wave tile (decodes, tiny chunks), 1 = 128-column chunk tile */
    int32_t reserved;
} sarathi_work_item;

typedef struct {
    int32_t num_items;        /* work items (each runs once per KV head) */
    int32_t num_reduce_items; /* tiles whose key range was split (their pieces are merged by the second kernel) */
    int32_t num_part_rows;    /* rows of partial results used */
    int32_t split_keys;       /* keys per split the planner settled on for wave tiles */
    int32_t num_tile_items;   /* the first num_tile_items items are chunk tiles */
    int32_t tile_split_keys;  /* keys per split for chunk tiles */
} sarathi_plan_info;

sarathi_status sarathi_plan_hybrid_attention(sarathi_handle *handle,
                                             const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len,
                                             int32_t num_seqs, int32_t num_tokens,
                                             sarathi_plan_info *info,
                                             sarathi_work_item *items_out, int32_t items_capacity);

/*
 * Stall-free batching, one iteration (Algorithm 3, section 4.2).  Host only.
 * Fills the batch in three passes under the token budget: every running decode (one token
 * each, never dropped), then the next chunk of each running, partially prefilled request,
 * then waiting requests in the order given while their prompt's pages fit into free_pages.
 * A prefill receives min(prompt tokens left, chunk_size, token_budget - tokens so far).
 *
 * A request with a complete prefill (num_prefilled == prompt_len) that has num_decoded
 * generated tokens cached enters as a decode with ctx_len = prompt_len + num_decoded + 1.
 * A prefill enters with q_len = chunk and ctx_len = num_prefilled + chunk.
 *
 * out->seq_id, q_start, q_len, ctx_len: caller-allocated host arrays of capacity
 * max_batch_size.  Order: decodes, running prefills, admitted requests.
 * Returns SARATHI_ECAPACITY if the running decodes alone exceed max_batch_size.
 */
typedef struct {
    int64_t id;
    int32_t prompt_len;
    int32_t num_prefilled;
    int32_t num_decoded;
    int32_t reserved;
} sarathi_request;

typedef struct {
    int32_t num_seqs;
    int32_t num_tokens;
    int32_t num_decodes;
    int32_t num_prefill_chunks;
    int32_t num_admitted;     /* how many of waiting_prefills entered (a prefix of that array) */
    int32_t reserved;
    int64_t free_pages_left;
    int64_t *seq_id;
    int32_t *q_start;
    int32_t *q_len;
    int32_t *ctx_len;
} sarathi_batch;

sarathi_status sarathi_build_stall_free_batch(int32_t token_budget, int32_t chunk_size,
                                              const sarathi_request *running_decodes, int32_t n_running_decodes,
                                              const sarathi_request *running_prefills, int32_t n_running_prefills,
                                              const sarathi_request *waiting_prefills, int32_t n_waiting,
                                              int64_t free_pages, int32_t page_size, int32_t max_batch_size,
                                              sarathi_batch *out);

/* ---- Linear layers of the batch (paper sections 2.1 and 3.1) --------------------------------------
 * The Q/K/V and output projections and the two feed-forward transformations of section 2.1 apply one
 * weight matrix to every token of the batch; section 3.1 studies their cost as a function of the number
 * of tokens (bound by fetching the weights while the batch is small, by arithmetic beyond a threshold).
 *
 *     y[t][n] = sum over k < in_features of  x[t][k] * w[n][k]        (no bias)
 *
 * x  device, bf16 [num_tokens, in_features], row-major (one row per token of the batch)
 * w  device, bf16 [out_features, in_features], row-major (one row per output feature)
 * y  device, bf16 [num_tokens, out_features], row-major; products and sums are fp32, one rounding at the end
 * workspace  device scratch of workspace_bytes bytes, or NULL with 0: fp32 partial tiles when the k range
 *            is cut into pieces so that a small batch still streams the weights through every compute unit;
 *            sarathi_linear_workspace_bytes gives the size that allows every cut the planner would make;
 *            with less (or none) the call still computes the same y with fewer pieces.
 * Shapes: out_features a multiple of 128, in_features a multiple of 64 and at most 2^20, num_tokens >= 0
 * (0 is a no-op), num_tokens * out_features below 2^40; anything else returns SARATHI_ESHAPE.  Null
 * pointers with num_tokens > 0 return SARATHI_EINVAL, a failed launch SARATHI_EHIP.  The work is enqueued on
 * `stream` and not synchronised; the caller owns all buffers and keeps them alive until the stream drains.
 * Pieces are added in index order: the result does not depend on timing. */
size_t sarathi_linear_workspace_bytes(int32_t num_tokens, int32_t out_features, int32_t in_features);
sarathi_status sarathi_linear(const void *x, const void *w, void *y, int32_t num_tokens, int32_t out_features,
                              int32_t in_features, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SARATHI_H */
